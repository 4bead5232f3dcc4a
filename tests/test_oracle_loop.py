"""Pins for the decode-step protocol (Alg. 3 loop with the budget gate) on the tiny configuration:
the eviction timeline in closed form, a shadow model that tracks which original tokens each row still
holds (pure integer bookkeeping) against dense attention, and the full-cache limit."""
import numpy as np
import pytest

import oracle
from oracle.decode_loop import decode_step
from paper_2509_04377_amd import synth

from _util import f32, oracle_prefill

SEED = 1234


def _dense_attention(q_row, K, V, scale):
    logit = scale * (K.astype(np.float64) @ q_row.astype(np.float64))
    p = np.exp(logit - logit.max())
    return (p[:, None] * V.astype(np.float64)).sum(0) / p.sum()


def _run(wl, budget, steps):
    lens = synth.context_lengths(wl, SEED)
    k_in, v_in, cu = synth.prompt_kv(wl, 0, lens, SEED)
    layout = synth.page_layout(wl, lens, SEED, budget=budget, steps=steps)
    cache, kept, _ = oracle_prefill(wl, lens, k_in, v_in, cu, layout, budget)
    S, Hk, Hq, B, D = wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.block_size, wl.head_dim
    G = Hq // Hk
    kin, vin, cu = f32(k_in), f32(v_in), cu.numpy()
    # shadow model: the K/V rows each (s, hk) row holds, as a list of (k_row, v_row) in cache order
    shadow = {(s, h): [(kin[cu[s] + t, h], vin[cu[s] + t, h]) for t in kept[s, h] if t >= 0]
              for s in range(S) for h in range(Hk)}
    scale = 1.0 / np.sqrt(D)
    history = []
    for step in range(steps):
        nk, nv, q = (f32(x) for x in synth.decode_inputs(wl, 0, step, SEED))
        len_before = cache.seq_lens.copy()
        out, scores, ev, fr = decode_step(cache, nk, nv, q)
        for s in range(S):
            for h in range(Hk):
                if ev[s, h] >= 0:
                    del shadow[s, h][ev[s, h] * B:(ev[s, h] + 1) * B]
                shadow[s, h].append((nk[s, h], nv[s, h]))
                assert len(shadow[s, h]) == cache.seq_lens[s]
            for hq in range(Hq):
                K = np.stack([r[0] for r in shadow[s, hq // G]])
                V = np.stack([r[1] for r in shadow[s, hq // G]])
                np.testing.assert_allclose(out[s, hq], _dense_attention(q[s, hq], K, V, scale),
                                           rtol=1e-11, atol=1e-13)
        history.append((len_before, cache.seq_lens.copy(), ev.copy(), out))
    return cache, history, (kin, vin, cu, lens)


def test_tiny_timeline_closed_form():
    """512 -> 256 tokens (16 pages); evictions exactly at steps 1 and 17 (1-based); the cached length
    at attention time runs 241..256 twice; never more than the budget; 16 pages per row."""
    wl = synth.TINY
    cache, history, _ = _run(wl, wl.budget, wl.steps)
    B, C = wl.block_size, wl.budget
    for i, (len_before, len_after, ev, _) in enumerate(history):
        step = i + 1
        want_len = C - B + 1 + (i % B)
        assert np.all(len_after == want_len)
        if step in (1, 17):
            assert np.all(ev >= 0) and np.all(len_before == C)
        else:
            assert np.all(ev == -1)
        assert np.all(len_after <= C)
    n_pages = (cache.block_table >= 0).sum(axis=2)
    assert np.all(n_pages == C // B)
    # no page is shared between rows or listed twice
    used = cache.block_table[cache.block_table >= 0]
    assert len(np.unique(used)) == len(used)


def test_budget_at_least_context_plus_steps_is_full_attention():
    """C >= L + steps: nothing is ever evicted and every step equals dense attention over all tokens."""
    wl = synth.TINY
    steps = 32
    cache, history, (kin, vin, cu, lens) = _run(wl, 1024, steps)
    S, Hk, Hq, D = wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim
    assert all(np.all(ev == -1) for _, _, ev, _ in history)
    assert np.all(cache.seq_lens == np.array(lens) + steps)
    Kall = {(s, h): [kin[cu[s] + t, h] for t in range(lens[s])] for s in range(S) for h in range(Hk)}
    Vall = {(s, h): [vin[cu[s] + t, h] for t in range(lens[s])] for s in range(S) for h in range(Hk)}
    for step, (_, _, _, out) in enumerate(history):
        nk, nv, q = (f32(x) for x in synth.decode_inputs(wl, 0, step, SEED))
        for s in range(S):
            for h in range(Hk):
                Kall[s, h].append(nk[s, h]); Vall[s, h].append(nv[s, h])
            for hq in range(Hq):
                g = hq // (Hq // Hk)
                want = _dense_attention(q[s, hq], np.stack(Kall[s, g]), np.stack(Vall[s, g]), 1 / np.sqrt(D))
                np.testing.assert_allclose(out[s, hq], want, rtol=1e-11, atol=1e-13)


def test_under_budget_prompt_grows_then_evicts():
    """L < C: the cache grows page by page from the spare list up to C, then starts evicting."""
    wl = synth.TINY.with_(context=(40,), budget=64, steps=60)
    cache, history, _ = _run(wl, wl.budget, wl.steps)
    lens_at_attention = [int(h[1][0]) for h in history]
    # 41..64, then eviction (64 -> 48) and 49..64 again, ...
    want, cur = [], 40
    for _ in range(60):
        if cur == 64:
            cur -= 16
        cur += 1
        want.append(cur)
    assert lens_at_attention == want
    first_evict = [i for i, h in enumerate(history) if np.all(h[2] >= 0)]
    assert first_evict[0] == 24 and first_evict == [24, 40, 56]


def test_append_consumes_the_freed_page_once():
    """A row at a page boundary takes the page it has just freed and forgets it: B tokens later, with no
    eviction in between, the next page comes from the spare list.  Rows elsewhere in a page touch no
    bookkeeping, and every new K/V row lands in (tail page, slot len % B)."""
    rng = np.random.default_rng(70)
    S, Hk, D, B, mb, n_spare = 2, 2, 64, 16, 5, 2
    k = np.zeros((40, B, D), np.float32); v = np.zeros_like(k)
    table = np.full((S, Hk, mb), -1, np.int32)
    table[0, :, 0] = [3, 4]                          # sequence 0: one full page per row -> boundary
    table[1, :, 0] = [5, 6]                          # sequence 1: 5 tokens -> mid-page
    lens = np.array([B, 5], np.int32)
    freed = np.array([[11, -1], [-1, -1]], np.int32)   # only row (0, 0) holds a freed page
    spare = (20 + np.arange(S * Hk * n_spare, dtype=np.int32)).reshape(S, Hk, n_spare)
    used = np.zeros((S, Hk), np.int32)
    for step in range(B + 1):
        nk = rng.standard_normal((S, Hk, D)).astype(np.float32); nv = rng.standard_normal((S, Hk, D)).astype(np.float32)
        before = lens.copy()
        oracle.append_kv(nk, nv, k, v, table, lens, freed, spare, used)
        for s in range(S):
            for h in range(Hk):
                page = table[s, h, before[s] // B]
                assert np.array_equal(k[page, before[s] % B], nk[s, h]) and np.array_equal(v[page, before[s] % B], nv[s, h])
        if step == 0:
            assert table[0, 0, 1] == 11 and table[0, 1, 1] == spare[0, 1, 0]
            assert freed[0, 0] == -1 and used.tolist() == [[0, 1], [0, 0]]
    # step B was sequence 0's next boundary: both rows took a spare page, the freed one was not reused
    assert table[0, 0, 2] == spare[0, 0, 0] and table[0, 1, 2] == spare[0, 1, 1]
    assert used[0].tolist() == [1, 2] and np.all(freed == -1)
    assert lens.tolist() == [2 * B + 1, 5 + B + 1] and table[1, 0, 1] == spare[1, 0, 0]


def test_budget_of_one_page_restarts_from_the_new_token():
    """C = B: each eviction drops the row's only page, so right after it the cache holds the new token alone
    and its attention output is that token's V row; the shadow model checks every other step."""
    wl = synth.TINY.with_(context=(40,), budget=16)
    cache, history, _ = _run(wl, 16, 35)
    trig = [i for i, (_, _, ev, _) in enumerate(history) if (ev >= 0).any()]
    assert trig == [0, 16, 32]
    for i in trig:
        len_before, len_after, ev, out = history[i]
        assert len_before[0] == 16 and len_after[0] == 1 and np.all(ev == 0)
        nk, nv, q = (f32(x) for x in synth.decode_inputs(wl, 0, i, SEED))
        G = wl.num_q_heads // wl.num_kv_heads
        for hq in range(wl.num_q_heads):
            np.testing.assert_allclose(out[0, hq], nv[0, hq // G].astype(np.float64), rtol=1e-12)
    assert np.all(cache.spare_used == 0)        # the freed page is reused every time
