"""Pins of the head-shared oracle (one table row and one decision per sequence, pages [B, Hk, D]).

It is pinned to the per-head oracle (itself pinned by the other test_oracle_* files) through two reductions that
share no code with it -- Hk = 1, where the two layouts coincide, and head slices of a shared pool handed to the
per-head functions with the head mean retyped in numpy -- and to brute force and closed forms of its own."""
import itertools

import numpy as np
import pytest

import oracle
from oracle import shared as osh


def _shared_cache(rng, lens, Hk, D, B, extra=2, pad=3):
    S = len(lens)
    nb = [(L + B - 1) // B for L in lens]
    mb = max(max(nb), 1) + extra
    P = sum(nb) + pad
    ids = rng.permutation(P).astype(np.int32)
    table = np.full((S, mb), -1, np.int32)
    pos = 0
    for s in range(S):
        table[s, :nb[s]] = ids[pos:pos + nb[s]]
        pos += nb[s]
    k = (rng.standard_normal((P, B, Hk, D)) * np.exp(0.5 * rng.standard_normal((P, B, Hk, 1)))).astype(np.float32)
    v = (rng.standard_normal((P, B, Hk, D)) * np.exp(0.5 * rng.standard_normal((P, B, Hk, 1)))).astype(np.float32)
    return k, v, table, np.array(lens, np.int32)


def _head_mean(per_head):
    """[..., Hk, n] fp32 -> [..., n] fp32: head order, fp64, one rounding (retyped here on purpose)."""
    Hk = per_head.shape[-2]
    acc = np.zeros(per_head.shape[:-2] + per_head.shape[-1:], np.float64)
    for h in range(Hk):
        acc = acc + per_head[..., h, :].astype(np.float64)
    with np.errstate(invalid="ignore"):
        return (acc / float(Hk)).astype(np.float32)


def _per_head_tables(table, Hk):
    return np.ascontiguousarray(np.repeat(table[:, None, :], Hk, axis=1))


@pytest.mark.parametrize("Hk,D,B", [(1, 64, 16), (3, 64, 16), (8, 128, 32)])
def test_scores_equal_per_head_oracle_on_head_slices(Hk, D, B):
    rng = np.random.default_rng(10 + Hk)
    lens = [5 * B, 3 * B + 7, 0, B]
    k, v, table, sl = _shared_cache(rng, lens, Hk, D, B)
    hs, ps = osh.score_blocks(k, v, table, sl)
    for h in range(Hk):
        want = oracle.score_blocks(np.ascontiguousarray(k[:, :, h]), np.ascontiguousarray(v[:, :, h]),
                                   np.ascontiguousarray(table[:, None, :]), sl)
        assert np.array_equal(hs[:, h].view(np.int32), want[:, 0].view(np.int32))
    assert np.array_equal(ps.view(np.int32), _head_mean(hs).view(np.int32))
    assert np.all(np.isinf(ps[1, 3:])) and np.all(np.isfinite(ps[1, :3]))


def test_page_score_is_the_mean_of_head_scores_not_a_pooled_ratio():
    """Two heads with ratios 1 and 3 on every token: the shared score is 2, whatever the norms' magnitudes."""
    B, D, Hk = 16, 64, 2
    k = np.zeros((1, B, Hk, D), np.float32)
    v = np.zeros_like(k)
    k[0, :, 0, 0] = 1.0; v[0, :, 0, 1] = 1.0        # head 0: ratio 1
    k[0, :, 1, 0] = 100.0; v[0, :, 1, 1] = 300.0    # head 1: ratio 3, much larger norms
    hs, ps = osh.score_blocks(k, v, np.array([[0]], np.int32), np.array([B], np.int32))
    assert hs[0, 0, 0] == 1.0 and hs[0, 1, 0] == 3.0 and ps[0, 0] == 2.0


@pytest.mark.parametrize("Hk", [1, 4])
def test_decode_equals_per_head_oracle_on_head_slices(Hk):
    rng = np.random.default_rng(20 + Hk)
    D, B, G = 64, 16, 2
    lens = [37, 0, 16, 100]
    k, v, table, sl = _shared_cache(rng, lens, Hk, D, B)
    q = rng.standard_normal((len(lens), Hk * G, D)).astype(np.float32)
    got, ws = osh.paged_decode(q, k, v, table, sl, want_weight_sums=True)
    for h in range(Hk):
        want = oracle.paged_decode(np.ascontiguousarray(q[:, h * G:(h + 1) * G]), np.ascontiguousarray(k[:, :, h]),
                                   np.ascontiguousarray(v[:, :, h]), np.ascontiguousarray(table[:, None, :]), sl)
        assert np.array_equal(got[:, h * G:(h + 1) * G], want)
    assert np.all(got[1] == 0.0)
    assert np.allclose(np.delete(ws, 1, axis=0), 1.0, atol=1e-12)


@pytest.mark.parametrize("policy,pf,pl", [(0, 0, 0), (0, 1, 2), (1, 1, 0), (1, 0, 0)])
def test_evict_equals_per_head_oracle_with_shared_decision(policy, pf, pl):
    rng = np.random.default_rng(30)
    B, Hk, mb = 16, 3, 12
    n_pages = [1, 2, 5, 9, 10, 0, 7]
    S = len(n_pages)
    lens = np.array([n * B for n in n_pages], np.int32)
    lens[6] -= 3
    C = 2 * B
    scores = (rng.integers(0, 4, size=(S, Hk, mb)) * 0.25).astype(np.float32)   # many ties after averaging
    table = np.full((S, mb), -1, np.int32)
    for s in range(S):
        n = (lens[s] + B - 1) // B
        table[s, :n] = rng.permutation(100)[:n] + 100 * s
    t_ph, l_ph = _per_head_tables(table, Hk), lens.copy()
    for call in range(3):
        ev, fr = osh.evict_blocks(scores, table, lens, B, C, policy, pf, pl)
        ev2, fr2 = oracle.evict_blocks_ex(scores, t_ph, l_ph, B, C, policy=policy, protect_first=pf,
                                          protect_last=pl, share_heads=True)
        for h in range(Hk):
            assert np.array_equal(ev, ev2[:, h]) and np.array_equal(fr, fr2[:, h])
            assert np.array_equal(table, t_ph[:, h])
        assert np.array_equal(lens, l_ph)
    assert (ev >= 0).any() and (ev < 0).any()


def test_evict_brute_force_tiny():
    """Every score pattern of 2 heads x 3 pages over 3 levels: the winner is the first minimum of the head mean."""
    B = 16
    for pat in itertools.product(range(3), repeat=6):
        sc = np.array(pat, np.float32).reshape(1, 2, 3)
        mean = [(float(sc[0, 0, j]) + float(sc[0, 1, j])) / 2.0 for j in range(3)]
        want = min(range(3), key=lambda j: (mean[j], j))
        table = np.array([[7, 8, 9]], np.int32)
        lens = np.array([3 * B], np.int32)
        ev, fr = osh.evict_blocks(sc, table, lens, B, B)
        assert ev[0] == want and fr[0] == 7 + want
        assert table[0].tolist() == [p for j, p in enumerate([7, 8, 9]) if j != want] + [-1]
        assert lens[0] == 2 * B


def test_append_places_every_head_in_the_sequence_page():
    rng = np.random.default_rng(40)
    S, Hk, D, B, mb, n_spare = 3, 4, 64, 16, 6, 3
    lens = np.array([B, 5, 2 * B], np.int32)       # 0: boundary, freed page reused; 1: mid-page; 2: boundary, spare
    P = 40
    k = np.zeros((P, B, Hk, D), np.float32); v = np.zeros_like(k)
    table = np.full((S, mb), -1, np.int32)
    table[0, 0] = 3; table[1, 0] = 4; table[2, :2] = [5, 6]
    freed = np.array([11, -1, -1], np.int32)
    spare = (20 + np.arange(S * n_spare, dtype=np.int32)).reshape(S, n_spare)
    used = np.array([0, 0, 1], np.int32)
    nk = rng.standard_normal((S, Hk, D)).astype(np.float32); nv = rng.standard_normal((S, Hk, D)).astype(np.float32)
    osh.append_kv(nk, nv, k, v, table, lens, freed, spare, used)
    assert table[0, 1] == 11 and freed[0] == -1 and used[0] == 0
    assert table[2, 2] == spare[2, 1] and used[2] == 2
    assert lens.tolist() == [B + 1, 6, 2 * B + 1]
    assert np.array_equal(k[11, 0], nk[0]) and np.array_equal(v[11, 0], nv[0])
    assert np.array_equal(k[4, 5], nk[1]) and np.array_equal(k[spare[2, 1], 0], nk[2])
    assert np.count_nonzero(k) == S * Hk * D        # nothing else was written


def _prompt(rng, lens, Hk, D):
    T = sum(lens)
    k = (rng.standard_normal((T, Hk, D)) * np.exp(0.5 * rng.standard_normal((T, Hk, 1)))).astype(np.float32)
    v = (rng.standard_normal((T, Hk, D)) * np.exp(0.5 * rng.standard_normal((T, Hk, 1)))).astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return k, v, cu


def _prune_tables(lens, C, B):
    nb = [(min(L, C) + B - 1) // B for L in lens]
    mb = max(max(nb), 1) + 1
    table = np.full((len(lens), mb), -1, np.int32)
    pos = 0
    for s, n in enumerate(nb):
        table[s, :n] = np.arange(pos, pos + n)[::-1]
        pos += n
    return table, pos


def test_prune_with_one_head_is_the_per_head_prune():
    rng = np.random.default_rng(50)
    lens, D, B, C = [300, 64, 10, 129], 64, 16, 64
    k_in, v_in, cu = _prompt(rng, lens, 1, D)
    table, P = _prune_tables(lens, C, B)
    ks = np.zeros((P, B, 1, D), np.float32); vs = np.zeros_like(ks)
    sl, kept, tsc = osh.prefill_prune(k_in, v_in, cu, C, ks, vs, table, want_scores=True)
    kp = np.zeros((P, B, D), np.float32); vp = np.zeros_like(kp)
    sl2, kept2, tsc2 = oracle.prefill_prune(k_in, v_in, cu, C, kp, vp, np.ascontiguousarray(table[:, None, :]),
                                            want_scores=True)
    assert np.array_equal(sl, sl2) and np.array_equal(kept, kept2[:, 0]) and np.array_equal(tsc, tsc2[0])
    assert np.array_equal(ks[:, :, 0], kp) and np.array_equal(vs[:, :, 0], vp)


def test_prune_selection_is_the_library_sort_of_head_mean_scores():
    rng = np.random.default_rng(51)
    lens, Hk, D, B, C = [500, 200, 33], 4, 64, 16, 128
    k_in, v_in, cu = _prompt(rng, lens, Hk, D)
    table, P = _prune_tables(lens, C, B)
    ks = np.zeros((P, B, Hk, D), np.float32); vs = np.zeros_like(ks)
    sl, kept, tsc = osh.prefill_prune(k_in, v_in, cu, C, ks, vs, table, want_scores=True)
    per_head = oracle.token_ratios(k_in, v_in).astype(np.float32)              # [Hk, T], pinned elsewhere
    assert np.array_equal(tsc.view(np.int32), _head_mean(per_head).view(np.int32))
    for s, L in enumerate(lens):
        sc = tsc[cu[s]:cu[s + 1]]
        E = max(0, L - C)
        order = np.lexsort((np.arange(L), sc))
        want = np.sort(order[E:])
        assert sl[s] == min(L, C)
        assert np.array_equal(kept[s, :len(want)], want) and np.all(kept[s, len(want):] == -1)
        for i, t in enumerate(want):
            assert np.array_equal(ks[table[s, i // B], i % B], k_in[cu[s] + t])
            assert np.array_equal(vs[table[s, i // B], i % B], v_in[cu[s] + t])


def test_prune_all_ties_and_under_budget():
    rng = np.random.default_rng(52)
    lens, Hk, D, B, C = [100, 20], 2, 64, 16, 32
    k_in, _, cu = _prompt(rng, lens, Hk, D)
    table, P = _prune_tables(lens, C, B)
    ks = np.zeros((P, B, Hk, D), np.float32); vs = np.zeros_like(ks)
    sl, kept = osh.prefill_prune(k_in, k_in.copy(), cu, C, ks, vs, table)      # V = K: every score exactly 1
    assert np.array_equal(kept[0], np.arange(100 - C, 100))                     # the E lowest indices go
    assert np.array_equal(kept[1, :20], np.arange(20)) and np.all(kept[1, 20:] == -1) and sl.tolist() == [32, 20]
    with pytest.raises(ValueError):
        osh.prefill_prune(k_in, k_in.copy(), cu, 40, ks, vs, table)             # budget not a multiple of B


def test_loop_with_a_huge_budget_is_dense_attention():
    """Nothing is ever evicted: every step must equal softmax attention over all tokens seen so far (numpy)."""
    rng = np.random.default_rng(60)
    S, Hk, G, D, B, L0, steps = 2, 2, 2, 64, 16, 20, 30
    k_in, v_in, cu = _prompt(rng, [L0] * S, Hk, D)
    mb, n_spare = 5, 4
    table = np.full((S, mb), -1, np.int32)
    table[:, :2] = [[0, 1], [2, 3]]
    P = 4 + S * n_spare
    ks = np.zeros((P, B, Hk, D), np.float32); vs = np.zeros_like(ks)
    sl, _ = osh.prefill_prune(k_in, v_in, cu, 1024, ks, vs, table)
    spare = (4 + np.arange(S * n_spare, dtype=np.int32)).reshape(S, n_spare)
    cache = osh.SharedOracleCache(ks, vs, table, sl, spare, np.zeros(S, np.int32), np.full(S, -1, np.int32), 1024)
    hist_k = [[k_in[cu[s]:cu[s + 1]]] for s in range(S)]
    hist_v = [[v_in[cu[s]:cu[s + 1]]] for s in range(S)]
    for st in range(steps):
        nk = rng.standard_normal((S, Hk, D)).astype(np.float32); nv = rng.standard_normal((S, Hk, D)).astype(np.float32)
        q = rng.standard_normal((S, Hk * G, D)).astype(np.float32)
        out, scores, ev, _ = osh.decode_step(cache, nk, nv, q)
        assert scores is None and np.all(ev == -1)
        for s in range(S):
            hist_k[s].append(nk[s][None]); hist_v[s].append(nv[s][None])
            K = np.concatenate(hist_k[s]).astype(np.float64); V = np.concatenate(hist_v[s]).astype(np.float64)
            for hq in range(Hk * G):
                logit = K[:, hq // G] @ q[s, hq].astype(np.float64) / np.sqrt(D)
                w = np.exp(logit - logit.max()); w /= w.sum()
                assert np.allclose(out[s, hq], w @ V[:, hq // G], rtol=1e-12, atol=1e-13)
    assert cache.seq_lens.tolist() == [L0 + steps] * S


def test_loop_eviction_timeline():
    """Budget 64, pages of 16: after the prune the sequence sits at 64 tokens, evicts at once, then every 16 steps."""
    rng = np.random.default_rng(61)
    S, Hk, D, B, C = 1, 2, 64, 16, 64
    k_in, v_in, cu = _prompt(rng, [200], Hk, D)
    table = np.full((S, 5), -1, np.int32); table[0, :4] = [3, 1, 2, 0]
    ks = np.zeros((6, B, Hk, D), np.float32); vs = np.zeros_like(ks)
    sl, _ = osh.prefill_prune(k_in, v_in, cu, C, ks, vs, table)
    cache = osh.SharedOracleCache(ks, vs, table, sl, np.array([[4, 5]], np.int32), np.zeros(S, np.int32),
                                  np.full(S, -1, np.int32), C)
    trig = []
    for st in range(40):
        nk = rng.standard_normal((S, Hk, D)).astype(np.float32)
        out, scores, ev, fr = osh.decode_step(cache, nk, nk, rng.standard_normal((S, Hk, D)).astype(np.float32))
        if ev[0] >= 0:
            trig.append(st)
            assert fr[0] in (0, 1, 2, 3) and scores is not None
        assert C - B + 1 <= cache.seq_lens[0] <= C
        assert sorted(p for p in cache.block_table[0] if p >= 0) == sorted(set(p for p in cache.block_table[0] if p >= 0))
    assert trig == [0, 16, 32] and cache.spare_used[0] == 0
