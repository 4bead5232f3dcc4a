"""Pins for the oracle's paged decode attention (Eq. 1; Alg. 3 "PagedAttention(Q,K,V)")."""
import numpy as np
import pytest
import torch

import oracle


def _paged(rng, lens, Hk, D, B, extra=1):
    """Random K/V for each row, laid out in shuffled pages.  Returns dense copies as well."""
    S = len(lens)
    nb = [(L + B - 1) // B for L in lens]
    mb = max(max(nb), 1) + extra
    P = Hk * sum(nb) + 2
    ids = rng.permutation(P).astype(np.int32)
    table = np.full((S, Hk, mb), -1, np.int32)
    k_pool = rng.standard_normal((P, B, D)).astype(np.float32)    # unused slots hold junk on purpose
    v_pool = rng.standard_normal((P, B, D)).astype(np.float32)
    dense_k, dense_v = {}, {}
    pos = 0
    for s in range(S):
        for h in range(Hk):
            table[s, h, :nb[s]] = ids[pos:pos + nb[s]]
            pos += nb[s]
            kk = rng.standard_normal((lens[s], D)).astype(np.float32) * 1.5
            vv = rng.standard_normal((lens[s], D)).astype(np.float32)
            for t in range(lens[s]):
                k_pool[table[s, h, t // B], t % B] = kk[t]
                v_pool[table[s, h, t // B], t % B] = vv[t]
            dense_k[s, h], dense_v[s, h] = kk, vv
    return k_pool, v_pool, table, np.array(lens, np.int32), dense_k, dense_v


@pytest.mark.parametrize("Hk,Hq,D,B", [(2, 4, 64, 16), (2, 6, 128, 16), (1, 4, 64, 32), (3, 3, 128, 32)])
def test_full_cache_equals_textbook_sdpa(Hk, Hq, D, B):
    """With nothing evicted the path is softmax(q K^T / sqrt(D)) V: compare with torch's fp64 SDPA."""
    rng = np.random.default_rng(30)
    lens = [1, 15, 16, 17, 100]
    k_pool, v_pool, table, sl, dk, dv = _paged(rng, lens, Hk, D, B)
    q = rng.standard_normal((len(lens), Hq, D)).astype(np.float32)
    out, ws = oracle.paged_decode(q, k_pool, v_pool, table, sl, want_weight_sums=True)
    G = Hq // Hk
    for s, L in enumerate(lens):
        K = torch.tensor(np.stack([dk[s, h] for h in range(Hk)]), dtype=torch.float64)    # [Hk, L, D]
        V = torch.tensor(np.stack([dv[s, h] for h in range(Hk)]), dtype=torch.float64)
        K = K.repeat_interleave(G, dim=0)                                                   # q head h -> kv head h // G
        V = V.repeat_interleave(G, dim=0)
        Q = torch.tensor(q[s], dtype=torch.float64).unsqueeze(1)                            # [Hq, 1, D]
        want = torch.nn.functional.scaled_dot_product_attention(Q, K, V).squeeze(1).numpy()
        np.testing.assert_allclose(out[s], want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ws, 1.0, rtol=0, atol=1e-12)        # softmax weights sum to 1


def test_numpy_definition_with_explicit_scale_and_group_map():
    rng = np.random.default_rng(31)
    Hk, Hq, D, B = 2, 8, 64, 16
    lens = [37]
    k_pool, v_pool, table, sl, dk, dv = _paged(rng, lens, Hk, D, B)
    q = rng.standard_normal((1, Hq, D)).astype(np.float32)
    scale = 0.3
    out = oracle.paged_decode(q, k_pool, v_pool, table, sl, scale=scale)
    for hq in range(Hq):
        g = hq // (Hq // Hk)
        logit = scale * dk[0, g].astype(np.float64) @ q[0, hq].astype(np.float64)
        p = np.exp(logit - logit.max())
        want = (p[:, None] * dv[0, g].astype(np.float64)).sum(0) / p.sum()
        np.testing.assert_allclose(out[0, hq], want, rtol=1e-12, atol=1e-14)


def test_special_cases():
    rng = np.random.default_rng(32)
    Hk, Hq, D, B = 1, 2, 64, 16
    # all V rows equal -> out = that row, whatever the weights
    k_pool, v_pool, table, sl, _, _ = _paged(rng, [40], Hk, D, B)
    vrow = rng.standard_normal(D).astype(np.float32)
    v_pool[:] = vrow
    q = rng.standard_normal((1, Hq, D)).astype(np.float32)
    out = oracle.paged_decode(q, k_pool, v_pool, table, sl)
    np.testing.assert_allclose(out[0], np.broadcast_to(vrow.astype(np.float64), (Hq, D)), rtol=1e-13)
    # one dominant logit -> out -> that token's V
    k_pool, v_pool, table, sl, dk, dv = _paged(rng, [40], Hk, D, B)
    t = 23
    q = np.stack([dk[0, 0][t] * 100.0] * Hq)[None].astype(np.float32)
    out = oracle.paged_decode(q, k_pool, v_pool, table, sl)
    np.testing.assert_allclose(out[0, 0], dv[0, 0][t].astype(np.float64), rtol=1e-9, atol=1e-9)
    # len = 1 -> out = v_0 ; len = 0 -> zeros
    k_pool, v_pool, table, sl, dk, dv = _paged(rng, [1, 0], Hk, D, B)
    q = rng.standard_normal((2, Hq, D)).astype(np.float32)
    out, ws = oracle.paged_decode(q, k_pool, v_pool, table, sl, want_weight_sums=True)
    np.testing.assert_array_equal(out[0, 1], dv[0, 0][0].astype(np.float64))
    assert np.all(out[1] == 0.0) and np.all(ws[1] == 0.0) and np.all(ws[0] == 1.0)


def test_zero_query_gives_the_mean_of_v():
    """q = 0 makes every weight 1/len: out is the plain mean (a closed form that needs no softmax)."""
    rng = np.random.default_rng(33)
    Hk, Hq, D, B = 2, 4, 64, 16
    k_pool, v_pool, table, sl, dk, dv = _paged(rng, [50], Hk, D, B)
    out = oracle.paged_decode(np.zeros((1, Hq, D), np.float32), k_pool, v_pool, table, sl)
    for hq in range(Hq):
        np.testing.assert_allclose(out[0, hq], dv[0, hq // 2].astype(np.float64).mean(0), rtol=1e-13, atol=1e-15)


def test_logical_page_order_is_irrelevant_up_to_roundoff():
    rng = np.random.default_rng(34)
    Hk, Hq, D, B = 1, 4, 64, 16
    k_pool, v_pool, table, sl, _, _ = _paged(rng, [96], Hk, D, B, extra=0)
    q = rng.standard_normal((1, Hq, D)).astype(np.float32)
    base = oracle.paged_decode(q, k_pool, v_pool, table, sl)
    t2 = table.copy()
    t2[0, 0] = table[0, 0][rng.permutation(6)]
    np.testing.assert_allclose(oracle.paged_decode(q, k_pool, v_pool, t2, sl), base, rtol=1e-12, atol=1e-14)


def test_masks_the_tail_of_a_partial_page():
    """Slots past len in the tail page (junk, even inf/nan) must not leak in."""
    rng = np.random.default_rng(35)
    Hk, Hq, D, B = 1, 2, 64, 16
    k_pool, v_pool, table, sl, dk, dv = _paged(rng, [21], Hk, D, B)
    q = rng.standard_normal((1, Hq, D)).astype(np.float32)
    base = oracle.paged_decode(q, k_pool, v_pool, table, sl)
    tail = table[0, 0, 1]
    k_pool[tail, 5:] = np.nan
    v_pool[tail, 5:] = np.inf
    assert np.array_equal(oracle.paged_decode(q, k_pool, v_pool, table, sl), base)
