"""Pins for the oracle's prefill prune (Alg. 2: score, E = L - C, evict E tokens, split into pages)."""
import numpy as np
import pytest

import oracle


def _setup(rng, lens, Hk, D, B, C, permute=True, extra=2):
    S = len(lens)
    T = sum(lens)
    k = rng.standard_normal((T, Hk, D)).astype(np.float32) * np.exp(0.5 * rng.standard_normal((T, Hk, 1))).astype(np.float32)
    v = rng.standard_normal((T, Hk, D)).astype(np.float32) * np.exp(0.5 * rng.standard_normal((T, Hk, 1))).astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    need = [(min(L, C) + B - 1) // B for L in lens]
    mb = max(need) + extra
    P = Hk * sum(need) + 3
    ids = rng.permutation(P).astype(np.int32) if permute else np.arange(P, dtype=np.int32)
    table = np.full((S, Hk, mb), -1, np.int32)
    pos = 0
    for s in range(S):
        for h in range(Hk):
            table[s, h, :need[s]] = ids[pos:pos + need[s]]
            pos += need[s]
    k_pool = np.full((P, B, D), np.float32(-777.0))
    v_pool = np.full((P, B, D), np.float32(-777.0))
    return k, v, cu, table, k_pool, v_pool


@pytest.mark.parametrize("lens,C", [([100, 37, 64, 65], 32), ([512], 256), ([5, 16, 17], 16), ([40, 200], 64)])
def test_prune_structure_and_contents(lens, C):
    rng = np.random.default_rng(10)
    Hk, D, B = 3, 64, 16
    k, v, cu, table, k_pool, v_pool = _setup(rng, lens, Hk, D, B, C)
    seq_lens, kept, tsc = oracle.prefill_prune(k, v, cu, C, k_pool, v_pool, table, want_scores=True)
    ratios = oracle.token_ratios(k, v)
    assert np.array_equal(tsc, ratios.astype(np.float32))
    for s, L in enumerate(lens):
        keep = min(L, C)
        assert seq_lens[s] == keep                                   # kept count = min(L, C)
        assert (keep + B - 1) // B == np.count_nonzero(table[s, 0] >= 0)
        for h in range(Hk):
            idx = kept[s, h]
            assert np.all(idx[keep:] == -1)
            idx = idx[:keep]
            assert np.all(np.diff(idx) > 0)                          # strictly ascending original order
            assert idx.min() >= 0 and idx.max() < L
            sc = tsc[h, cu[s]:cu[s + 1]]
            # the same selection through a library sort: lexsort by (score, index), drop the first E
            order = np.lexsort((np.arange(L), sc))
            want = np.sort(order[L - keep:])
            assert np.array_equal(idx, want)
            # separation under the total order (score, index)
            ev = np.setdiff1d(np.arange(L), idx)
            if len(ev):
                kmax = max((sc[i], i) for i in ev)
                kmin = min((sc[i], i) for i in idx)
                assert kmax < kmin
            # page contents are the kept rows, byte for byte, in order
            for i, t in enumerate(idx):
                p = table[s, h, i // B]
                assert np.array_equal(k_pool[p, i % B].view(np.int32), k[cu[s] + t, h].view(np.int32))
                assert np.array_equal(v_pool[p, i % B].view(np.int32), v[cu[s] + t, h].view(np.int32))
            # slots past the kept count were not written
            if keep % B:
                p = table[s, h, keep // B]
                assert np.all(k_pool[p, keep % B:] == np.float32(-777.0))


def test_identity_when_under_budget():
    rng = np.random.default_rng(11)
    lens, C, Hk, D, B = [33, 48], 64, 2, 64, 16
    k, v, cu, table, k_pool, v_pool = _setup(rng, lens, Hk, D, B, C)
    seq_lens, kept = oracle.prefill_prune(k, v, cu, C, k_pool, v_pool, table)
    assert list(seq_lens) == lens
    for s, L in enumerate(lens):
        for h in range(Hk):
            assert np.array_equal(kept[s, h, :L], np.arange(L))
            got = np.concatenate([k_pool[p] for p in table[s, h, :(L + B - 1) // B]])[:L]
            assert np.array_equal(got, k[cu[s]:cu[s + 1], h])


def test_all_ties_evict_lowest_indices_first():
    """V = K makes every score exactly 1: the E evicted tokens must be 0..E-1."""
    rng = np.random.default_rng(12)
    lens, C, Hk, D, B = [50, 90], 32, 2, 64, 16
    k, _, cu, table, k_pool, v_pool = _setup(rng, lens, Hk, D, B, C)
    seq_lens, kept = oracle.prefill_prune(k, k.copy(), cu, C, k_pool, v_pool, table)
    for s, L in enumerate(lens):
        for h in range(Hk):
            assert np.array_equal(kept[s, h], np.arange(L - C, L))


def test_partial_ties_at_the_threshold():
    """Dyadic one-hot scores with many duplicates at the cut: ties leave in index order."""
    L, C, B, D = 40, 16, 16, 64
    score = np.array([4, 1, 2, 2, 8, 2, 1, 2, 2, 4] * 4, dtype=np.float64)   # exact dyadics
    k = np.zeros((L, 1, D), np.float32); v = np.zeros((L, 1, D), np.float32)
    k[:, 0, 3] = 1.0
    v[:, 0, 5] = score
    cu = np.array([0, L], np.int32)
    table = np.array([[[1, 0]]], np.int32)
    k_pool = np.zeros((2, B, D), np.float32); v_pool = np.zeros((2, B, D), np.float32)
    seq_lens, kept = oracle.prefill_prune(k, v, cu, C, k_pool, v_pool, table)
    # E = 24: the eight 1s, then the sixteen 2s (all of them) -> kept = the 4s and 8s... count them:
    # 1 appears 8x, 2 appears 20x, 4 appears 8x, 8 appears 4x.  E = 24 removes 8 ones + the first 16 twos.
    twos = [i for i in range(L) if score[i] == 2]
    want = sorted(twos[16:] + [i for i in range(L) if score[i] > 2])
    assert list(kept[0, 0]) == want and seq_lens[0] == C


def test_brute_force_tiny():
    """Every subset of size C of a tiny prompt: the kept set is the one whose evicted part is the
    E smallest under (score, index) -- checked by enumerating all subsets."""
    from itertools import combinations
    rng = np.random.default_rng(13)
    L, C, B, D = 9, 4, 4, 8
    for trial in range(5):
        k = rng.integers(1, 4, size=(L, 1, D)).astype(np.float32)
        v = rng.integers(1, 4, size=(L, 1, D)).astype(np.float32)
        if trial == 0:
            v = k.copy()
        cu = np.array([0, L], np.int32)
        table = np.array([[[0]]], np.int32)
        k_pool = np.zeros((1, B, D), np.float32); v_pool = np.zeros((1, B, D), np.float32)
        _, kept, sc = oracle.prefill_prune(k, v, cu, C, k_pool, v_pool, table, want_scores=True)
        key = [(float(sc[0, i]), i) for i in range(L)]
        good = [c for c in combinations(range(L), C)
                if max(key[i] for i in range(L) if i not in c) < min(key[i] for i in c)]
        assert len(good) == 1 and list(good[0]) == list(kept[0, 0])


def test_budget_must_be_multiple_of_block():
    rng = np.random.default_rng(14)
    k, v, cu, table, k_pool, v_pool = _setup(rng, [40], 1, 64, 16, 32)
    with pytest.raises(ValueError):
        oracle.prefill_prune(k, v, cu, 24, k_pool, v_pool, table)
