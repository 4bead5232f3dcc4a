"""Pins for the eviction variants (oldest-page / sliding-window policy, protected first and last pages,
one decision per sequence from head-averaged scores): brute force over the candidate set on tiny inputs,
reduction to the plain eviction, a token-id shadow model for the sliding window, library mean/argmin."""
from itertools import product

import numpy as np
import pytest

import oracle


def _table(rng, S, Hk, n_pages, mb):
    table = np.full((S, Hk, mb), -1, np.int32)
    ids = rng.permutation(S * Hk * mb).astype(np.int32)
    pos = 0
    for s in range(S):
        for h in range(Hk):
            table[s, h, :n_pages[s]] = ids[pos:pos + n_pages[s]]
            pos += n_pages[s]
    return table


def test_defaults_reduce_to_plain_eviction():
    rng = np.random.default_rng(40)
    S, Hk, B, mb = 4, 3, 16, 10
    n_pages = [10, 5, 1, 7]
    scores = rng.integers(0, 5, size=(S, Hk, mb)).astype(np.float32)
    t1 = _table(rng, S, Hk, n_pages, mb); t2 = t1.copy()
    l1 = (np.array(n_pages) * B).astype(np.int32); l2 = l1.copy()
    a = oracle.evict_blocks(scores, t1, l1, B, 5 * B)
    b = oracle.evict_blocks_ex(scores, t2, l2, B, 5 * B)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(t1, t2) and np.array_equal(l1, l2)


def test_brute_force_candidates_with_protection():
    """All score patterns on <= 6 pages x all (protect_first, protect_last): the winner is the unique
    minimum of (score, index) over the candidate range; protection yields so that one candidate remains."""
    B = 4
    levels = [0.5, 1.0, 2.0]
    for n in range(1, 7):
        for pattern in product(range(3), repeat=n):
            for pf, pl in product(range(0, 4), range(0, 4)):
                scores = np.full((1, 1, n + 1), np.inf, np.float32)
                scores[0, 0, :n] = [levels[i] for i in pattern]
                table = np.full((1, 1, n + 1), -1, np.int32)
                table[0, 0, :n] = np.arange(100, 100 + n)
                lens = np.array([n * B], np.int32)
                ev, fr = oracle.evict_blocks_ex(scores, table, lens, B, B, protect_first=pf, protect_last=pl)
                lo = min(pf, n - 1)
                hi = max(n - pl, lo + 1)
                cands = [(levels[pattern[j]], j) for j in range(lo, hi)]
                want = min(cands)[1]
                assert ev[0, 0] == want and fr[0, 0] == 100 + want
                assert list(table[0, 0, :n - 1]) == [100 + j for j in range(n) if j != want]
                assert table[0, 0, n - 1] == -1 and lens[0] == (n - 1) * B


def test_oldest_policy_is_a_sliding_window_with_sinks():
    """Shadow model on token ids: sink pages stay, the oldest other page goes, whatever the scores say."""
    rng = np.random.default_rng(41)
    B, sink, n0 = 4, 2, 6
    table = np.full((1, 2, n0 + 1), -1, np.int32)
    table[0, :, :n0] = rng.permutation(50)[:2 * n0].reshape(2, n0)
    pages = [list(table[0, h, :n0]) for h in range(2)]
    lens = np.array([n0 * B], np.int32)
    for step in range(5):
        ev, fr = oracle.evict_blocks_ex(None, table, lens, B, B, policy=oracle.POLICY_OLDEST, protect_first=sink)
        for h in range(2):
            assert ev[0, h] == sink and fr[0, h] == pages[h][sink]
            del pages[h][sink]
            new_page = 60 + 2 * step + h                      # the harness links a fresh page at the end
            pages[h].append(new_page)
            table[0, h, lens[0] // B] = new_page
            assert list(table[0, h, :n0]) == pages[h]
        lens[0] += B
    assert all(p[:sink] == list(q[:sink]) for p, q in zip(pages, [pages[0], pages[1]]))


def test_shared_heads_uses_the_mean_over_heads():
    rng = np.random.default_rng(42)
    S, Hk, B, mb = 3, 4, 16, 9
    n_pages = [9, 6, 9]
    scores = rng.random((S, Hk, mb)).astype(np.float32)
    scores[2] = 1.0                                            # all ties -> page 0 everywhere
    table = _table(rng, S, Hk, n_pages, mb)
    before = table.copy()
    lens = (np.array(n_pages) * B).astype(np.int32)
    ev, fr = oracle.evict_blocks_ex(scores, table, lens, B, 6 * B, share_heads=True)
    for s in range(S):
        n = n_pages[s]
        mean = scores[s, :, :n].astype(np.float64).mean(axis=0).astype(np.float32)   # library mean, one rounding
        j = int(np.argmin(mean))
        assert np.all(ev[s] == j)                              # every head drops the same logical page
        for h in range(Hk):
            assert fr[s, h] == before[s, h, j]
            assert list(table[s, h, :n - 1]) == [x for i, x in enumerate(before[s, h, :n]) if i != j]
    assert ev[2, 0] == 0
    # a head-local decision would differ somewhere: the two readings are distinguishable
    t2 = before.copy(); l2 = (np.array(n_pages) * B).astype(np.int32)
    ev2, _ = oracle.evict_blocks_ex(scores, t2, l2, B, 6 * B, share_heads=False)
    assert not np.array_equal(ev, ev2)


def test_argument_checks():
    table = np.zeros((1, 1, 2), np.int32); lens = np.array([32], np.int32)
    with pytest.raises(ValueError):
        oracle.evict_blocks_ex(None, table, lens, 16, 16)                       # lowest-score needs scores
    with pytest.raises(ValueError):
        oracle.evict_blocks_ex(None, table, lens, 16, 16, policy=7)
    with pytest.raises(ValueError):
        oracle.evict_blocks_ex(None, table, lens, 16, 16, policy=1, protect_first=-1)
