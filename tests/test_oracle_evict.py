"""Pins for the oracle's decode-time eviction (Alg. 3: evict the page with the lowest score, update the
block table), incl. brute force over every candidate page on tiny inputs."""
from itertools import product

import numpy as np
import pytest

import oracle


def _read_fixture(golden_dir):
    d = {}
    with open(golden_dir + "/alg3_eviction_example.txt") as f:
        for line in f:
            if line.startswith("#") or "|" not in line:
                continue
            k, val = [x.strip() for x in line.split("|")]
            d[k] = val.split()
    return d


def test_golden_worked_example(golden_dir):
    d = _read_fixture(golden_dir)
    B, C = 4, 16
    table = np.array([[d["table_before"]]], dtype=np.int32)
    scores = np.array([[d["scores"]]], dtype=np.float32)
    lens = np.array([16], np.int32)
    ev, fr = oracle.evict_blocks(scores, table, lens, B, C)
    assert ev[0, 0] == int(d["evicted"][0]) and fr[0, 0] == int(d["freed"][0])
    assert list(table[0, 0]) == [int(x) for x in d["table_after"]]
    assert lens[0] == int(d["len_after"][0])
    # tail page not full -> nothing; under budget -> nothing
    for length, budget in ((15, 16), (16, 32)):
        t = np.array([[d["table_before"]]], dtype=np.int32)
        l2 = np.array([length], np.int32)
        ev, fr = oracle.evict_blocks(scores, t, l2, B, budget)
        assert ev[0, 0] == -1 and fr[0, 0] == -1 and l2[0] == length
        assert list(t[0, 0]) == [int(x) for x in d["table_before"]]


def _brute_force(scores_row, table_row, n):
    """All candidate deletions; the winner is the unique candidate with minimal (score, index)."""
    cands = []
    for j in range(n):
        new = list(table_row[:j]) + list(table_row[j + 1:n]) + [-1] + list(table_row[n:])
        cands.append(((float(scores_row[j]), j), new, int(table_row[j])))
    best = min(cands, key=lambda c: c[0])
    assert sum(1 for c in cands if c[0] == best[0]) == 1
    return best[0][1], best[1], best[2]


def test_brute_force_all_score_patterns():
    """Every assignment of 3 score levels to up to 6 pages (incl. all-tie and two-way ties)."""
    B = 4
    levels = [0.5, 1.0, 2.0]
    rng = np.random.default_rng(20)
    for n in range(1, 7):
        for pattern in product(range(3), repeat=n):
            mb = n + 2
            scores = np.full((1, 1, mb), np.inf, np.float32)
            scores[0, 0, :n] = [levels[i] for i in pattern]
            table = np.full((1, 1, mb), -1, np.int32)
            table[0, 0, :n] = rng.permutation(50)[:n]
            before = table[0, 0].copy()
            lens = np.array([n * B], np.int32)
            ev, fr = oracle.evict_blocks(scores, table, lens, B, n * B)
            j, new, freed = _brute_force(scores[0, 0], before, n)
            assert ev[0, 0] == j and fr[0, 0] == freed and list(table[0, 0]) == new
            assert lens[0] == (n - 1) * B


def test_matches_library_argmin_and_structure():
    rng = np.random.default_rng(21)
    S, Hk, B, mb = 5, 3, 16, 12
    n_per_seq = np.array([12, 7, 1, 9, 12])
    lens = (n_per_seq * B).astype(np.int32)
    lens[3] -= 2                                     # tail page not full -> this sequence does not trigger
    C = 7 * B                                        # sequence 2 (len 16) is under budget
    scores = rng.integers(0, 4, size=(S, Hk, mb)).astype(np.float32)   # many ties
    table = np.full((S, Hk, mb), -1, np.int32)
    ids = rng.permutation(S * Hk * mb).astype(np.int32)
    pos = 0
    for s in range(S):
        for h in range(Hk):
            table[s, h, :n_per_seq[s]] = ids[pos:pos + n_per_seq[s]]
            pos += n_per_seq[s]
    before, lens_before = table.copy(), lens.copy()
    ev, fr = oracle.evict_blocks(scores, table, lens, B, C)
    for s in range(S):
        trig = lens_before[s] % B == 0 and lens_before[s] >= C
        assert lens[s] == lens_before[s] - (B if trig else 0)
        for h in range(Hk):
            if not trig:
                assert ev[s, h] == -1 and fr[s, h] == -1
                assert np.array_equal(table[s, h], before[s, h])
                continue
            n = n_per_seq[s]
            j = int(np.argmin(scores[s, h, :n]))                      # first occurrence of the minimum
            assert ev[s, h] == j and fr[s, h] == before[s, h, j]
            old = [x for x in before[s, h] if x >= 0]
            new = [x for x in table[s, h] if x >= 0]
            assert new == old[:j] + old[j + 1:]                        # stable: a subsequence of the old row
            assert sorted(new + [int(fr[s, h])]) == sorted(old)        # nothing lost, nothing duplicated
            assert np.all(table[s, h, n - 1:] == -1)
    assert set(np.nonzero(lens != lens_before)[0]) == {0, 1, 4}


def test_ignores_scores_beyond_the_row_length():
    """Entries at j >= len/B never win, whatever they hold."""
    B = 16
    scores = np.array([[[3.0, 2.0, 5.0, -1.0, 0.0]]], np.float32)
    table = np.array([[[4, 8, 6, -1, -1]]], np.int32)
    lens = np.array([48], np.int32)
    ev, fr = oracle.evict_blocks(scores, table, lens, B, 48)
    assert ev[0, 0] == 1 and fr[0, 0] == 8 and list(table[0, 0]) == [4, 6, -1, -1, -1]


def test_one_page_per_call_and_len_zero():
    B = 16
    scores = np.zeros((1, 1, 4), np.float32)
    table = np.array([[[0, 1, 2, 3]]], np.int32)
    lens = np.array([64], np.int32)
    oracle.evict_blocks(scores, table, lens, B, 16)       # far over budget: still exactly one page
    assert lens[0] == 48 and list(table[0, 0]) == [1, 2, 3, -1]
    lens0 = np.array([0], np.int32)
    t0 = np.full((1, 1, 4), -1, np.int32)
    ev, fr = oracle.evict_blocks(scores, t0, lens0, B, 16)
    assert ev[0, 0] == -1 and lens0[0] == 0
    with pytest.raises(ValueError):
        oracle.evict_blocks(scores, table, lens, B, 24)
