"""Pins for the oracle's importance scores (Alg. 1; Alg. 3 "Compute Score of Page i").

Each test checks the C oracle against something fixed by the paper or the mathematics, not against
itself: hand-derived exact rationals, closed forms on dyadic inputs, invariances, and the library
2-norm.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _read_pythagorean(golden_dir):
    rows, blocks = [], {}
    with open(golden_dir + "/alg1_pythagorean.txt") as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split("|")]
            if parts[0].startswith("block"):
                blocks[int(parts[0].split()[1])] = Fraction(parts[1])
            else:
                rows.append((np.array(parts[0].split(), dtype=np.float32),
                             np.array(parts[1].split(), dtype=np.float32), Fraction(parts[2])))
    return rows, blocks


def test_golden_pythagorean_token_ratios(golden_dir):
    rows, _ = _read_pythagorean(golden_dir)
    assert len(rows) == 8
    for k, v, want in rows:
        got = oracle.token_ratio(k, v)
        # integer norms: sqrt and the quotient are correctly rounded, so the fp64 result is the
        # fp64 nearest to the exact rational.
        assert got == float(want), (k, v, got, want)


def test_golden_pythagorean_block_means(golden_dir):
    rows, blocks = _read_pythagorean(golden_dir)
    B, D = 4, 4
    k_pool = np.zeros((3, B, D), np.float32)
    v_pool = np.zeros((3, B, D), np.float32)
    # logical block 0 -> physical 2, logical block 1 -> physical 0 (physical 1 unused)
    phys = [2, 0]
    for i, (k, v, _) in enumerate(rows):
        k_pool[phys[i // B], i % B] = k
        v_pool[phys[i // B], i % B] = v
    table = np.array([[[2, 0, -1]]], np.int32)
    sc = oracle.score_blocks(k_pool, v_pool, table, np.array([8], np.int32))
    for j in (0, 1):
        want = np.float32(float(blocks[j]))
        assert abs(float(sc[0, 0, j]) - float(want)) <= np.spacing(want), (j, sc[0, 0, j], want)
    assert np.isinf(sc[0, 0, 2]) and sc[0, 0, 2] > 0


def test_closed_form_one_hot_dyadic():
    """K_i = k_i e_a, V_i = v_i e_b with powers of two: r_i = v_i/k_i exactly, block mean exact."""
    rng = np.random.default_rng(1)
    S, Hk, D, B, nb = 2, 3, 64, 16, 5
    P = S * Hk * nb
    k_pool = np.zeros((P, B, D), np.float32)
    v_pool = np.zeros((P, B, D), np.float32)
    ek = rng.integers(-3, 4, size=(P, B))
    ev = rng.integers(-3, 4, size=(P, B))
    for p in range(P):
        for i in range(B):
            k_pool[p, i, rng.integers(D)] = -(2.0 ** ek[p, i]) if rng.random() < 0.5 else 2.0 ** ek[p, i]
            v_pool[p, i, rng.integers(D)] = 2.0 ** ev[p, i]
    table = rng.permutation(P).astype(np.int32).reshape(S, Hk, nb)
    lens = np.array([nb * B, nb * B - 3], np.int32)
    sc = oracle.score_blocks(k_pool, v_pool, table, lens)
    ratio = 2.0 ** (ev - ek).astype(np.float64)           # exact
    for s in range(S):
        for h in range(Hk):
            for j in range(nb):
                if j < lens[s] // B:
                    want = ratio[table[s, h, j]].sum() / B  # dyadic sum of <= 16 terms: exact in fp64
                    assert sc[s, h, j] == np.float32(want)
                else:
                    assert sc[s, h, j] == np.inf


def test_mean_of_ratios_not_ratio_of_page_norms():
    """The two readings of "score of page i" differ; the oracle takes Alg. 1's mean of ratios."""
    B, D = 16, 64
    k = np.zeros((1, B, D), np.float32)
    v = np.zeros((1, B, D), np.float32)
    k[0, :, 0] = 1.0
    v[0, :, 0] = 1.0
    k[0, 0, 0] = 8.0   # token 0: ratio 1/8 ; the other 15: ratio 1
    sc = oracle.score_blocks(k, v, np.array([[[0]]], np.int32), np.array([B], np.int32))
    assert sc[0, 0, 0] == np.float32((15 + 0.125) / 16)
    frob = np.sqrt((v.astype(np.float64) ** 2).sum()) / np.sqrt((k.astype(np.float64) ** 2).sum())
    assert abs(float(sc[0, 0, 0]) - frob) > 0.3


def test_v_equals_k_gives_exactly_one():
    rng = np.random.default_rng(2)
    k = rng.standard_normal((7, 16, 128)).astype(np.float32)
    table = np.arange(6, dtype=np.int32).reshape(1, 2, 3)
    sc = oracle.score_blocks(k, k.copy(), table, np.array([48], np.int32))
    assert np.all(sc == np.float32(1.0))
    r = oracle.token_ratios(k.reshape(-1, 1, 128), k.reshape(-1, 1, 128))
    assert np.all(r == 1.0)


def test_scale_invariance_power_of_two():
    """Scaling a token's K and V rows by the same power of two changes nothing, bit for bit."""
    rng = np.random.default_rng(3)
    P, B, D = 6, 16, 64
    k = rng.standard_normal((P, B, D)).astype(np.float32)
    v = rng.standard_normal((P, B, D)).astype(np.float32)
    table = np.arange(P, dtype=np.int32).reshape(1, 1, P)
    lens = np.array([P * B], np.int32)
    base = oracle.score_blocks(k, v, table, lens)
    f = (2.0 ** rng.integers(-8, 9, size=(P, B, 1))).astype(np.float32)
    scaled = oracle.score_blocks(k * f, v * f, table, lens)
    assert np.array_equal(base.view(np.int32), scaled.view(np.int32))


def test_ratio_direction_and_scaling_laws():
    """||V|| is the numerator and ||K|| the denominator: doubling V doubles r, doubling K halves it."""
    rng = np.random.default_rng(4)
    k = rng.standard_normal(128).astype(np.float32)
    v = rng.standard_normal(128).astype(np.float32)
    r = oracle.token_ratio(k, v)
    assert oracle.token_ratio(k, 2 * v) == 2 * r
    assert oracle.token_ratio(2 * k, v) == r / 2
    assert oracle.token_ratio(v, k) == pytest.approx(1.0 / r, rel=1e-15)


def test_against_library_norm():
    rng = np.random.default_rng(5)
    T, Hk, D = 257, 3, 128
    k = (rng.standard_normal((T, Hk, D)) * np.exp(0.5 * rng.standard_normal((T, Hk, 1)))).astype(np.float32)
    v = (rng.standard_normal((T, Hk, D)) * np.exp(0.5 * rng.standard_normal((T, Hk, 1)))).astype(np.float32)
    got = oracle.token_ratios(k, v)                              # [Hk, T]
    want = (np.linalg.norm(v.astype(np.float64), axis=-1) / np.linalg.norm(k.astype(np.float64), axis=-1)).T
    assert got.shape == (Hk, T)
    np.testing.assert_allclose(got, want, rtol=1e-14, atol=0)


def test_every_element_counts():
    """A change in any single coordinate of K or V moves the score (no dropped term, no wrong stride)."""
    D = 64
    k = np.ones(D, np.float32)
    v = np.ones(D, np.float32)
    base = oracle.token_ratio(k, v)
    for d in range(D):
        k2 = k.copy(); k2[d] = 3.0
        v2 = v.copy(); v2[d] = 3.0
        assert oracle.token_ratio(k2, v) == pytest.approx(np.sqrt(D / (D + 8.0)), rel=1e-15)
        assert oracle.token_ratio(k, v2) == pytest.approx(np.sqrt((D + 8.0) / D), rel=1e-15)
        assert oracle.token_ratio(k2, v2) == base


def test_zero_norm_conventions():
    z = np.zeros(64, np.float32)
    x = np.ones(64, np.float32)
    assert oracle.token_ratio(x, z) == 0.0      # ||V|| = 0
    assert oracle.token_ratio(z, z) == 0.0      # 0/0 := 0
    assert oracle.token_ratio(z, x) == np.inf   # ||K|| = 0
    B, D = 16, 64
    k = np.ones((2, B, D), np.float32)
    v = np.ones((2, B, D), np.float32)
    k[1, 5] = 0.0                                # one +inf token makes its page +inf
    sc = oracle.score_blocks(k, v, np.array([[[0, 1]]], np.int32), np.array([32], np.int32))
    assert sc[0, 0, 0] == 1.0 and sc[0, 0, 1] == np.inf


def test_physical_permutation_invariance():
    rng = np.random.default_rng(6)
    S, Hk, nb, B, D = 2, 2, 4, 16, 64
    P = S * Hk * nb
    k = rng.standard_normal((P, B, D)).astype(np.float32)
    v = rng.standard_normal((P, B, D)).astype(np.float32)
    table = np.arange(P, dtype=np.int32).reshape(S, Hk, nb)
    lens = np.array([nb * B, (nb - 1) * B + 5], np.int32)
    table[1, :, nb - 1] = table[1, :, nb - 1]      # partial tail page still allocated
    base = oracle.score_blocks(k, v, table, lens)
    perm = rng.permutation(P)                       # new physical id of old page p is perm[p]
    k2 = np.empty_like(k); v2 = np.empty_like(v)
    k2[perm] = k; v2[perm] = v
    table2 = perm[table].astype(np.int32)
    assert np.array_equal(base.view(np.int32), oracle.score_blocks(k2, v2, table2, lens).view(np.int32))


def test_partial_and_unused_entries_are_inf():
    rng = np.random.default_rng(7)
    B, D = 16, 64
    k = rng.standard_normal((4, B, D)).astype(np.float32)
    v = rng.standard_normal((4, B, D)).astype(np.float32)
    table = np.array([[[0, 1, 2, -1, -1]]], np.int32)
    for length, nfull in ((0, 0), (1, 0), (16, 1), (17, 1), (47, 2), (48, 3)):
        t = table.copy()
        t[0, 0, (length + B - 1) // B:] = -1
        sc = oracle.score_blocks(k, v, t, np.array([length], np.int32))
        assert np.all(np.isfinite(sc[0, 0, :nfull]))
        assert np.all(sc[0, 0, nfull:] == np.inf)
