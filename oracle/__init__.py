"""CPU oracle for the PagedEviction hot path -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``pe_oracle.c`` (plain C, fp64) plus the decode-step
protocol written as a plain Python loop (``decode_loop.py``).  Only the tests, the smoke
check and the benchmark's CPU-baseline leg may import this package; the product path never
does and shares nothing with it.

All tensors are numpy arrays on the host.  K/V/q data are float32 arrays (a bf16 value is
handed over after its exact conversion to float32); tables and lengths are int32.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)


def _load():
    global _lib
    if _lib is None:
        # PE_ORACLE_LIB: tests/test_oracle_mutants.py points its child processes at a deliberately broken
        # build of the oracle to check that the pins notice.  It is honoured only together with the marker
        # that test sets (PE_ORACLE_MUTANT_RUN=1) and never in a process that has a GPU test selected
        # (tests/conftest.py refuses to start a GPU run with it); set alone it is an error, not a silent swap.
        path = os.environ.get("PE_ORACLE_LIB")
        if path:
            if os.environ.get("PE_ORACLE_MUTANT_RUN") != "1":
                raise RuntimeError("PE_ORACLE_LIB is set outside the oracle mutation test: refusing to load a "
                                   "substitute oracle (%s)" % path)
        else:
            path = _build.build(force=False, sanitize=os.environ.get("PE_ORACLE_SANITIZE") == "1")
        lib = ctypes.CDLL(path)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_token_ratio.restype = ctypes.c_double
        lib.oracle_token_ratio.argtypes = [_f32p, _f32p, ctypes.c_int]
        lib.oracle_token_ratios.restype = None
        lib.oracle_token_ratios.argtypes = [_f32p, _f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, _f64p]
        lib.oracle_score_blocks.restype = None
        lib.oracle_score_blocks.argtypes = [_f32p, _f32p, _i32p, _i32p] + [ctypes.c_int] * 5 + [_f32p]
        lib.oracle_prefill_prune.restype = ctypes.c_int
        lib.oracle_prefill_prune.argtypes = ([_f32p, _f32p, _i32p] + [ctypes.c_int] * 6 +
                                             [_f32p, _f32p, _i32p, _i32p, _i32p, _f32p])
        lib.oracle_evict_blocks.restype = ctypes.c_int
        lib.oracle_evict_blocks.argtypes = [_f32p, _i32p, _i32p] + [ctypes.c_int] * 5 + [_i32p, _i32p]
        lib.oracle_evict_blocks_ex.restype = ctypes.c_int
        lib.oracle_evict_blocks_ex.argtypes = [_f32p, _i32p, _i32p] + [ctypes.c_int] * 9 + [_i32p, _i32p]
        lib.oracle_append_kv.restype = ctypes.c_int
        lib.oracle_append_kv.argtypes = ([_f32p, _f32p, _f32p, _f32p, _i32p, _i32p, _i32p, _i32p, _i32p] +
                                         [ctypes.c_int] * 6)
        lib.oracle_paged_decode.restype = None
        lib.oracle_paged_decode.argtypes = ([_f32p, _f32p, _f32p, _i32p, _i32p] + [ctypes.c_int] * 6 +
                                            [ctypes.c_double, _f64p, _f64p])
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle expects float32 data, got %s" % a.dtype)
    return a


def _i32(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.int32:
        raise TypeError("oracle expects int32 tables, got %s" % a.dtype)
    return a


def _p(a, t):
    return a.ctypes.data_as(t)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def token_ratio(k_row, v_row) -> float:
    """||v||/||k|| of one token (fp64)."""
    k_row, v_row = _f32(k_row), _f32(v_row)
    assert k_row.ndim == 1 and k_row.shape == v_row.shape
    return float(_load().oracle_token_ratio(_p(k_row, _f32p), _p(v_row, _f32p), k_row.shape[0]))


def token_ratios(k_in, v_in):
    """k_in, v_in [T, Hk, D] -> fp64 ratios [Hk, T]."""
    k_in, v_in = _f32(k_in), _f32(v_in)
    T, Hk, D = k_in.shape
    out = np.empty((Hk, T), dtype=np.float64)
    _load().oracle_token_ratios(_p(k_in, _f32p), _p(v_in, _f32p), T, Hk, D, _p(out, _f64p))
    return out


def score_blocks(k_pool, v_pool, block_table, seq_lens):
    """Pools [P, B, D], table [S, Hk, max_blocks], lens [S] -> fp32 scores [S, Hk, max_blocks]."""
    k_pool, v_pool = _f32(k_pool), _f32(v_pool)
    block_table, seq_lens = _i32(block_table), _i32(seq_lens)
    P, B, D = k_pool.shape
    S, Hk, mb = block_table.shape
    assert v_pool.shape == k_pool.shape and seq_lens.shape == (S,)
    _check_table(block_table, seq_lens, B, P)
    out = np.empty((S, Hk, mb), dtype=np.float32)
    _load().oracle_score_blocks(_p(k_pool, _f32p), _p(v_pool, _f32p), _p(block_table, _i32p),
                                _p(seq_lens, _i32p), S, Hk, D, B, mb, _p(out, _f32p))
    return out


def prefill_prune(k_in, v_in, cu_seqlens, budget, k_pool, v_pool, block_table, want_scores=False):
    """Prune a packed prompt into the paged pools (modified in place).

    Returns (seq_lens [S], kept_idx [S, Hk, budget]) and, if asked, the fp32 token scores [Hk, T]."""
    k_in, v_in = _f32(k_in), _f32(v_in)
    cu_seqlens, block_table = _i32(cu_seqlens), _i32(block_table)
    T, Hk, D = k_in.shape
    P, B, D2 = k_pool.shape
    S, Hk2, mb = block_table.shape
    assert D == D2 and Hk == Hk2 and cu_seqlens.shape == (S + 1,) and int(cu_seqlens[-1]) == T
    assert k_pool.dtype == np.float32 and k_pool.flags.c_contiguous
    assert v_pool.dtype == np.float32 and v_pool.flags.c_contiguous
    lens = np.minimum(np.diff(cu_seqlens), budget).astype(np.int32)
    _check_table(block_table, lens, B, P)
    seq_lens = np.zeros((S,), dtype=np.int32)
    kept = np.empty((S, Hk, budget), dtype=np.int32)
    tsc = np.empty((Hk, T), dtype=np.float32) if want_scores else None
    rc = _load().oracle_prefill_prune(_p(k_in, _f32p), _p(v_in, _f32p), _p(cu_seqlens, _i32p), S, Hk, D, B,
                                      int(budget), mb, _p(k_pool, _f32p), _p(v_pool, _f32p),
                                      _p(block_table, _i32p), _p(seq_lens, _i32p), _p(kept, _i32p),
                                      _p(tsc, _f32p) if want_scores else None)
    if rc != 0:
        raise ValueError("oracle_prefill_prune failed with status %d" % rc)
    return (seq_lens, kept, tsc) if want_scores else (seq_lens, kept)


def evict_blocks(scores, block_table, seq_lens, block_size, budget):
    """In place on block_table / seq_lens.  Returns (evicted_logical, freed_phys), both [S, Hk]."""
    scores = _f32(scores)
    S, Hk, mb = block_table.shape
    assert block_table.dtype == np.int32 and block_table.flags.c_contiguous
    assert seq_lens.dtype == np.int32 and seq_lens.flags.c_contiguous
    assert scores.shape == (S, Hk, mb)
    ev = np.empty((S, Hk), dtype=np.int32)
    fr = np.empty((S, Hk), dtype=np.int32)
    rc = _load().oracle_evict_blocks(_p(scores, _f32p), _p(block_table, _i32p), _p(seq_lens, _i32p), S, Hk,
                                     int(block_size), mb, int(budget), _p(ev, _i32p), _p(fr, _i32p))
    if rc != 0:
        raise ValueError("oracle_evict_blocks failed with status %d" % rc)
    return ev, fr


POLICY_LOWEST_SCORE, POLICY_OLDEST = 0, 1


def evict_blocks_ex(scores, block_table, seq_lens, block_size, budget, policy=POLICY_LOWEST_SCORE, protect_first=0,
                    protect_last=0, share_heads=False):
    """Eviction with a policy, protected pages and optionally one decision per sequence.  In place on
    block_table / seq_lens.  `scores` may be None for POLICY_OLDEST.  Returns (evicted_logical, freed_phys)."""
    S, Hk, mb = block_table.shape
    assert block_table.dtype == np.int32 and block_table.flags.c_contiguous
    assert seq_lens.dtype == np.int32 and seq_lens.flags.c_contiguous
    if scores is not None:
        scores = _f32(scores)
        assert scores.shape == (S, Hk, mb)
    ev = np.empty((S, Hk), dtype=np.int32)
    fr = np.empty((S, Hk), dtype=np.int32)
    rc = _load().oracle_evict_blocks_ex(_p(scores, _f32p) if scores is not None else None, _p(block_table, _i32p),
                                        _p(seq_lens, _i32p), S, Hk, int(block_size), mb, int(budget), int(policy),
                                        int(protect_first), int(protect_last), int(bool(share_heads)), _p(ev, _i32p),
                                        _p(fr, _i32p))
    if rc != 0:
        raise ValueError("oracle_evict_blocks_ex failed with status %d" % rc)
    return ev, fr


def append_kv(new_k, new_v, k_pool, v_pool, block_table, seq_lens, freed_phys, spare, spare_used):
    """In place on pools, table, lens, freed_phys, spare_used."""
    new_k, new_v = _f32(new_k), _f32(new_v)
    S, Hk, D = new_k.shape
    P, B, _ = k_pool.shape
    mb = block_table.shape[2]
    n_spare = spare.shape[2]
    for a in (block_table, seq_lens, freed_phys, spare, spare_used):
        assert a.dtype == np.int32 and a.flags.c_contiguous
    rc = _load().oracle_append_kv(_p(new_k, _f32p), _p(new_v, _f32p), _p(k_pool, _f32p), _p(v_pool, _f32p),
                                  _p(block_table, _i32p), _p(seq_lens, _i32p), _p(freed_phys, _i32p),
                                  _p(spare, _i32p), _p(spare_used, _i32p), n_spare, S, Hk, D, B, mb)
    if rc != 0:
        raise ValueError("oracle_append_kv failed with status %d" % rc)


def paged_decode(q, k_pool, v_pool, block_table, seq_lens, scale=None, want_weight_sums=False):
    """q [S, Hq, D] -> fp64 out [S, Hq, D] (and the per-(s, hq) sums of softmax weights)."""
    q, k_pool, v_pool = _f32(q), _f32(k_pool), _f32(v_pool)
    block_table, seq_lens = _i32(block_table), _i32(seq_lens)
    S, Hq, D = q.shape
    P, B, _ = k_pool.shape
    _, Hk, mb = block_table.shape
    assert Hq % Hk == 0
    _check_table(block_table, seq_lens, B, P)
    if scale is None:
        scale = 1.0 / np.sqrt(float(D))
    out = np.empty((S, Hq, D), dtype=np.float64)
    ws = np.empty((S, Hq), dtype=np.float64)
    _load().oracle_paged_decode(_p(q, _f32p), _p(k_pool, _f32p), _p(v_pool, _f32p), _p(block_table, _i32p),
                                _p(seq_lens, _i32p), S, Hk, Hq, D, B, mb, float(scale), _p(out, _f64p),
                                _p(ws, _f64p))
    return (out, ws) if want_weight_sums else out


def _check_table(block_table, seq_lens, B, P):
    """Host-side bounds check so the C loops never index outside the pools."""
    S, Hk, mb = block_table.shape
    for s in range(S):
        n = (int(seq_lens[s]) + B - 1) // B
        if n > mb:
            raise ValueError("sequence %d needs %d pages, table row holds %d" % (s, n, mb))
        used = block_table[s, :, :n]
        if used.size and (used.min() < 0 or used.max() >= P):
            raise ValueError("sequence %d: table entry outside [0, %d)" % (s, P))
