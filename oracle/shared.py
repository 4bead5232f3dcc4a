"""Head-shared reading (one block table row and one decision per sequence, pages [B, Hk, D]) -- numpy front
end of ``pe_oracle_shared.c`` and its decode-step protocol.  TEST INFRASTRUCTURE ONLY."""
import ctypes
from dataclasses import dataclass

import numpy as np

from . import _f32, _f32p, _f64p, _i32, _i32p, _load, _p

_ready = False


def _lib():
    global _ready
    lib = _load()
    if not _ready:
        ci = ctypes.c_int
        lib.oracle_sh_score_blocks.restype = None
        lib.oracle_sh_score_blocks.argtypes = [_f32p, _f32p, _i32p, _i32p] + [ci] * 5 + [_f32p, _f32p]
        lib.oracle_sh_prefill_prune.restype = ci
        lib.oracle_sh_prefill_prune.argtypes = ([_f32p, _f32p, _i32p] + [ci] * 6 +
                                                [_f32p, _f32p, _i32p, _i32p, _i32p, _f32p])
        lib.oracle_sh_evict_blocks.restype = ci
        lib.oracle_sh_evict_blocks.argtypes = [_f32p, _i32p, _i32p] + [ci] * 8 + [_i32p, _i32p]
        lib.oracle_sh_append_kv.restype = ci
        lib.oracle_sh_append_kv.argtypes = [_f32p, _f32p, _f32p, _f32p, _i32p, _i32p, _i32p, _i32p, _i32p] + [ci] * 6
        lib.oracle_sh_paged_decode.restype = None
        lib.oracle_sh_paged_decode.argtypes = ([_f32p, _f32p, _f32p, _i32p, _i32p] + [ci] * 6 +
                                               [ctypes.c_double, _f64p, _f64p])
        _ready = True
    return lib


def _check_table(block_table, seq_lens, B, P):
    S, mb = block_table.shape
    for s in range(S):
        n = (int(seq_lens[s]) + B - 1) // B
        if n > mb:
            raise ValueError("sequence %d needs %d pages, table row holds %d" % (s, n, mb))
        used = block_table[s, :n]
        if used.size and (used.min() < 0 or used.max() >= P):
            raise ValueError("sequence %d: table entry outside [0, %d)" % (s, P))


def score_blocks(k_pool, v_pool, block_table, seq_lens):
    """Pools [P, B, Hk, D], table [S, max_blocks] -> (head scores [S, Hk, max_blocks], page scores [S, max_blocks])."""
    k_pool, v_pool = _f32(k_pool), _f32(v_pool)
    block_table, seq_lens = _i32(block_table), _i32(seq_lens)
    P, B, Hk, D = k_pool.shape
    S, mb = block_table.shape
    assert v_pool.shape == k_pool.shape and seq_lens.shape == (S,)
    _check_table(block_table, seq_lens, B, P)
    hs = np.empty((S, Hk, mb), np.float32)
    ps = np.empty((S, mb), np.float32)
    _lib().oracle_sh_score_blocks(_p(k_pool, _f32p), _p(v_pool, _f32p), _p(block_table, _i32p), _p(seq_lens, _i32p),
                                  S, Hk, D, B, mb, _p(hs, _f32p), _p(ps, _f32p))
    return hs, ps


def prefill_prune(k_in, v_in, cu_seqlens, budget, k_pool, v_pool, block_table, want_scores=False):
    """Packed prompt [T, Hk, D] pruned into pools [P, B, Hk, D] (in place).  Returns (seq_lens [S],
    kept_idx [S, budget]) and, if asked, the fp32 head-mean token scores [T]."""
    k_in, v_in = _f32(k_in), _f32(v_in)
    cu_seqlens, block_table = _i32(cu_seqlens), _i32(block_table)
    T, Hk, D = k_in.shape
    P, B, Hk2, D2 = k_pool.shape
    S, mb = block_table.shape
    assert (Hk, D) == (Hk2, D2) and cu_seqlens.shape == (S + 1,) and int(cu_seqlens[-1]) == T
    for a in (k_pool, v_pool):
        assert a.dtype == np.float32 and a.flags.c_contiguous
    lens = np.minimum(np.diff(cu_seqlens), budget).astype(np.int32)
    _check_table(block_table, lens, B, P)
    seq_lens = np.zeros((S,), np.int32)
    kept = np.empty((S, budget), np.int32)
    tsc = np.empty((T,), np.float32) if want_scores else None
    rc = _lib().oracle_sh_prefill_prune(_p(k_in, _f32p), _p(v_in, _f32p), _p(cu_seqlens, _i32p), S, Hk, D, B,
                                        int(budget), mb, _p(k_pool, _f32p), _p(v_pool, _f32p),
                                        _p(block_table, _i32p), _p(seq_lens, _i32p), _p(kept, _i32p),
                                        _p(tsc, _f32p) if want_scores else None)
    if rc != 0:
        raise ValueError("oracle_sh_prefill_prune failed with status %d" % rc)
    return (seq_lens, kept, tsc) if want_scores else (seq_lens, kept)


def evict_blocks(head_scores, block_table, seq_lens, block_size, budget, policy=0, protect_first=0, protect_last=0):
    """In place on block_table [S, max_blocks] / seq_lens.  Returns (evicted_logical [S], freed_phys [S])."""
    S, mb = block_table.shape
    assert block_table.dtype == np.int32 and block_table.flags.c_contiguous
    assert seq_lens.dtype == np.int32 and seq_lens.flags.c_contiguous
    Hk = 1
    if head_scores is not None:
        head_scores = _f32(head_scores)
        Hk = head_scores.shape[1]
        assert head_scores.shape == (S, Hk, mb)
    ev = np.empty((S,), np.int32)
    fr = np.empty((S,), np.int32)
    rc = _lib().oracle_sh_evict_blocks(_p(head_scores, _f32p) if head_scores is not None else None,
                                       _p(block_table, _i32p), _p(seq_lens, _i32p), S, Hk, int(block_size), mb,
                                       int(budget), int(policy), int(protect_first), int(protect_last),
                                       _p(ev, _i32p), _p(fr, _i32p))
    if rc != 0:
        raise ValueError("oracle_sh_evict_blocks failed with status %d" % rc)
    return ev, fr


def append_kv(new_k, new_v, k_pool, v_pool, block_table, seq_lens, freed_phys, spare, spare_used):
    """In place.  new_k/new_v [S, Hk, D]; freed_phys [S]; spare [S, n_spare]; spare_used [S]."""
    new_k, new_v = _f32(new_k), _f32(new_v)
    S, Hk, D = new_k.shape
    P, B, _, _ = k_pool.shape
    mb = block_table.shape[1]
    for a in (block_table, seq_lens, freed_phys, spare, spare_used):
        assert a.dtype == np.int32 and a.flags.c_contiguous
    rc = _lib().oracle_sh_append_kv(_p(new_k, _f32p), _p(new_v, _f32p), _p(k_pool, _f32p), _p(v_pool, _f32p),
                                    _p(block_table, _i32p), _p(seq_lens, _i32p), _p(freed_phys, _i32p),
                                    _p(spare, _i32p), _p(spare_used, _i32p), spare.shape[1], S, Hk, D, B, mb)
    if rc != 0:
        raise ValueError("oracle_sh_append_kv failed with status %d" % rc)


def paged_decode(q, k_pool, v_pool, block_table, seq_lens, scale=None, want_weight_sums=False):
    q, k_pool, v_pool = _f32(q), _f32(k_pool), _f32(v_pool)
    block_table, seq_lens = _i32(block_table), _i32(seq_lens)
    S, Hq, D = q.shape
    P, B, Hk, _ = k_pool.shape
    mb = block_table.shape[1]
    assert Hq % Hk == 0
    _check_table(block_table, seq_lens, B, P)
    if scale is None:
        scale = 1.0 / np.sqrt(float(D))
    out = np.empty((S, Hq, D), np.float64)
    ws = np.empty((S, Hq), np.float64)
    _lib().oracle_sh_paged_decode(_p(q, _f32p), _p(k_pool, _f32p), _p(v_pool, _f32p), _p(block_table, _i32p),
                                  _p(seq_lens, _i32p), S, Hk, Hq, D, B, mb, float(scale), _p(out, _f64p),
                                  _p(ws, _f64p))
    return (out, ws) if want_weight_sums else out


@dataclass
class SharedOracleCache:
    k_pool: np.ndarray       # [P, B, Hk, D] float32
    v_pool: np.ndarray
    block_table: np.ndarray  # [S, max_blocks] int32
    seq_lens: np.ndarray     # [S] int32
    spare: np.ndarray        # [S, n_spare] int32
    spare_used: np.ndarray   # [S] int32
    freed_phys: np.ndarray   # [S] int32
    budget: int


def decode_step(cache: SharedOracleCache, new_k, new_v, q, scale=None, policy=0, protect_first=0, protect_last=0):
    """Evict (if a sequence's newest page has filled at budget), append, attend.  Returns
    (out fp64, head scores or None, evicted_logical [S], freed_phys [S])."""
    B, C = cache.k_pool.shape[1], cache.budget
    lens = cache.seq_lens
    S = lens.shape[0]
    scores = None
    if np.any((lens > 0) & (lens % B == 0) & (lens >= C)):
        if policy == 0:
            scores, _ = score_blocks(cache.k_pool, cache.v_pool, cache.block_table, cache.seq_lens)
        evicted, freed = evict_blocks(scores, cache.block_table, cache.seq_lens, B, C, policy, protect_first,
                                      protect_last)
    else:
        evicted = np.full((S,), -1, np.int32)
        freed = np.full((S,), -1, np.int32)
    cache.freed_phys[...] = freed
    append_kv(new_k, new_v, cache.k_pool, cache.v_pool, cache.block_table, cache.seq_lens, cache.freed_phys,
              cache.spare, cache.spare_used)
    out = paged_decode(q, cache.k_pool, cache.v_pool, cache.block_table, cache.seq_lens, scale)
    return out, scores, evicted, freed.copy()
