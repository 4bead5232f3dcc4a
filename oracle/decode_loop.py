"""Decode-step protocol of the oracle (TEST INFRASTRUCTURE ONLY).

One step, per layer, in the order of Alg. 3 with the harness append in between:
  (i)   score every page and evict one page from each row whose tail page is full and which
        holds at least the budget (Alg. 3, the "L % B == 0" branch);
  (ii)  append the new token's K/V (a new page is linked in when the tail is full);
  (iii) attention of the new query over everything cached, the new token included
        (Alg. 3, "PagedAttention(Q, K, V)").
"""
from dataclasses import dataclass

import numpy as np

from . import POLICY_OLDEST, append_kv, evict_blocks, evict_blocks_ex, paged_decode, score_blocks


@dataclass
class OracleCache:
    k_pool: np.ndarray       # [P, B, D] float32
    v_pool: np.ndarray       # [P, B, D] float32
    block_table: np.ndarray  # [S, Hk, max_blocks] int32, -1 = unused
    seq_lens: np.ndarray     # [S] int32
    spare: np.ndarray        # [S, Hk, n_spare] int32 physical pages a row may still take
    spare_used: np.ndarray   # [S, Hk] int32
    freed_phys: np.ndarray   # [S, Hk] int32, page freed by the last eviction and not yet reused
    budget: int

    @property
    def block_size(self) -> int:
        return self.k_pool.shape[1]


def decode_step(cache: OracleCache, new_k, new_v, q, scale=None, evict_opts=None):
    """Runs (i)-(iii) in place on `cache`.  Returns (out fp64, scores, evicted_logical, freed_phys);
    scores is None on a step where no sequence's newest page has just filled at budget (Alg. 3 scores
    pages only inside its "L % B == 0" branch).  `evict_opts` (policy, protect_first, protect_last,
    share_heads) selects an eviction variant; None is the paper's lowest-score rule."""
    B, C = cache.block_size, cache.budget
    lens = cache.seq_lens
    if np.any((lens > 0) & (lens % B == 0) & (lens >= C)):
        if evict_opts is None:
            scores = score_blocks(cache.k_pool, cache.v_pool, cache.block_table, cache.seq_lens)
            evicted, freed = evict_blocks(scores, cache.block_table, cache.seq_lens, B, C)
        else:
            scores = None
            if evict_opts.get("policy", 0) != POLICY_OLDEST:
                scores = score_blocks(cache.k_pool, cache.v_pool, cache.block_table, cache.seq_lens)
            evicted, freed = evict_blocks_ex(scores, cache.block_table, cache.seq_lens, B, C, **evict_opts)
    else:
        scores = None
        evicted = np.full(cache.freed_phys.shape, -1, np.int32)
        freed = np.full(cache.freed_phys.shape, -1, np.int32)
    freed_report = freed.copy()
    cache.freed_phys[...] = freed
    append_kv(new_k, new_v, cache.k_pool, cache.v_pool, cache.block_table, cache.seq_lens,
              cache.freed_phys, cache.spare, cache.spare_used)
    out = paged_decode(q, cache.k_pool, cache.v_pool, cache.block_table, cache.seq_lens, scale)
    return out, scores, evicted, freed_report
