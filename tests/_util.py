"""Shared test helpers: turn a synthetic workload into oracle-side (numpy) state."""
import numpy as np
import torch

import oracle
from oracle.decode_loop import OracleCache
from paper_2509_04377_amd import synth


def f32(t: torch.Tensor) -> np.ndarray:
    """Exact conversion of a torch tensor (fp32 or bf16, any device) to a float32 numpy array."""
    return t.detach().to("cpu").to(torch.float32).contiguous().numpy()


def i32(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.int32).contiguous().numpy()


def oracle_prefill(wl, lens, k_in, v_in, cu, layout, budget):
    """Run the oracle's prefill prune into fresh pools.  Returns (OracleCache, kept_idx, token scores)."""
    B, D = wl.block_size, wl.head_dim
    k_pool = np.zeros((layout.num_phys_blocks, B, D), np.float32)
    v_pool = np.zeros((layout.num_phys_blocks, B, D), np.float32)
    table = i32(layout.block_table).copy()
    seq_lens, kept, tsc = oracle.prefill_prune(f32(k_in), f32(v_in), i32(cu), budget, k_pool, v_pool, table,
                                               want_scores=True)
    S, Hk = table.shape[:2]
    cache = OracleCache(k_pool, v_pool, table, seq_lens, i32(layout.spare).copy(),
                        np.zeros((S, Hk), np.int32), np.full((S, Hk), -1, np.int32), budget)
    return cache, kept, tsc


def rel_err(got: np.ndarray, ref: np.ndarray):
    """Per-vector errors over the last axis: (||got-ref||_2/||ref||_2, max|got-ref|/max|ref|), worst case."""
    got = got.astype(np.float64)
    d = got - ref
    n2 = np.linalg.norm(d, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-300)
    mx = np.abs(d).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-300)
    return float(n2.max()), float(mx.max())
