"""Seeded synthetic workloads: shapes, value distributions and page layouts only.

This module serves both the HIP path and the CPU oracle's tests.  It holds none of the method's
arithmetic (no norms, scores, selection, softmax): it draws random K/V/q with the stated
distributions and hands out physical page ids.

The paper's throughput workload is itself synthetic on real weights and its accuracy workload is a
public long-context benchmark (Sec. 5.1); neither weights nor benchmark data are used here.  The
caches below only take the SHAPES of the three Llama models the paper names, its budgets
{256..4096} and its page sizes {16, 32}.
"""
from dataclasses import dataclass, replace
from typing import List, Optional, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    index: int               # position in the benchmark's config list (1-based)
    dtype: str               # "f32" or "bf16"
    layers: int
    num_kv_heads: int
    num_q_heads: int
    head_dim: int
    block_size: int
    num_seqs: int
    context: Tuple[int, ...]  # (L,) fixed, or (lo, hi) drawn uniformly per sequence
    budget: int
    steps: int
    dist: str                # "outlier5" | "lognormal" | "lognormal_sink"
    permute_pool: bool

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five configurations of the benchmark definition.
TINY = Workload("tiny_f32", 1, "f32", 1, 4, 8, 64, 16, 1, (512,), 256, 32, "outlier5", False)
LLAMA32_1B = Workload("llama32_1b", 2, "bf16", 16, 8, 32, 64, 16, 8, (4096,), 1024, 256, "lognormal", False)
LLAMA32_3B = Workload("llama32_3b", 3, "bf16", 28, 8, 24, 128, 16, 16, (2048, 16384), 1024, 512,
                      "lognormal_sink", False)
LLAMA31_8B = Workload("llama31_8b", 4, "bf16", 32, 8, 32, 128, 16, 32, (16384,), 2048, 256,
                      "lognormal_sink", True)
LONG_8B = Workload("llama31_8b_long", 5, "bf16", 32, 8, 32, 128, 16, 4, (65536,), 4096, 128,
                   "lognormal_sink", True)

WORKLOADS = {w.name: w for w in (TINY, LLAMA32_1B, LLAMA32_3B, LLAMA31_8B, LONG_8B)}


def seed_for(base_seed: int, workload: Workload, layer: int = 0) -> int:
    return int(base_seed) + 1000 * workload.index + int(layer)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def context_lengths(wl: Workload, base_seed: int) -> List[int]:
    """Prompt length of every sequence (the same for all layers)."""
    if len(wl.context) == 1:
        return [int(wl.context[0])] * wl.num_seqs
    lo, hi = wl.context
    g = _gen(seed_for(base_seed, wl) + 500, "cpu")
    return [int(x) for x in torch.randint(lo, hi + 1, (wl.num_seqs,), generator=g)]


def _rows(wl: Workload, n_tokens: int, heads: int, g: torch.Generator, device, scaled: bool) -> torch.Tensor:
    """[n_tokens, heads, D] fp32 rows ~ N(0,1), times the workload's per-(token, head) scale."""
    x = torch.randn((n_tokens, heads, wl.head_dim), generator=g, device=device, dtype=torch.float32)
    if not scaled:
        return x
    if wl.dist == "outlier5":
        hit = torch.rand((n_tokens, heads, 1), generator=g, device=device) < 0.05
        fac = 2.0 + 2.0 * torch.rand((n_tokens, heads, 1), generator=g, device=device)
        x = x * torch.where(hit, fac, torch.ones_like(fac))
    else:
        sc = torch.exp(0.5 * torch.randn((n_tokens, heads, 1), generator=g, device=device))
        x = x * sc
    return x


def prompt_kv(wl: Workload, layer: int, lens: List[int], base_seed: int, device="cpu"):
    """Packed prompt K and V, [sum(lens), Hk, D] in the workload dtype, and cu_seqlens [S+1] int32.

    K and V get independent scale draws.  With "lognormal_sink" the V rows of each sequence's first
    four tokens are multiplied by 8 (K unchanged)."""
    g = _gen(seed_for(base_seed, wl, layer), device)
    total = sum(lens)
    k = _rows(wl, total, wl.num_kv_heads, g, device, True)
    v = _rows(wl, total, wl.num_kv_heads, g, device, True)
    cu = [0]
    for n in lens:
        cu.append(cu[-1] + n)
    if wl.dist == "lognormal_sink":
        for s, n in enumerate(lens):
            v[cu[s]:cu[s] + min(4, n)] *= 8.0
    cu_t = torch.tensor(cu, dtype=torch.int32, device=device)
    return k.to(wl.torch_dtype), v.to(wl.torch_dtype), cu_t


def decode_inputs(wl: Workload, layer: int, step: int, base_seed: int, device="cpu", num_seqs: Optional[int] = None):
    """New token K, V [S, Hk, D] (same distribution as the prompt, no sink scaling) and q [S, Hq, D]."""
    S = wl.num_seqs if num_seqs is None else num_seqs
    g = _gen(seed_for(base_seed, wl, layer) + 7919 * (step + 1), device)
    k = _rows(wl, S, wl.num_kv_heads, g, device, True)
    v = _rows(wl, S, wl.num_kv_heads, g, device, True)
    q = _rows(wl, S, wl.num_q_heads, g, device, False)
    return k.to(wl.torch_dtype), v.to(wl.torch_dtype), q.to(wl.torch_dtype)


@dataclass
class PageLayout:
    block_table: torch.Tensor   # [R, Hk, max_blocks] int32 (R = folded sequences), -1 = unused
    spare: torch.Tensor         # [R, Hk, n_spare] int32
    max_blocks: int
    n_spare: int
    num_phys_blocks: int


def page_layout(wl: Workload, lens: List[int], base_seed: int, budget: Optional[int] = None,
                steps: Optional[int] = None, extra_blocks: int = 0, shared: bool = False) -> PageLayout:
    """Physical pages for `len(lens)` sequences x Hk rows (fold layers in by repeating `lens`).

    A row gets ceil(min(L, C)/B) pages for the pruned prompt and as many spare pages as it can still
    grow into before it reaches the budget (at least one).  Ids are consecutive in row order, or a
    seeded random permutation of the whole pool when the workload asks for a shared, shuffled pool.
    shared=True lays out the head-shared cache: one row per sequence (the Hk axis has length 1)."""
    B = wl.block_size
    C = wl.budget if budget is None else budget
    steps = wl.steps if steps is None else steps
    R, Hk = len(lens), (1 if shared else wl.num_kv_heads)
    init = [(min(L, C) + B - 1) // B for L in lens]
    grown = [(min(L + steps, C) + B - 1) // B for L in lens]
    max_blocks = max(max(grown), max(init)) + extra_blocks
    n_spare = max(1, max(gr - it for gr, it in zip(grown, init)))
    per_row = [it + n_spare for it in init]
    P = Hk * sum(per_row)
    if wl.permute_pool:
        ids = torch.randperm(P, generator=_gen(seed_for(base_seed, wl) + 900, "cpu")).to(torch.int32)
    else:
        ids = torch.arange(P, dtype=torch.int32)
    table = torch.full((R, Hk, max_blocks), -1, dtype=torch.int32)
    spare = torch.empty((R, Hk, n_spare), dtype=torch.int32)
    pos = 0
    for r in range(R):
        for h in range(Hk):
            table[r, h, :init[r]] = ids[pos:pos + init[r]]
            pos += init[r]
            spare[r, h] = ids[pos:pos + n_spare]
            pos += n_spare
    return PageLayout(table, spare, max_blocks, n_spare, P)
