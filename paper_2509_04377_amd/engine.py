"""Host-side sequencing of C-ABI calls: the state of one paged cache, the decode step, and a multi-layer driver.

Nothing here computes a step of the path; every operation is a call into libpe through binding.py.  What
lives here is the control flow that belongs to the caller of the library: which calls a decode step makes
(Alg. 3: score + evict when a sequence's newest page has just filled at budget, then append, then attend),
and an integer mirror of the sequence lengths, so that the host can tell trigger steps without reading
anything back from the device (the kernels evaluate the same predicate on the device lengths).

Multi-layer driver: all layers' pages live in one physical pool; the block table is
[layers * S, Hk, max_blocks] with layer l owning rows l*S .. (l+1)*S - 1 ("layers folded into the sequence
dimension").  Scoring, eviction and the prefill prune see the folded table in ONE launch each; append and
attention are launched per layer, in layer order, because in a model layer l+1's query depends on layer l's
output.
"""
import ctypes
from dataclasses import dataclass
from typing import List, Optional

import torch

from . import binding as pe


class HostOnly:
    """While active, the drivers below advance their host-side bookkeeping (length mirror, which lengths array is
    current) without calling the library: the launches of such a step are replayed from a captured HIP graph."""
    active = False

    def __enter__(self):
        HostOnly.active = True

    def __exit__(self, *exc):
        HostOnly.active = False


def host_only():
    return HostOnly()


def _launch(fn, *args):
    """Call a binding function unless the step's launches come from a graph replay."""
    if not HostOnly.active:
        fn(*args)


def triggers(host_lens, block_size: int, budget: int) -> List[bool]:
    """Alg. 3's branch per sequence: the newest page has just filled (L % B == 0) and the sequence holds at
    least the budget (with a budget >= context nothing is ever evicted: Sec. 4.3)."""
    return [n > 0 and n % block_size == 0 and n >= budget for n in host_lens]


@dataclass
class PagedCache:
    """Device-side state of one paged KV cache (one layer, or several layers folded into num_seqs).

    Owns nothing but tensors; every operation is a C-ABI call."""
    desc: pe.pe_cache_desc
    k_pool: torch.Tensor       # [P, B, D]
    v_pool: torch.Tensor       # [P, B, D]
    block_table: torch.Tensor  # [S, Hk, max_blocks] int32
    seq_lens: torch.Tensor     # [S] int32
    spare: torch.Tensor        # [S, Hk, n_spare] int32
    spare_used: torch.Tensor   # [S, Hk] int32
    freed_phys: torch.Tensor   # [S, Hk] int32
    evicted_logical: torch.Tensor  # [S, Hk] int32
    scores: torch.Tensor       # [S, Hk, max_blocks] fp32
    budget: int
    decode_ws: torch.Tensor = None
    host_lens: list = None     # host mirror of seq_lens (pure integer bookkeeping, never read back)
    seq_lens_alt: torch.Tensor = None  # second lengths array for pe_append_paged_decode (swapped after each call)
    cached_scores: bool = False    # keep `scores` alive across steps and score only newly filled pages
    host_scored: list = None       # per sequence: full pages whose score is in `scores` (host bookkeeping)
    evict_opts: pe.pe_evict_opts = None  # eviction variant (policy, protected pages, shared heads); None = Alg. 3
    fused_evict: bool = False  # score + evict of a trigger step in one pass over the pages (pe_score_evict)

    @staticmethod
    def create(dtype, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, layout, budget, device="cuda",
               k_pool=None, v_pool=None, shared=False, decode_opts=None):
        """`layout`: block table, spare lists and pool size (synth.page_layout).  shared=True builds the
        head-shared cache (pe.PE_LAYOUT_SHARED): `layout` then describes ONE row per sequence (a layout made for a
        single KV head), pools are [P, B, Hk, D] and the per-row arrays lose their head dimension.  decode_opts:
        decode_splits / decode_shape / decode_flat_order of the descriptor (launch shape of the attention)."""
        desc = pe.make_desc(dtype, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, layout.max_blocks,
                            layout.num_phys_blocks, pe.PE_LAYOUT_SHARED if shared else pe.PE_LAYOUT_PER_HEAD,
                            **(decode_opts or {}))
        table, spare = layout.block_table, layout.spare
        if shared:
            assert table.shape[1] == 1, "a shared cache takes a layout with one row per sequence"
            table, spare = table[:, 0], spare[:, 0]
            shape = (layout.num_phys_blocks, block_size, num_kv_heads, head_dim)
            per_row = (num_seqs,)
        else:
            shape = (layout.num_phys_blocks, block_size, head_dim)
            per_row = (num_seqs, num_kv_heads)
        if k_pool is None:
            k_pool = torch.zeros(shape, dtype=dtype, device=device)
            v_pool = torch.zeros(shape, dtype=dtype, device=device)
        i32 = dict(dtype=torch.int32, device=device)
        cache = PagedCache(desc, k_pool, v_pool, table.to(device).contiguous(),
                           torch.zeros(num_seqs, **i32), spare.to(device).contiguous(),
                           torch.zeros(per_row, **i32), torch.full(per_row, -1, **i32),
                           torch.full(per_row, -1, **i32),
                           torch.empty((num_seqs, num_kv_heads, layout.max_blocks), dtype=torch.float32, device=device),
                           int(budget))
        cache.decode_ws = pe.alloc_workspace(pe.PE_OP_PAGED_DECODE, desc, device=device)
        cache.host_lens = [0] * num_seqs
        return cache

    @property
    def shared(self) -> bool:
        return self.desc.layout == pe.PE_LAYOUT_SHARED

    def prefill_prune(self, k_in, v_in, cu_seqlens, max_seqlen, kept_idx_out=None, workspace=None):
        total = k_in.shape[0]
        if workspace is None:
            workspace = pe.alloc_workspace(pe.PE_OP_PREFILL_PRUNE, self.desc, total, device=k_in.device)
        _launch(pe.pe_prefill_prune, self.desc, k_in, v_in, cu_seqlens, total, max_seqlen, self.budget, self.k_pool, self.v_pool,
                         self.block_table, self.seq_lens, kept_idx_out, workspace)

    def set_host_lens(self, prompt_lens):
        """Tell the host mirror what the prune was given: cached length = min(L, C)."""
        self.host_lens = [min(int(L), self.budget) for L in prompt_lens]

    def triggers(self) -> List[bool]:
        return triggers(self.host_lens, self.desc.block_size, self.budget)

    def any_trigger(self) -> bool:
        return any(self.triggers())

    def _sp(self, name, dtype=None):
        """Checked device pointer of one of the cache's own tensors, remembered per tensor object (the state
        tensors are passed on every call of a decode loop; their checks need not be repeated)."""
        t = getattr(self, name)
        memo = self.__dict__.setdefault("_ptr_memo", {})
        hit = memo.get(name)
        if hit is not None and hit[0] is t:
            return hit[1]
        alt = memo.get(name + "~")          # the two lengths arrays alternate
        if alt is not None and alt[0] is t:
            memo[name], memo[name + "~"] = alt, hit
            return alt[1]
        p = pe.ptr(t, name, dtype)
        if hit is not None:
            memo[name + "~"] = hit
        memo[name] = (t, p)
        return p

    def append_paged_decode(self, new_k, new_v, q, out, softmax_scale=None):
        if softmax_scale is None:
            softmax_scale = float(self.desc.head_dim) ** -0.5
        if self.seq_lens_alt is None:
            self.seq_lens_alt = torch.empty_like(self.seq_lens)
        if not HostOnly.active:
            i32 = torch.int32
            wp, wn = pe.ws_args(self.decode_ws)
            pe.check(pe.lib().pe_append_paged_decode(
                ctypes.byref(self.desc), pe.ptr(new_k, "new_k"), pe.ptr(new_v, "new_v"), pe.ptr(q, "q"),
                self._sp("k_pool"), self._sp("v_pool"), self._sp("block_table", i32), self._sp("seq_lens", i32),
                self._sp("seq_lens_alt", i32), self._sp("freed_phys", i32), self._sp("spare", i32),
                self._sp("spare_used", i32), int(self.spare.shape[-1]), ctypes.c_float(softmax_scale),
                pe.ptr(out, "out"), wp, wn, pe.stream_arg()), "pe_append_paged_decode")
        self.seq_lens, self.seq_lens_alt = self.seq_lens_alt, self.seq_lens

    def decode_step(self, new_k, new_v, q, out, softmax_scale=None, fused=True):
        """One decode iteration of one layer (Alg. 3): score + evict when some sequence's newest page has
        filled at budget, append the new token, attend.  Which steps trigger follows from the lengths
        alone, so the host decides it without reading anything back."""
        B = self.desc.block_size
        trig = self.triggers()
        if any(trig):
            self.score_and_evict()
            self.host_lens = [n - B if t else n for n, t in zip(self.host_lens, trig)]
        if fused:
            self.append_paged_decode(new_k, new_v, q, out, softmax_scale)
        else:
            self.append_kv(new_k, new_v)
            self.paged_decode(q, out, softmax_scale)
        self.host_lens = [n + 1 for n in self.host_lens]

    def score_blocks(self):
        _launch(pe.pe_score_blocks, self.desc, self.k_pool, self.v_pool, self.block_table, self.seq_lens, self.scores)

    def score_triggered_blocks(self):
        _launch(pe.pe_score_triggered_blocks, self.desc, self.k_pool, self.v_pool, self.block_table, self.seq_lens, self.budget,
                                  self.scores)

    def evict_blocks(self):
        _launch(pe.pe_evict_blocks, self.desc, self.scores, self.block_table, self.seq_lens, self.budget, self.evicted_logical,
                        self.freed_phys)

    def score_and_evict(self):
        """Score + evict of a trigger step.  With cached scores only the pages filled since the last call are
        scored (all of them the first time) and the eviction keeps the score rows aligned with the table."""
        B = self.desc.block_size
        if self.evict_opts is not None:
            o = self.evict_opts
            opts = pe.pe_evict_opts(o.policy, o.protect_first, o.protect_last, o.share_heads, 0)
            if o.policy != pe.PE_POLICY_OLDEST:
                self.score_triggered_blocks()
            _launch(pe.pe_evict_blocks_ex, self.desc, opts, self.scores if o.policy != pe.PE_POLICY_OLDEST else None,
                               self.block_table, self.seq_lens, self.budget, self.evicted_logical, self.freed_phys)
            return
        if self.fused_evict and not self.cached_scores:
            _launch(pe.pe_score_evict, self.desc, self.k_pool, self.v_pool, self.block_table, self.seq_lens, self.budget, None,
                           self.evicted_logical, self.freed_phys)
            return
        if not self.cached_scores:   # Alg. 3: score the pages of the sequences that evict now, then evict
            self.score_triggered_blocks()
            self.evict_blocks()
            return
        full = [n // B for n in self.host_lens]
        if self.host_scored is None:
            self.score_blocks()
        else:
            recent = max(f - sc for f, sc in zip(full, self.host_scored))
            if recent > 0:
                _launch(pe.pe_score_recent_blocks, self.desc, self.k_pool, self.v_pool, self.block_table, self.seq_lens, recent,
                                       self.scores)
        _launch(pe.pe_evict_blocks_cached, self.desc, self.scores, self.block_table, self.seq_lens, self.budget,
                               self.evicted_logical, self.freed_phys)
        self.host_scored = [f - 1 if t else f for f, t in zip(full, self.triggers())]

    def append_kv(self, new_k, new_v):
        if HostOnly.active:
            return
        i32 = torch.int32
        pe.check(pe.lib().pe_append_kv(ctypes.byref(self.desc), pe.ptr(new_k, "new_k"), pe.ptr(new_v, "new_v"),
                                  self._sp("k_pool"), self._sp("v_pool"), self._sp("block_table", i32),
                                  self._sp("seq_lens", i32), self._sp("freed_phys", i32), self._sp("spare", i32),
                                  self._sp("spare_used", i32), int(self.spare.shape[-1]), pe.stream_arg()), "pe_append_kv")

    def paged_decode(self, q, out, softmax_scale=None):
        if softmax_scale is None:
            softmax_scale = float(self.desc.head_dim) ** -0.5
        if HostOnly.active:
            return
        wp, wn = pe.ws_args(self.decode_ws)
        pe.check(pe.lib().pe_paged_decode(ctypes.byref(self.desc), pe.ptr(q, "q"), self._sp("k_pool"), self._sp("v_pool"),
                                     self._sp("block_table", torch.int32), self._sp("seq_lens", torch.int32),
                                     ctypes.c_float(softmax_scale), pe.ptr(out, "out"), wp, wn, pe.stream_arg()),
               "pe_paged_decode")


class LayeredCache:
    def __init__(self, dtype, layers, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, layout, budget,
                 device="cuda", shared=False, decode_opts=None):
        self.layers, self.S = layers, num_seqs
        self.Hk, self.Hq, self.D, self.B = num_kv_heads, num_q_heads, head_dim, block_size
        self.dtype, self.budget, self.device = dtype, int(budget), device
        R = layers * num_seqs
        assert layout.block_table.shape[0] == R
        self.folded = PagedCache.create(dtype, R, num_kv_heads, num_q_heads, head_dim, block_size, layout, budget,
                                        device, shared=shared)
        f = self.folded
        self.per_layer: List[PagedCache] = []
        for l in range(layers):
            sl = slice(l * num_seqs, (l + 1) * num_seqs)
            desc = pe.make_desc(dtype, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, layout.max_blocks,
                                layout.num_phys_blocks, pe.PE_LAYOUT_SHARED if shared else pe.PE_LAYOUT_PER_HEAD,
                                **(decode_opts or {}))
            c = PagedCache(desc, f.k_pool, f.v_pool, f.block_table[sl], f.seq_lens[sl], f.spare[sl],
                              f.spare_used[sl], f.freed_phys[sl], f.evicted_logical[sl], f.scores[sl], int(budget))
            self.per_layer.append(c)
        # one split workspace serves every layer: launches are ordered on one stream
        self.decode_ws = pe.alloc_workspace(pe.PE_OP_PAGED_DECODE, self.per_layer[0].desc, device=device)
        # second lengths array for the fused append + attention call; all layers swap in lockstep
        f.seq_lens_alt = torch.empty_like(f.seq_lens)
        for l, c in enumerate(self.per_layer):
            c.decode_ws = self.decode_ws
            c.seq_lens_alt = f.seq_lens_alt[l * num_seqs:(l + 1) * num_seqs]
        self.fused = True
        self.native_layers = True   # fused mode: the per-layer launches are issued by one native call
        self.host_lens = [0] * num_seqs   # the same in every layer

    def prefill_prune_layer(self, layer, k_in, v_in, cu_seqlens, max_seqlen, kept_idx_out=None, workspace=None):
        self.per_layer[layer].prefill_prune(k_in, v_in, cu_seqlens, max_seqlen, kept_idx_out, workspace)

    def set_host_lens(self, prompt_lens):
        self.host_lens = [min(int(L), self.budget) for L in prompt_lens]

    def _triggers(self):
        return triggers(self.host_lens, self.B, self.budget)

    def decode_step(self, new_k, new_v, q, out, softmax_scale: Optional[float] = None, layer_hook=None):
        """new_k, new_v [layers, S, Hk, D]; q, out [layers, S, Hq, D].  One decode iteration of all layers."""
        trig = self._triggers()
        if any(trig):
            self.folded.host_lens = self.host_lens * self.layers
            self.folded.score_and_evict()
            self.host_lens = [n - self.B if t else n for n, t in zip(self.host_lens, trig)]
        if self.fused and self.native_layers:
            # one native call issues the fused append + attention launch of every layer, in layer order
            f = self.folded
            if layer_hook is not None:
                layer_hook(0, 0)
            _launch(pe.pe_append_paged_decode_layers, self.per_layer[0].desc, self.layers, new_k, new_v, q, f.k_pool, f.v_pool,
                                             f.block_table, f.seq_lens, f.seq_lens_alt, f.freed_phys, f.spare,
                                             f.spare_used, float(self.D) ** -0.5 if softmax_scale is None
                                             else softmax_scale, out, self.decode_ws)
            if layer_hook is not None:
                layer_hook(self.layers - 1, 1)
            for c in self.per_layer:
                c.seq_lens, c.seq_lens_alt = c.seq_lens_alt, c.seq_lens
        for l, c in enumerate(self.per_layer if not (self.fused and self.native_layers) else ()):
            if self.fused:
                if layer_hook is not None:
                    layer_hook(l, 0)
                c.append_paged_decode(new_k[l], new_v[l], q[l], out[l], softmax_scale)
            else:
                c.append_kv(new_k[l], new_v[l])
                if layer_hook is not None:
                    layer_hook(l, 0)
                c.paged_decode(q[l], out[l], softmax_scale)
            if layer_hook is not None:
                layer_hook(l, 1)
        if self.fused:   # every layer wrote its new lengths into the other array
            self.folded.seq_lens, self.folded.seq_lens_alt = self.folded.seq_lens_alt, self.folded.seq_lens
        self.host_lens = [n + 1 for n in self.host_lens]
        return any(trig)


class GraphedStepper:
    """Replays the launches of a decode step from captured HIP graphs (one per distinct launch sequence).

    The inputs live in fixed buffers (new_k, new_v, q, out), as a serving loop would keep them.  A step's
    launch sequence depends only on host-side integers (which lengths array is current, whether this is a
    trigger step, how many pages the cached-score mode has to score), so that tuple keys the graph.  The
    first step with a new key is captured and then replayed; later ones advance the host bookkeeping with
    the launches switched off and replay the stored graph."""

    def __init__(self, eng: "LayeredCache", new_k, new_v, q, out, softmax_scale: Optional[float] = None):
        self.eng, self.args = eng, (new_k, new_v, q, out, softmax_scale)
        self.graphs = {}

    def _key(self):
        e, f = self.eng, self.eng.folded
        trig = any(e._triggers())
        recent = None
        if trig and f.cached_scores:
            if f.host_scored is None:
                recent = -1
            else:
                recent = max(n // e.B - sc for n, sc in zip(e.host_lens * e.layers, f.host_scored))
        return (f.seq_lens.data_ptr(), trig, e.fused, f.cached_scores, f.fused_evict, recent)

    def step(self) -> bool:
        key = self._key()
        g = self.graphs.get(key)
        if g is None:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                trig = self.eng.decode_step(*self.args)
            self.graphs[key] = g
        else:
            with host_only():
                trig = self.eng.decode_step(*self.args)
        g.replay()
        return trig
