"""Multi-layer decode driver over one shared page pool (host-side sequencing of C-ABI calls only).

All layers' pages live in one physical pool; the block table is [layers * S, Hk, max_blocks] with
layer l owning rows l*S .. (l+1)*S - 1 ("layers folded into the sequence dimension").  Scoring,
eviction and the prefill prune see the folded table in ONE launch each; append and attention are
launched per layer, in layer order, because in a model layer l+1's query depends on layer l's output.
"""
from typing import List, Optional

import torch

from . import binding as pe


class LayeredCache:
    def __init__(self, dtype, layers, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, layout, budget,
                 device="cuda", shared=False):
        self.layers, self.S = layers, num_seqs
        self.Hk, self.Hq, self.D, self.B = num_kv_heads, num_q_heads, head_dim, block_size
        self.dtype, self.budget, self.device = dtype, int(budget), device
        R = layers * num_seqs
        assert layout.block_table.shape[0] == R
        self.folded = pe.PagedCache.create(dtype, R, num_kv_heads, num_q_heads, head_dim, block_size, layout, budget,
                                           device, shared=shared)
        f = self.folded
        self.per_layer: List[pe.PagedCache] = []
        for l in range(layers):
            sl = slice(l * num_seqs, (l + 1) * num_seqs)
            desc = pe.make_desc(dtype, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, layout.max_blocks,
                                layout.num_phys_blocks, pe.PE_LAYOUT_SHARED if shared else pe.PE_LAYOUT_PER_HEAD)
            c = pe.PagedCache(desc, f.k_pool, f.v_pool, f.block_table[sl], f.seq_lens[sl], f.spare[sl],
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
        self.host_lens = [0] * num_seqs   # the same in every layer

    def prefill_prune_layer(self, layer, k_in, v_in, cu_seqlens, max_seqlen, kept_idx_out=None, workspace=None):
        self.per_layer[layer].prefill_prune(k_in, v_in, cu_seqlens, max_seqlen, kept_idx_out, workspace)

    def set_host_lens(self, prompt_lens):
        self.host_lens = [min(int(L), self.budget) for L in prompt_lens]

    def _triggers(self):
        B, C = self.B, self.budget
        return [n > 0 and n % B == 0 and n >= C for n in self.host_lens]

    def decode_step(self, new_k, new_v, q, out, softmax_scale: Optional[float] = None, layer_hook=None):
        """new_k, new_v [layers, S, Hk, D]; q, out [layers, S, Hq, D].  One decode iteration of all layers."""
        trig = self._triggers()
        if any(trig):
            self.folded.host_lens = self.host_lens * self.layers
            self.folded.score_and_evict()
            self.host_lens = [n - self.B if t else n for n, t in zip(self.host_lens, trig)]
        for l, c in enumerate(self.per_layer):
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
            with pe.host_only():
                trig = self.eng.decode_step(*self.args)
        g.replay()
        return trig
