"""A decode step replayed from captured HIP graphs must do exactly what the eager launches do: two engines
on identical state, one stepped eagerly and one through GraphedStepper, compared bit for bit after every
step (tables, lengths, scores, outputs), with the eager engine's work and synchronisations in between the
replays, over several trigger periods, with and without cached page scores."""
import numpy as np
import pytest
import torch

from paper_2509_04377_amd import synth
from paper_2509_04377_amd.engine import GraphedStepper, LayeredCache

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = 77


def _engine(wl, lens, layout, prompts, cached):
    eng = LayeredCache(wl.torch_dtype, wl.layers, wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim,
                       wl.block_size, layout, wl.budget, DEV)
    for l, (k_in, v_in, cu) in enumerate(prompts):
        eng.prefill_prune_layer(l, k_in.to(DEV), v_in.to(DEV), cu.to(DEV), max(lens))
    eng.set_host_lens(lens)
    eng.folded.cached_scores = cached
    return eng


@pytest.mark.parametrize("cached", [False, True])
def test_graph_replay_equals_eager(cached):
    print("case graph replay cached", cached, flush=True)
    wl = synth.LLAMA32_1B.with_(layers=3, num_seqs=3, context=(300,), budget=256)
    steps = 40
    lens = synth.context_lengths(wl, SEED)
    layout = synth.page_layout(wl, lens * wl.layers, SEED, steps=steps)
    prompts = [synth.prompt_kv(wl, l, lens, SEED) for l in range(wl.layers)]
    eager = _engine(wl, lens, layout, prompts, cached)
    graphed = _engine(wl, lens, layout, prompts, cached)
    L, S, Hk, Hq, D = wl.layers, wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim
    bufs = [torch.empty((L, S, Hk, D), dtype=wl.torch_dtype, device=DEV) for _ in range(2)]
    qbuf = torch.empty((L, S, Hq, D), dtype=wl.torch_dtype, device=DEV)
    out_g = torch.empty((L, S, Hq, D), dtype=wl.torch_dtype, device=DEV)
    out_e = torch.empty_like(out_g)
    stepper = GraphedStepper(graphed, bufs[0], bufs[1], qbuf, out_g)
    n_trig = 0
    for step in range(steps):
        ins = [synth.decode_inputs(wl, l, step, SEED) for l in range(L)]
        nk = torch.stack([x[0] for x in ins]).to(DEV)
        nv = torch.stack([x[1] for x in ins]).to(DEV)
        q = torch.stack([x[2] for x in ins]).to(DEV)
        bufs[0].copy_(nk); bufs[1].copy_(nv); qbuf.copy_(q)
        torch.cuda.synchronize()
        n_trig += bool(stepper.step())
        eager.decode_step(nk, nv, q, out_e)
        torch.cuda.synchronize()
        where = "step %d" % step
        assert torch.equal(out_g.view(torch.int16), out_e.view(torch.int16)), where
        assert torch.equal(graphed.folded.block_table, eager.folded.block_table), where
        assert torch.equal(graphed.folded.seq_lens, eager.folded.seq_lens), where
        assert graphed.host_lens == eager.host_lens
        if cached:
            assert torch.equal(graphed.folded.scores.view(torch.int32), eager.folded.scores.view(torch.int32)), where
    assert n_trig == 3                       # steps 0, 16, 32 (the pruned prompt sits exactly at budget)
    assert len(stepper.graphs) <= 5          # a handful of distinct launch sequences, replayed many times
    assert np.array_equal(graphed.folded.seq_lens.cpu().numpy(), np.array(graphed.host_lens * L, dtype=np.int32))
