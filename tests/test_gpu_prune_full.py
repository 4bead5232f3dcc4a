"""Prefill prune (Alg. 2) at the full batch of every benchmark shape, in the launches bench.py makes.

bench.py prunes one layer at a time through the layered driver: total_tokens = sum of the prompt lengths of the
whole batch, max_seqlen = the longest prompt, the layer's slice of the folded block table, one pool shared by
the layers.  These tests make exactly those calls (a two-layer driver, the second layer compared, so that the
table slice and the pool offsets are not the trivial ones) and compare seq_lens, the kept token indices and the
whole pool, bit for bit, with the oracle's prune of the same seeded prompts.  What differs from the smaller
prune tests is what depends on many sequences and a large total_tokens: the per-chunk count slots, the
head-major score stores, the multi-workgroup selection of long rows.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import shared as osh
from paper_2509_04377_amd import synth
from paper_2509_04377_amd.engine import LayeredCache

from _util import f32, i32

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = 4377

CASES = [
    pytest.param(synth.LLAMA31_8B, id="llama31_8b_32x16384_to_2048"),
    pytest.param(synth.LLAMA32_3B, id="llama32_3b_16_ragged_to_1024"),
    pytest.param(synth.LLAMA32_1B, id="llama32_1b_8x4096_to_1024"),
    pytest.param(synth.LONG_8B, id="long_4x65536_to_4096_B16"),
    pytest.param(synth.LONG_8B.with_(context=(131072,), budget=8192, block_size=32), id="long_4x131072_to_8192_B32"),
]


@pytest.mark.parametrize("shared", [False, True], ids=["per_head", "shared"])
@pytest.mark.parametrize("wl", CASES)
def test_prune_full_batch(wl, shared):
    print("case prune full batch", wl.name, wl.context, wl.budget, wl.block_size, "shared" if shared else "per_head",
          flush=True)
    layers, l = 2, 1
    S, Hk, Hq, D, B, C = wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim, wl.block_size, wl.budget
    lens = synth.context_lengths(wl, SEED)
    assert max(lens) > C, "the case must really prune"
    layout = synth.page_layout(wl, lens * layers, SEED, steps=4, shared=shared)
    eng = LayeredCache(wl.torch_dtype, layers, S, Hk, Hq, D, B, layout, C, DEV, shared=shared)
    k_dev, v_dev, cu = synth.prompt_kv(wl, l, lens, SEED, device=DEV)   # drawn on the device, as bench.py does
    kept = torch.full((S, C) if shared else (S, Hk, C), -9, dtype=torch.int32, device=DEV)
    eng.prefill_prune_layer(l, k_dev, v_dev, cu, max(lens), kept)
    torch.cuda.synchronize()
    k_in, v_in = f32(k_dev), f32(v_dev)                                 # the same values for the oracle
    del k_dev, v_dev
    print("  gpu prune done", flush=True)

    P = layout.num_phys_blocks
    rows = slice(l * S, (l + 1) * S)
    if shared:
        kp = np.zeros((P, B, Hk, D), np.float32)
        vp = np.zeros_like(kp)
        table = i32(layout.block_table[rows, 0]).copy()
        o_lens, o_kept = osh.prefill_prune(k_in, v_in, i32(cu), C, kp, vp, table)
    else:
        kp = np.zeros((P, B, D), np.float32)
        vp = np.zeros_like(kp)
        table = i32(layout.block_table[rows]).copy()
        o_lens, o_kept = oracle.prefill_prune(k_in, v_in, i32(cu), C, kp, vp, table)
    print("  oracle prune done", flush=True)
    gl = eng.per_layer[l]
    assert np.array_equal(gl.seq_lens.cpu().numpy(), o_lens)
    assert o_lens.tolist() == [min(n, C) for n in lens]
    got_kept = kept.cpu().numpy()
    assert np.array_equal(got_kept, o_kept), "kept token indices differ from the oracle"
    # the layer's pages hold exactly the oracle's bytes; the other layer's pages and the spares stay zero
    assert np.array_equal(f32(eng.folded.k_pool).view(np.int32), kp.view(np.int32))
    assert np.array_equal(f32(eng.folded.v_pool).view(np.int32), vp.view(np.int32))
    assert np.array_equal(gl.block_table.cpu().numpy(), table), "the prune must not touch the table"
    # the other layer's lengths are untouched
    assert int(eng.per_layer[0].seq_lens.abs().sum()) == 0
