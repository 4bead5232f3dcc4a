"""GPU parity of the whole decode loop (prefill prune, then score + evict + append + attention per step)
against the oracle's loop, on the benchmark's workloads: the tiny configuration in full, the Llama-shaped
ones on subsets at their real per-row shape, and the headline shape at full size for one layer in the
launch configuration the benchmark times."""
import numpy as np
import pytest
import torch

import oracle
from oracle import shared as osh
from oracle.decode_loop import decode_step as oracle_step
from paper_2509_04377_amd import binding as pe
from paper_2509_04377_amd import synth
from paper_2509_04377_amd.engine import LayeredCache, PagedCache

from _util import f32, i32, oracle_prefill, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = 2024
TOL = {"f32": 1e-5, "bf16": 2e-2}


def _ulp(a, b):
    return np.abs(a.view(np.int32).astype(np.int64) - b.view(np.int32).astype(np.int64))


def _compare_state(cache_gpu, cache_cpu, where):
    assert np.array_equal(cache_gpu.block_table.cpu().numpy(), cache_cpu.block_table), where
    assert np.array_equal(cache_gpu.seq_lens.cpu().numpy(), cache_cpu.seq_lens), where
    assert np.array_equal(cache_gpu.spare_used.cpu().numpy(), cache_cpu.spare_used), where


def run_loop(wl, steps, layer=0, check_pool=True, fused=True, cached_scores=False, evict_opts=None,
             fused_evict=False):
    """One layer of workload `wl`: prune, then `steps` decode steps on both sides, compared every step."""
    lens = synth.context_lengths(wl, SEED)
    k_in, v_in, cu = synth.prompt_kv(wl, layer, lens, SEED)
    layout = synth.page_layout(wl, lens, SEED, steps=steps)
    ocache, okept, _ = oracle_prefill(wl, lens, k_in, v_in, cu, layout, wl.budget)

    S, Hk, Hq, D, B = wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim, wl.block_size
    gcache = PagedCache.create(wl.torch_dtype, S, Hk, Hq, D, B, layout, wl.budget, DEV)
    kept = torch.full((S, Hk, wl.budget), -9, dtype=torch.int32, device=DEV)
    gcache.prefill_prune(k_in.to(DEV), v_in.to(DEV), cu.to(DEV), max(lens), kept)
    gcache.set_host_lens(lens)
    gcache.cached_scores = cached_scores
    gcache.fused_evict = fused_evict  # decisions only: the one-pass form is not asked for the scores here
    if evict_opts is not None:
        gcache.evict_opts = pe.pe_evict_opts(evict_opts.get("policy", 0), evict_opts.get("protect_first", 0),
                                             evict_opts.get("protect_last", 0), int(evict_opts.get("share_heads", False)), 0)
    torch.cuda.synchronize()
    assert np.array_equal(kept.cpu().numpy(), okept)
    _compare_state(gcache, ocache, "after prune")
    if check_pool:
        assert np.array_equal(f32(gcache.k_pool).view(np.int32), ocache.k_pool.view(np.int32))
        assert np.array_equal(f32(gcache.v_pool).view(np.int32), ocache.v_pool.view(np.int32))

    out = torch.empty((S, Hq, D), dtype=wl.torch_dtype, device=DEV)
    n_evictions, worst = 0, (0.0, 0.0)
    for step in range(steps):
        nk, nv, q = synth.decode_inputs(wl, layer, step, SEED)
        triggered = gcache.any_trigger()
        want, oscores, oev, ofr = oracle_step(ocache, f32(nk), f32(nv), f32(q), evict_opts=evict_opts)
        gcache.evicted_logical.fill_(-1)
        gcache.decode_step(nk.to(DEV), nv.to(DEV), q.to(DEV), out, fused=fused)
        torch.cuda.synchronize()
        where = "step %d" % step
        _compare_state(gcache, ocache, where)
        assert np.array_equal(gcache.evicted_logical.cpu().numpy(), oev), where
        assert (oev >= 0).any() == triggered, where
        if triggered:
            n_evictions += 1
        if triggered and oscores is not None and not fused_evict:
            gs = gcache.scores.cpu().numpy()
            if cached_scores:   # the kept array has already lost the evicted entry of every row that evicted
                want_sc = oscores.copy()
                for s_ in range(S):
                    for h_ in range(Hk):
                        j = oev[s_, h_]
                        if j >= 0:
                            want_sc[s_, h_, j:-1] = oscores[s_, h_, j + 1:]
                            want_sc[s_, h_, -1] = np.inf
                oscores = want_sc
            if not cached_scores:   # only the sequences that evict at this step are scored (Alg. 3)
                rows = (oev >= 0).any(axis=1)
                gs, oscores = gs[rows], oscores[rows]
            assert np.array_equal(np.isinf(gs), np.isinf(oscores)), where
            fin = np.isfinite(oscores)
            assert _ulp(gs[fin], oscores[fin]).max() <= 1, where
        e2, emax = rel_err(f32(out), want)
        worst = (max(worst[0], e2), max(worst[1], emax))
        assert e2 <= TOL[wl.dtype] and emax <= TOL[wl.dtype], (where, e2, emax)
    assert gcache.host_lens == [int(x) for x in ocache.seq_lens]
    if check_pool:
        used = ocache.block_table[ocache.block_table >= 0]
        gk, gv = f32(gcache.k_pool), f32(gcache.v_pool)
        assert np.array_equal(gk[used].view(np.int32), ocache.k_pool[used].view(np.int32))
        assert np.array_equal(gv[used].view(np.int32), ocache.v_pool[used].view(np.int32))
    return n_evictions, worst


@pytest.mark.parametrize("fused", [True, False])
def test_tiny_full(fused):
    """Configuration 1 in full: 512 -> 256 tokens, 32 steps, evictions at steps 1 and 17; with the append
    fused into the attention launch, and with the separate append + attention calls."""
    print("case loop tiny_f32 fused", fused, flush=True)
    n_ev, worst = run_loop(synth.TINY, synth.TINY.steps, fused=fused)
    assert n_ev == 2
    print("tiny worst attention error", worst, flush=True)


def test_many_kv_heads_without_grouping():
    """32 KV heads, one query head each (more heads than a workgroup has waves, in every kernel that loops
    over the heads of a sequence)."""
    print("case loop many heads", flush=True)
    n_ev, _ = run_loop(synth.TINY.with_(num_kv_heads=32, num_q_heads=32, num_seqs=2), 20)
    assert n_ev == 2


@pytest.mark.parametrize("fused", [True, False])
def test_budget_of_one_page(fused):
    """The smallest budget there is, C = B: every eviction drops the row's only page, the cache restarts from
    the new token alone and the freed page is taken again at once."""
    print("case loop one-page budget", fused, flush=True)
    wl = synth.TINY.with_(context=(40,), budget=16, num_seqs=2)
    n_ev, _ = run_loop(wl, 35, fused=fused)
    assert n_ev == 3          # steps 0, 16, 32


def test_tiny_under_budget_growth():
    print("case loop tiny under budget", flush=True)
    wl = synth.TINY.with_(context=(40,), budget=64)
    n_ev, _ = run_loop(wl, 60)
    assert n_ev == 3


@pytest.mark.parametrize("wl,steps,n_want", [(synth.TINY, 70, 5), (synth.TINY.with_(context=(40,), budget=64), 60, 3),
                                             (synth.LLAMA32_1B.with_(budget=512), 36, 3)])
def test_cached_scores_give_the_same_decisions(wl, steps, n_want):
    """Scores kept across steps (only newly filled pages scored, score rows compacted with the table) must
    equal the oracle's full re-scoring at every trigger, and so must every decision."""
    print("case loop cached scores", wl.name, flush=True)
    n_ev, _ = run_loop(wl, steps, cached_scores=True)
    assert n_ev == n_want


@pytest.mark.parametrize("kw", [{}, dict(fused_evict=True), dict(cached_scores=True), dict(fused=False),
                                dict(evict_opts=dict(policy=0, protect_first=1, share_heads=True))])
def test_staggered_triggers(kw):
    """Prompts a little under the budget and of different lengths: the sequences reach the budget, and later
    their page boundaries, at different steps, so most trigger steps evict from only some of them."""
    print("case loop staggered", kw, flush=True)
    wl = synth.LLAMA32_1B.with_(num_seqs=6, context=(470, 512), budget=512)
    lens = synth.context_lengths(wl, SEED)
    assert len(set(L % wl.block_size for L in lens)) >= 4
    n_ev, _ = run_loop(wl, 60, **kw)
    assert n_ev >= 8          # many more trigger steps than the 4 a lockstep batch would see in 60 steps


@pytest.mark.parametrize("B,kw", [(64, {}), (128, {}), (64, dict(fused_evict=True)), (64, dict(cached_scores=True)),
                                  (128, dict(cached_scores=True, fused=False))])
def test_larger_pages(B, kw):
    """Pages of 64 and 128 tokens (the method is stated for any page size): the whole loop against the oracle."""
    print("case loop larger pages", B, kw, flush=True)
    wl = synth.LLAMA32_1B.with_(block_size=B, budget=1024, num_seqs=4)
    n_ev, _ = run_loop(wl, 2 * B + 3, **kw)
    assert n_ev == 3


@pytest.mark.parametrize("wl,steps,n_want", [(synth.TINY, 70, 5), (synth.LLAMA32_1B.with_(budget=512), 36, 3),
                                             (synth.LLAMA31_8B.with_(num_seqs=6, budget=1024), 20, 2)])
def test_score_and_evict_in_one_launch(wl, steps, n_want):
    """pe_score_evict in place of pe_score_blocks + pe_evict_blocks: same tables, lengths, evicted pages and
    attention outputs as the oracle at every step."""
    print("case loop fused score+evict", wl.name, flush=True)
    n_ev, _ = run_loop(wl, steps, fused_evict=True, check_pool=wl.num_seqs <= 8)
    assert n_ev == n_want


@pytest.mark.parametrize("opts", [dict(policy=1, protect_first=1), dict(policy=0, protect_first=1, protect_last=2),
                                  dict(policy=0, share_heads=True), dict(policy=1)])
def test_eviction_variants_loop(opts):
    """Sliding window with a sink page, protected first/last pages, one decision per sequence: the whole
    loop against the oracle's loop with the same variant, tables bit-exact at every step."""
    print("case loop variants", opts, flush=True)
    n_ev, _ = run_loop(synth.TINY.with_(num_seqs=2), 40, evict_opts=opts)
    assert n_ev == 3


def test_tiny_full_cache_never_evicts():
    print("case loop tiny full cache", flush=True)
    wl = synth.TINY.with_(budget=1024)
    n_ev, _ = run_loop(wl, 32)
    assert n_ev == 0


@pytest.mark.parametrize("budget", [512, 1024, 2048])
def test_llama32_1b_subset(budget):
    """Configuration 2 shape (bf16, D=64, G=4), all 8 sequences of one layer, 36 steps (3 evictions)."""
    print("case loop llama32_1b budget", budget, flush=True)
    wl = synth.LLAMA32_1B.with_(budget=budget)
    n_ev, worst = run_loop(wl, 36)
    assert n_ev == 3
    print("1b worst attention error", worst, flush=True)


def test_llama32_3b_subset():
    """Configuration 3 shape (bf16, D=128, G=3, ragged prompts, sink tokens): 5 sequences, 20 steps."""
    print("case loop llama32_3b", flush=True)
    wl = synth.LLAMA32_3B.with_(num_seqs=5)
    n_ev, worst = run_loop(wl, 20, check_pool=False)
    assert n_ev == 2
    print("3b worst attention error", worst, flush=True)


def test_llama31_8b_subset():
    """Configuration 4 shape (bf16, D=128, G=4, shuffled shared pool): 3 sequences, 20 steps."""
    print("case loop llama31_8b", flush=True)
    wl = synth.LLAMA31_8B.with_(num_seqs=3)
    n_ev, worst = run_loop(wl, 20, check_pool=False)
    assert n_ev == 2
    print("8b worst attention error", worst, flush=True)
    n_ev, worst = run_loop(wl, 18, check_pool=False, fused=False)
    assert n_ev == 2


@pytest.mark.parametrize("B,C,L", [(16, 4096, 65536), (32, 8192, 65536), (32, 8192, 131072), (16, 4096, 131072)])
def test_long_context_subset(B, C, L):
    """Configuration 5 shape: one 65536- or 131072-token prompt (the largest), budgets 4096 / 8192, page sizes
    16 / 32: prefill select over a row far larger than LDS, 8 attention splits per row."""
    print("case loop long", B, C, L, flush=True)
    wl = synth.LONG_8B.with_(num_seqs=1, block_size=B, budget=C, context=(L,))
    n_ev, worst = run_loop(wl, B + 2, check_pool=False)
    assert n_ev == 2
    print("long worst attention error", worst, flush=True)


FULL_SIZE = [synth.LLAMA31_8B, synth.LLAMA32_1B, synth.LLAMA32_1B.with_(budget=2048), synth.LLAMA32_3B, synth.LONG_8B,
             synth.LONG_8B.with_(block_size=32, budget=8192)]


@pytest.mark.parametrize("wl", FULL_SIZE, ids=lambda w: "%s_C%d_B%d" % (w.name, w.budget, w.block_size))
def test_full_size_one_layer_and_determinism(wl):
    """Every benchmark shape at its full batch and budget (the headline one: 32 sequences x 8 KV heads x 2048
    tokens, bf16, shuffled pool), one layer of the layered driver the benchmark uses, in the benchmark's launch
    configuration (same split count, fused append): every score, every eviction decision, the whole table and
    every attention output against the oracle, for a trigger step and a plain step; then the same launch
    again from the same state must give identical bytes."""
    print("case full size", wl.name, wl.budget, wl.block_size, flush=True)
    layers = 2                                   # two layers share the pool; layer 1 is compared
    S, Hk, Hq, D, B, C = wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim, wl.block_size, wl.budget
    lens = [C] * S                               # the state right after the prune: every row at budget
    layout = synth.page_layout(wl, lens * layers, SEED, steps=4)
    eng = LayeredCache(wl.torch_dtype, layers, S, Hk, Hq, D, B, layout, C, DEV)
    cu = torch.tensor(np.arange(S + 1) * C, dtype=torch.int32)
    prompts = []
    for l in range(layers):
        k_in, v_in, _ = synth.prompt_kv(wl, l, lens, SEED)
        eng.prefill_prune_layer(l, k_in.to(DEV), v_in.to(DEV), cu.to(DEV), C)
        prompts.append((k_in, v_in))
    eng.set_host_lens(lens)
    torch.cuda.synchronize()
    # oracle state for layer 1 (L == C: the prune is the identity copy)
    l = 1
    lay1 = synth.PageLayout(layout.block_table[l * S:(l + 1) * S], layout.spare[l * S:(l + 1) * S],
                            layout.max_blocks, layout.n_spare, layout.num_phys_blocks)
    ocache, _, _ = oracle_prefill(wl, lens, prompts[l][0], prompts[l][1], cu, lay1, C)
    gl = eng.per_layer[l]
    assert np.array_equal(gl.block_table.cpu().numpy(), ocache.block_table)

    g = torch.Generator().manual_seed(SEED)
    out = torch.empty((layers, S, Hq, D), dtype=wl.torch_dtype, device=DEV)
    for step in range(2):                        # step 0 triggers (len == C), step 1 does not
        nk = torch.randn((layers, S, Hk, D), generator=g).to(wl.torch_dtype)
        nv = torch.randn((layers, S, Hk, D), generator=g).to(wl.torch_dtype)
        q = torch.randn((layers, S, Hq, D), generator=g).to(wl.torch_dtype)
        want, oscores, oev, ofr = oracle_step(ocache, f32(nk[l]), f32(nv[l]), f32(q[l]))
        trig = eng.decode_step(nk.to(DEV), nv.to(DEV), q.to(DEV), out)
        torch.cuda.synchronize()
        gl = eng.per_layer[l]
        assert trig == (step == 0)
        assert np.array_equal(gl.block_table.cpu().numpy(), ocache.block_table)
        assert np.array_equal(gl.seq_lens.cpu().numpy(), ocache.seq_lens)
        if trig:
            assert np.array_equal(gl.evicted_logical.cpu().numpy(), oev)
            gs = gl.scores.cpu().numpy()
            fin = np.isfinite(oscores)
            assert np.array_equal(np.isinf(gs), np.isinf(oscores))
            ulp = _ulp(gs[fin], oscores[fin])
            assert ulp.max() <= 1
            print("full size: %d scores, %d not bit-equal" % (fin.sum(), int((ulp != 0).sum())), flush=True)
        e2, emax = rel_err(f32(out[l]), want)
        print("full size step %d attention error %.3g %.3g" % (step, e2, emax), flush=True)
        assert e2 <= 2e-2 and emax <= 2e-2
    # determinism: the same attention launch twice gives identical bytes; the plain attention call on the
    # post-append state agrees with what the fused append + attention launch produced (same sum, other order)
    qd = q.to(DEV)
    o1 = torch.empty_like(out[l]); o2 = torch.empty_like(out[l])
    gl.paged_decode(qd[l], o1)
    gl.paged_decode(qd[l], o2)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    e2, emax = rel_err(f32(o1), f32(out[l]).astype(np.float64))
    assert e2 <= 2e-2 and emax <= 2e-2


def _oracle_layer_state(wl, lens, k_in, v_in, cu, layout, l, shared):
    """Oracle cache of layer `l` of a layered run: the oracle's own prune of that layer's prompts into pools of
    the shared size, with the layer's slice of the table and of the spare lists."""
    S, Hk, D, B, C = wl.num_seqs, wl.num_kv_heads, wl.head_dim, wl.block_size, wl.budget
    rows = slice(l * S, (l + 1) * S)
    if not shared:
        lay = synth.PageLayout(layout.block_table[rows], layout.spare[rows], layout.max_blocks, layout.n_spare,
                               layout.num_phys_blocks)
        return oracle_prefill(wl, lens, k_in, v_in, cu, lay, C)[0]
    P = layout.num_phys_blocks
    kp = np.zeros((P, B, Hk, D), np.float32)
    vp = np.zeros_like(kp)
    table = i32(layout.block_table[rows, 0]).copy()
    o_lens, _ = osh.prefill_prune(f32(k_in), f32(v_in), i32(cu), C, kp, vp, table)
    return osh.SharedOracleCache(kp, vp, table, o_lens, i32(layout.spare[rows, 0]).copy(), np.zeros(S, np.int32),
                                 np.full(S, -1, np.int32), C)


@pytest.mark.parametrize("shared,stagger", [(False, False), (False, True), (True, False), (True, True)])
def test_all_driver_modes_agree_at_full_size(shared, stagger):
    """The whole headline job (32 layers x 32 sequences x 8 KV heads at budget 2048, one shared shuffled pool)
    stepped 36 times in every mode of the layered driver: the paper's procedure, cached scores, one-pass
    score+evict, separate append launches, HIP-graph replay, the layers' launches issued by one native call or by one
    call per layer.  Every mode must end with the same block tables,
    lengths and spare counters, bit for bit (the decisions are the same decisions), and the same attention
    outputs within the bf16 tolerance (the fused and the separate attention sum in different orders).  Also in
    the head-shared layout (which has no one-pass score+evict), and with prompts just under the budget so that
    the sequences evict at different steps.  In the first mode one layer of the 32 is stepped by the oracle as
    well: its table, lengths, spare counters and attention outputs are compared at every step, so the other
    modes are compared with a run that is itself checked against the oracle."""
    from paper_2509_04377_amd.engine import GraphedStepper
    print("case loop modes agree", shared, stagger, flush=True)
    wl = synth.LLAMA31_8B
    L, S, Hk, Hq, D, B, C = wl.layers, wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim, wl.block_size, wl.budget
    lens = [C - (i % B) for i in range(S)] if stagger else [C] * S
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=DEV)
    steps = 36
    g = torch.Generator(device=DEV)
    g.manual_seed(SEED + 7)
    nk = torch.randn((4, L, S, Hk, D), generator=g, device=DEV).to(wl.torch_dtype)
    nv = torch.randn((4, L, S, Hk, D), generator=g, device=DEV).to(wl.torch_dtype)
    q = torch.randn((4, L, S, Hq, D), generator=g, device=DEV).to(wl.torch_dtype)
    ref = None
    ls = 17          # the layer of the first mode's run that is stepped by the oracle as well
    for mode in ("paper", "cached", "fused_evict", "unfused", "graph", "python_loop"):
        if shared and mode == "fused_evict":
            continue
        layout = synth.page_layout(wl, lens * L, SEED, steps=steps, shared=shared)
        eng = LayeredCache(wl.torch_dtype, L, S, Hk, Hq, D, B, layout, C, DEV, shared=shared)
        ocache = None
        for l in range(L):
            k_in, v_in, _ = synth.prompt_kv(wl, l, lens, SEED, device=DEV)
            eng.prefill_prune_layer(l, k_in, v_in, cu, max(lens))
            if mode == "paper" and l == ls:
                ocache = _oracle_layer_state(wl, lens, k_in, v_in, cu, layout, l, shared)
            del k_in, v_in
        eng.set_host_lens(lens)
        eng.folded.cached_scores = mode == "cached"
        eng.folded.fused_evict = mode == "fused_evict"
        eng.fused = mode != "unfused"
        eng.native_layers = mode != "python_loop"   # one native call per step, or one C-ABI call per layer
        out = torch.zeros((L, S, Hq, D), dtype=wl.torch_dtype, device=DEV)
        n_trig = 0
        if mode == "graph":
            bufs = (nk[0].clone(), nv[0].clone(), q[0].clone())
            stepper = GraphedStepper(eng, bufs[0], bufs[1], bufs[2], out)
        for st in range(steps):
            i = st % 4
            if mode == "graph":
                bufs[0].copy_(nk[i]); bufs[1].copy_(nv[i]); bufs[2].copy_(q[i])
                n_trig += bool(stepper.step())
            else:
                n_trig += bool(eng.decode_step(nk[i], nv[i], q[i], out))
            if ocache is not None:      # the sampled layer against the oracle, every step
                ostep = osh.decode_step if shared else oracle_step
                want = ostep(ocache, f32(nk[i][ls]), f32(nv[i][ls]), f32(q[i][ls]))[0]
                gl = eng.per_layer[ls]
                where = "layer %d step %d" % (ls, st)
                assert np.array_equal(gl.block_table.cpu().numpy(), ocache.block_table), where
                assert np.array_equal(gl.seq_lens.cpu().numpy(), ocache.seq_lens), where
                assert np.array_equal(gl.spare_used.cpu().numpy(), ocache.spare_used), where
                e2, emax = rel_err(f32(out[ls]), want)
                assert e2 <= 2e-2 and emax <= 2e-2, (where, e2, emax)
        torch.cuda.synchronize()
        assert n_trig == (steps if stagger else 3)
        state = (eng.folded.block_table.clone(), eng.folded.seq_lens.clone(), eng.folded.spare_used.clone(),
                 out.float().cpu().numpy())
        if ref is None:
            ref = state
        else:
            assert torch.equal(state[0], ref[0]) and torch.equal(state[1], ref[1]) and torch.equal(state[2], ref[2]), mode
            e2, emax = rel_err(state[3].reshape(-1, D), ref[3].reshape(-1, D).astype(np.float64))
            assert e2 <= 2e-2 and emax <= 2e-2, (mode, e2, emax)
        del eng, layout, out
        torch.cuda.empty_cache()
