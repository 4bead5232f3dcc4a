"""GPU parity of the head-shared layout (one table row and one decision per sequence, pages [B, Hk, D]) against
its oracle: every call on its own, then the decode loop step by step.  Bars as for the per-head layout."""
import numpy as np
import pytest
import torch

from oracle import shared as osh
from paper_2509_04377_amd import binding as pe
from paper_2509_04377_amd import synth
from paper_2509_04377_amd.engine import PagedCache

from _util import f32, i32, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda"
DTYPES = {"f32": torch.float32, "bf16": torch.bfloat16}
TOL = {"f32": 1e-5, "bf16": 2e-2}
SEED = 4377


def _ulp(a, b):
    return np.abs(a.view(np.int32).astype(np.int64) - b.view(np.int32).astype(np.int64))


def make_shared(seed, lens, Hk, D, B, dtype, extra=1, pad=3):
    g = torch.Generator().manual_seed(seed)
    S = len(lens)
    nb = [(L + B - 1) // B for L in lens]
    mb = max(max(nb), 1) + extra
    P = sum(nb) + pad
    ids = torch.randperm(P, generator=g).to(torch.int32)
    table = torch.full((S, mb), -1, dtype=torch.int32)
    pos = 0
    for s in range(S):
        table[s, :nb[s]] = ids[pos:pos + nb[s]]
        pos += nb[s]
    k = (torch.randn((P, B, Hk, D), generator=g) * torch.exp(0.5 * torch.randn((P, B, Hk, 1), generator=g))).to(dtype)
    v = (torch.randn((P, B, Hk, D), generator=g) * torch.exp(0.5 * torch.randn((P, B, Hk, 1), generator=g))).to(dtype)
    return k, v, table, torch.tensor(lens, dtype=torch.int32)


def _desc(dtype, S, Hk, Hq, D, B, mb, P):
    return pe.make_desc(dtype, S, Hk, Hq, D, B, mb, P, pe.PE_LAYOUT_SHARED)


@pytest.mark.parametrize("dt,D,B,Hk", [("bf16", 128, 16, 8), ("f32", 64, 32, 3), ("bf16", 64, 64, 2), ("f32", 128, 16, 1),
                                       ("bf16", 128, 128, 5)])
def test_shared_scores(dt, D, B, Hk):
    print("case shared scores", dt, D, B, Hk, flush=True)
    lens = [37 * B, 20 * B + 5, 0, B, 16 * B]
    k, v, table, sl = make_shared(100 + D + B, lens, Hk, D, B, DTYPES[dt], extra=2)
    S, mb = table.shape
    want, _ = osh.score_blocks(f32(k), f32(v), i32(table), i32(sl))
    got = torch.full((S, Hk, mb), -123.0, dtype=torch.float32, device=DEV)
    pe.pe_score_blocks(_desc(DTYPES[dt], S, Hk, Hk, D, B, mb, k.shape[0]), k.to(DEV), v.to(DEV), table.to(DEV),
                       sl.to(DEV), got)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert np.array_equal(np.isinf(got), np.isinf(want))
    fin = np.isfinite(want)
    ulp = _ulp(got[fin], want[fin])
    assert ulp.max() <= 1 and (ulp != 0).mean() < 1e-3


@pytest.mark.parametrize("policy,pf,pl,cached", [(0, 0, 0, False), (0, 1, 2, True), (1, 2, 0, False), (0, 0, 0, True)])
def test_shared_evict_bit_exact(policy, pf, pl, cached):
    print("case shared evict", policy, pf, pl, cached, flush=True)
    rng = np.random.default_rng(300)
    B, Hk, mb = 16, 5, 301
    n_pages = [1, 2, 63, 64, 65, 128, 129, 300, 7, 40, 256, 0]
    S = len(n_pages)
    lens = np.array([n * B for n in n_pages], np.int32)
    lens[8] -= 3
    C = 2 * B
    scores = (rng.integers(0, 6, size=(S, Hk, mb)) * 0.25).astype(np.float32)
    table = np.full((S, mb), -1, np.int32)
    ids = rng.permutation(S * mb).astype(np.int32)
    for s in range(S):
        n = (lens[s] + B - 1) // B
        table[s, :n] = ids[s * mb:s * mb + n]
    desc = _desc(torch.float32, S, Hk, Hk, 64, B, mb, S * mb)
    t_gpu, l_gpu = torch.tensor(table, device=DEV), torch.tensor(lens, device=DEV)
    sc_gpu = torch.tensor(scores, device=DEV)
    ev_gpu = torch.full((S,), -7, dtype=torch.int32, device=DEV)
    fr_gpu = torch.full((S,), -7, dtype=torch.int32, device=DEV)
    opts = pe.pe_evict_opts(policy, pf, pl, 0, int(cached))
    for call in range(3):
        n_before = lens // B
        ev, fr = osh.evict_blocks(scores, table, lens, B, C, policy, pf, pl)
        if cached:   # the kept score rows lose the evicted entry, as the table does (entries past the row stay)
            for s in range(S):
                if ev[s] >= 0:
                    n = n_before[s]
                    scores[s, :, ev[s]:n - 1] = scores[s, :, ev[s] + 1:n]
                    scores[s, :, n - 1] = np.inf
        else:
            sc_gpu.copy_(torch.tensor(scores))
        pe.pe_evict_blocks_ex(desc, opts, sc_gpu, t_gpu, l_gpu, C, ev_gpu, fr_gpu)
        torch.cuda.synchronize()
        assert np.array_equal(ev_gpu.cpu().numpy(), ev), call
        assert np.array_equal(fr_gpu.cpu().numpy(), fr), call
        assert np.array_equal(t_gpu.cpu().numpy(), table), call
        assert np.array_equal(l_gpu.cpu().numpy(), lens), call
        if cached:
            assert np.array_equal(sc_gpu.cpu().numpy().view(np.int32), scores.view(np.int32)), call
    assert (ev >= 0).any() and (ev < 0).any()


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("D,B,Hk,G", [(64, 16, 2, 1), (128, 16, 8, 4), (64, 32, 3, 2), (128, 32, 2, 3), (128, 64, 4, 8),
                                      (64, 128, 1, 6)])
def test_shared_paged_decode(dt, D, B, Hk, G):
    print("case shared paged_decode", dt, D, B, Hk, G, flush=True)
    lens = [0, 1, 15, 16, 17, 100, 700, 1300]
    k, v, table, sl = make_shared(400 + D + B + G, lens, Hk, D, B, DTYPES[dt])
    g = torch.Generator().manual_seed(401)
    S, Hq = len(lens), Hk * G
    q = torch.randn((S, Hq, D), generator=g).to(DTYPES[dt])
    want = osh.paged_decode(f32(q), f32(k), f32(v), i32(table), i32(sl))
    desc = _desc(DTYPES[dt], S, Hk, Hq, D, B, table.shape[1], k.shape[0])
    kd, vd, td, ld, qd = (x.to(DEV) for x in (k, v, table, sl, q))
    try:
        for splits in (0, 1, 3, 8):
            desc.decode_splits = splits
            ws = pe.alloc_workspace(pe.PE_OP_PAGED_DECODE, desc)
            out = torch.full((S, Hq, D), 7.0, dtype=DTYPES[dt], device=DEV)
            pe.pe_paged_decode(desc, qd, kd, vd, td, ld, D ** -0.5, out, ws)
            torch.cuda.synchronize()
            got = f32(out)
            assert np.all(got[0] == 0.0)
            e2, emax = rel_err(got[1:], want[1:])
            assert e2 <= TOL[dt] and emax <= TOL[dt], (splits, e2, emax)
    finally:
        desc.decode_splits = 0


@pytest.mark.parametrize("dt,D,B,Hk", [("bf16", 128, 16, 8), ("f32", 64, 32, 3), ("f32", 128, 16, 8)])
def test_shared_append(dt, D, B, Hk):
    print("case shared append", dt, D, B, Hk, flush=True)
    lens = [0, 1, B - 1, B, 2 * B, 5 * B + 3]
    k, v, table, sl = make_shared(800 + D + B, lens, Hk, D, B, DTYPES[dt], extra=2, pad=32)
    S, mb = table.shape
    P = k.shape[0]
    n_spare = 3
    used_pages = set(int(x) for x in table.flatten() if x >= 0)
    free = [p for p in range(P) if p not in used_pages]
    spare = torch.tensor(free[:S * n_spare], dtype=torch.int32).reshape(S, n_spare)
    freed = torch.full((S,), -1, dtype=torch.int32)
    freed[3] = free[S * n_spare]            # sequence 3 sits at a page boundary and holds a freed page
    used = torch.zeros((S,), dtype=torch.int32)
    desc = _desc(DTYPES[dt], S, Hk, Hk, D, B, mb, P)
    o = dict(k=f32(k).copy(), v=f32(v).copy(), t=i32(table).copy(), l=i32(sl).copy(), f=i32(freed).copy(),
             u=i32(used).copy())
    kd, vd, td, ld, fd, ud, sd = (x.to(DEV) for x in (k, v, table, sl, freed, used, spare))
    g = torch.Generator().manual_seed(801)
    for step in range(3):
        nk = torch.randn((S, Hk, D), generator=g).to(DTYPES[dt]); nv = torch.randn((S, Hk, D), generator=g).to(DTYPES[dt])
        osh.append_kv(f32(nk), f32(nv), o["k"], o["v"], o["t"], o["l"], o["f"], i32(spare), o["u"])
        pe.pe_append_kv(desc, nk.to(DEV), nv.to(DEV), kd, vd, td, ld, fd, sd, ud)
        torch.cuda.synchronize()
        for name, t in (("t", td), ("l", ld), ("f", fd), ("u", ud)):
            assert np.array_equal(t.cpu().numpy(), o[name]), (step, name)
        assert np.array_equal(f32(kd).view(np.int32), o["k"].view(np.int32))
        assert np.array_equal(f32(vd).view(np.int32), o["v"].view(np.int32))


def _prompt(seed, lens, Hk, D, dtype, ties=False):
    g = torch.Generator().manual_seed(seed)
    T = sum(lens)
    k = (torch.randn((T, Hk, D), generator=g) * torch.exp(0.5 * torch.randn((T, Hk, 1), generator=g))).to(dtype)
    v = (torch.randn((T, Hk, D), generator=g) * torch.exp(0.5 * torch.randn((T, Hk, 1), generator=g))).to(dtype)
    if ties:
        src = torch.randint(0, T, (T,), generator=g) % 7
        k, v = k[src].contiguous(), v[src].contiguous()
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32)
    return k, v, cu


@pytest.mark.parametrize("dt,D,Hk,C,B,ties", [("f32", 64, 2, 256, 16, False), ("bf16", 128, 8, 1024, 32, False),
                                             ("bf16", 64, 3, 512, 64, True), ("f32", 128, 8, 256, 16, True)])
def test_shared_prefill_prune(dt, D, Hk, C, B, ties):
    print("case shared prune", dt, D, Hk, C, B, ties, flush=True)
    lens = [1, 100, 1023, 1024, 1025, 3000, 5000, 256]
    S = len(lens)
    k, v, cu = _prompt(600 + D + C, lens, Hk, D, DTYPES[dt], ties)
    need = [(min(L, C) + B - 1) // B for L in lens]
    mb = max(need) + 1
    P = sum(need) + 2
    ids = torch.randperm(P, generator=torch.Generator().manual_seed(601)).to(torch.int32)
    table = torch.full((S, mb), -1, dtype=torch.int32)
    pos = 0
    for s in range(S):
        table[s, :need[s]] = ids[pos:pos + need[s]]
        pos += need[s]
    kp = np.zeros((P, B, Hk, D), np.float32); vp = np.zeros_like(kp)
    o_lens, o_kept = osh.prefill_prune(f32(k), f32(v), i32(cu), C, kp, vp, i32(table))
    desc = _desc(DTYPES[dt], S, Hk, Hk, D, B, mb, P)
    kpd = torch.zeros((P, B, Hk, D), dtype=DTYPES[dt], device=DEV); vpd = torch.zeros_like(kpd)
    lens_d = torch.full((S,), -5, dtype=torch.int32, device=DEV)
    kept_d = torch.full((S, C), -9, dtype=torch.int32, device=DEV)
    ws = pe.alloc_workspace(pe.PE_OP_PREFILL_PRUNE, desc, int(cu[-1]))
    pe.pe_prefill_prune(desc, k.to(DEV), v.to(DEV), cu.to(DEV), int(cu[-1]), max(lens), C, kpd, vpd, table.to(DEV),
                        lens_d, kept_d, ws)
    torch.cuda.synchronize()
    assert np.array_equal(lens_d.cpu().numpy(), o_lens)
    assert np.array_equal(kept_d.cpu().numpy(), o_kept)
    assert np.array_equal(f32(kpd).view(np.int32), kp.view(np.int32))
    assert np.array_equal(f32(vpd).view(np.int32), vp.view(np.int32))


def test_shared_layout_refuses_the_per_head_only_call():
    desc = _desc(torch.bfloat16, 2, 2, 2, 64, 16, 4, 16)
    z = lambda *shape, dt=torch.int32: torch.zeros(shape, dtype=dt, device=DEV)
    kp = z(16, 16, 2, 64, dt=torch.bfloat16)
    with pytest.raises(pe.PeError) as e:
        pe.pe_score_evict(desc, kp, kp, z(2, 4), z(2), 16, None, z(2), z(2))
    assert e.value.status == pe.PE_ERR_UNSUPPORTED


def run_shared_loop(wl, steps, layer=0, cached_scores=False, policy=0, protect_first=0, protect_last=0, fused=True):
    lens = synth.context_lengths(wl, SEED)
    k_in, v_in, cu = synth.prompt_kv(wl, layer, lens, SEED)
    layout = synth.page_layout(wl, lens, SEED, steps=steps, shared=True)
    S, Hk, Hq, D, B = wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim, wl.block_size
    P = layout.num_phys_blocks
    kp = np.zeros((P, B, Hk, D), np.float32); vp = np.zeros_like(kp)
    table = i32(layout.block_table[:, 0]).copy()
    o_lens, o_kept = osh.prefill_prune(f32(k_in), f32(v_in), i32(cu), wl.budget, kp, vp, table)
    oc = osh.SharedOracleCache(kp, vp, table, o_lens, i32(layout.spare[:, 0]).copy(), np.zeros(S, np.int32),
                               np.full(S, -1, np.int32), wl.budget)
    gc = PagedCache.create(wl.torch_dtype, S, Hk, Hq, D, B, layout, wl.budget, DEV, shared=True)
    kept = torch.full((S, wl.budget), -9, dtype=torch.int32, device=DEV)
    gc.prefill_prune(k_in.to(DEV), v_in.to(DEV), cu.to(DEV), max(lens), kept)
    gc.set_host_lens(lens)
    gc.cached_scores = cached_scores
    if policy or protect_first or protect_last:
        gc.evict_opts = pe.pe_evict_opts(policy, protect_first, protect_last, 0, 0)
    torch.cuda.synchronize()
    assert np.array_equal(kept.cpu().numpy(), o_kept)
    assert np.array_equal(f32(gc.k_pool).view(np.int32), kp.view(np.int32))
    out = torch.empty((S, Hq, D), dtype=wl.torch_dtype, device=DEV)
    n_ev = 0
    for step in range(steps):
        nk, nv, q = synth.decode_inputs(wl, layer, step, SEED)
        want, oscores, oev, ofr = osh.decode_step(oc, f32(nk), f32(nv), f32(q), None, policy, protect_first, protect_last)
        gc.evicted_logical.fill_(-1)
        gc.decode_step(nk.to(DEV), nv.to(DEV), q.to(DEV), out, fused=fused)   # fused: the combined C call
        torch.cuda.synchronize()
        where = "step %d" % step
        assert np.array_equal(gc.block_table.cpu().numpy(), oc.block_table), where
        assert np.array_equal(gc.seq_lens.cpu().numpy(), oc.seq_lens), where
        assert np.array_equal(gc.spare_used.cpu().numpy(), oc.spare_used), where
        assert np.array_equal(gc.evicted_logical.cpu().numpy(), oev), where
        n_ev += int((oev >= 0).any())
        e2, emax = rel_err(f32(out), want)
        assert e2 <= TOL[wl.dtype] and emax <= TOL[wl.dtype], (where, e2, emax)
    used = oc.block_table[oc.block_table >= 0]
    assert np.array_equal(f32(gc.k_pool)[used].view(np.int32), kp[used].view(np.int32))
    assert np.array_equal(f32(gc.v_pool)[used].view(np.int32), vp[used].view(np.int32))
    return n_ev


@pytest.mark.parametrize("wl,steps,n_want,kw", [
    (synth.TINY, 40, 3, {}),
    (synth.TINY.with_(num_kv_heads=32, num_q_heads=32, num_seqs=2), 20, 2, {}),      # many heads, no grouping
    (synth.TINY.with_(context=(40,), budget=64), 60, 3, {}),
    (synth.TINY.with_(context=(40,), budget=16, num_seqs=2), 35, 3, {}),             # one-page budget
    (synth.LLAMA32_1B.with_(budget=512, num_seqs=4), 36, 3, {}),
    (synth.LLAMA32_1B.with_(budget=512, num_seqs=4), 36, 3, dict(fused=False)),
    (synth.LLAMA32_1B.with_(budget=512, num_seqs=4), 36, 3, dict(cached_scores=True)),
    (synth.LLAMA32_3B.with_(num_seqs=3), 20, 2, dict(policy=0, protect_first=1, protect_last=2)),
    (synth.LLAMA32_3B.with_(num_seqs=3, block_size=64), 70, 2, dict(cached_scores=True)),
    (synth.LLAMA31_8B.with_(num_seqs=4, budget=1024), 20, 2, dict(policy=1, protect_first=1)),
])
def test_shared_decode_loop(wl, steps, n_want, kw):
    print("case shared loop", wl.name, kw, flush=True)
    assert run_shared_loop(wl, steps, **kw) == n_want


@pytest.mark.parametrize("wl", [synth.LLAMA31_8B, synth.LLAMA32_3B], ids=lambda w: w.name)
def test_shared_full_size_one_layer(wl):
    """A benchmark shape at its full batch and budget in the head-shared layout, through the layered driver
    the benchmark uses (two layers in one pool, layer 1 compared): every per-head score, every decision, the
    table and every attention output against the oracle, for a trigger step and a plain step."""
    from paper_2509_04377_amd.engine import LayeredCache
    print("case shared full size", wl.name, flush=True)
    layers, l = 2, 1
    S, Hk, Hq, D, B, C = wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim, wl.block_size, wl.budget
    lens = [C] * S
    layout = synth.page_layout(wl, lens * layers, SEED, steps=4, shared=True)
    eng = LayeredCache(wl.torch_dtype, layers, S, Hk, Hq, D, B, layout, C, DEV, shared=True)
    cu = torch.tensor(np.arange(S + 1) * C, dtype=torch.int32)
    prompts = []
    for i in range(layers):
        k_in, v_in, _ = synth.prompt_kv(wl, i, lens, SEED)
        eng.prefill_prune_layer(i, k_in.to(DEV), v_in.to(DEV), cu.to(DEV), C)
        prompts.append((k_in, v_in))
    eng.set_host_lens(lens)
    torch.cuda.synchronize()
    P = layout.num_phys_blocks
    kp = np.zeros((P, B, Hk, D), np.float32); vp = np.zeros_like(kp)
    table = i32(layout.block_table[l * S:(l + 1) * S, 0]).copy()
    o_lens, _ = osh.prefill_prune(f32(prompts[l][0]), f32(prompts[l][1]), i32(cu), C, kp, vp, table)
    oc = osh.SharedOracleCache(kp, vp, table, o_lens, i32(layout.spare[l * S:(l + 1) * S, 0]).copy(),
                               np.zeros(S, np.int32), np.full(S, -1, np.int32), C)
    g = torch.Generator().manual_seed(SEED)
    out = torch.empty((layers, S, Hq, D), dtype=wl.torch_dtype, device=DEV)
    for step in range(2):
        nk = torch.randn((layers, S, Hk, D), generator=g).to(wl.torch_dtype)
        nv = torch.randn((layers, S, Hk, D), generator=g).to(wl.torch_dtype)
        q = torch.randn((layers, S, Hq, D), generator=g).to(wl.torch_dtype)
        want, oscores, oev, _ = osh.decode_step(oc, f32(nk[l]), f32(nv[l]), f32(q[l]))
        trig = eng.decode_step(nk.to(DEV), nv.to(DEV), q.to(DEV), out)
        torch.cuda.synchronize()
        gl = eng.per_layer[l]
        assert trig == (step == 0)
        assert np.array_equal(gl.block_table.cpu().numpy(), oc.block_table)
        assert np.array_equal(gl.seq_lens.cpu().numpy(), oc.seq_lens)
        if trig:
            assert np.array_equal(gl.evicted_logical.cpu().numpy(), oev)
            gs = gl.scores.cpu().numpy()
            fin = np.isfinite(oscores)
            assert np.array_equal(np.isinf(gs), np.isinf(oscores)) and _ulp(gs[fin], oscores[fin]).max() <= 1
        e2, emax = rel_err(f32(out[l]), want)
        print("shared full size step %d attention error %.3g %.3g" % (step, e2, emax), flush=True)
        assert e2 <= TOL[wl.dtype] and emax <= TOL[wl.dtype]
