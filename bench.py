#!/usr/bin/env python3
"""Decode throughput of the PagedEviction hot path (score + evict + paged attention) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama31_8b]

A step is one decode iteration of ALL layers over the whole batch: on steps where the newest page of
the sequences has just filled at budget, one block-score sweep and one eviction over all layers (layers
folded into the sequence dimension), then per layer the append of the new token and the paged attention,
back to back on one stream.  K/V pools, tables and the per-step inputs are resident in HBM before the
timed region.  Prints ONE JSON line: tokens/s of the whole job, the roofline object of the attention kernel
(algorithmic bytes per launch over its measured launch time, against 8 TB/s) and the CPU oracle's rate.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
SHAPE_NAMES = {"llama31_8b": "Llama-3.1-8B", "llama32_1b": "Llama-3.2-1B", "llama32_3b": "Llama-3.2-3B",
               "llama31_8b_long": "Llama-3.1-8B long-context"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="llama31_8b")
    ap.add_argument("--budget", type=int, default=None)
    ap.add_argument("--block-size", type=int, default=None, help="override the page size (16, 32, 64, 128)")
    ap.add_argument("--q-heads", type=int, default=None, help="override the number of query heads (group size probe)")
    ap.add_argument("--seed", type=int, default=2509)
    ap.add_argument("--splits", type=int, default=None, help="override the split count of pe_paged_decode")
    ap.add_argument("--xcd-map", type=int, default=None, choices=(0, 1))
    ap.add_argument("--waves", type=int, default=None)
    ap.add_argument("--depth", type=int, default=None)
    ap.add_argument("--loads", type=int, default=None)
    ap.add_argument("--sample-every", type=int, default=8, help="time the attention launches of every n-th step")
    ap.add_argument("--unfused", action="store_true", help="separate append and attention launches per layer")
    ap.add_argument("--cached-scores", action="store_true",
                    help="keep page scores across steps and score only newly filled pages (not the paper's stated "
                         "procedure; the score sweep then drops out of the byte count too)")
    ap.add_argument("--fused-evict", action="store_true",
                    help="score + evict of a trigger step in one launch (pe_score_evict)")
    ap.add_argument("--layout", choices=("per_head", "shared"), default="per_head",
                    help="shared: one block-table row and one eviction decision per sequence, pages [B, Hk, D] "
                         "(separate append and attention launches)")
    ap.add_argument("--stagger", action="store_true",
                    help="prompts of budget - (s mod B) tokens instead of the workload's: sequences reach their page "
                         "boundaries at different steps, as in a serving batch (the prefill prune is then a plain copy)")
    ap.add_argument("--graph", action="store_true", help="replay each step from captured HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-breakdown", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=16)
    ap.add_argument("--cpu-layers", type=int, default=2)
    ap.add_argument("--cpu-steps", type=int, default=33)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference dispatch for rocprofv3 --pmc scaling)")
    return ap.parse_args()


def traffic_from_profiles(workload):
    """HBM bytes per attention launch measured with rocprofv3 --pmc, if a summary is committed."""
    if workload is None:
        return None
    path = os.path.join(ROOT, "profiles", "paged_decode_%s_pmc.md" % workload)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def build_engine(wl, seed, dev, shared=False, stagger=False, decode_opts=None):
    import torch
    from paper_2509_04377_amd import binding as pe
    from paper_2509_04377_amd import synth
    from paper_2509_04377_amd.engine import LayeredCache

    lens = synth.context_lengths(wl, seed)
    if stagger:   # just under the budget, a different distance for every sequence: page boundaries never line up
        lens = [wl.budget - (s % wl.block_size) for s in range(wl.num_seqs)]
    layout = synth.page_layout(wl, lens * wl.layers, seed, shared=shared)
    eng = LayeredCache(wl.torch_dtype, wl.layers, wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim,
                       wl.block_size, layout, wl.budget, dev, shared=shared, decode_opts=decode_opts)
    total = sum(lens)
    ws = pe.alloc_workspace(pe.PE_OP_PREFILL_PRUNE, eng.per_layer[0].desc, total, device=dev)
    prune_ms = []
    for l in range(wl.layers):
        k_in, v_in, cu = synth.prompt_kv(wl, l, lens, seed, device=dev)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        eng.prefill_prune_layer(l, k_in, v_in, cu, max(lens), None, ws)
        torch.cuda.synchronize()
        prune_ms.append((time.perf_counter() - t0) * 1e3)
        del k_in, v_in
    eng.set_host_lens(lens)
    elem = 2 if wl.dtype == "bf16" else 4
    prune_bytes = 2 * total * wl.num_kv_heads * wl.head_dim * elem      # K and V sweep of one layer
    return eng, lens, prune_ms, prune_bytes


def cpu_baseline(wl, seed, n_seqs, n_layers, steps):
    """The oracle, as it stands, on a bounded sample of the same workload: `n_seqs` sequences of `n_layers`
    layers, prune (untimed) then `steps` decode steps (timed).  Scaled to whole-model tokens/s."""
    import numpy as np
    import torch
    import oracle
    from oracle.decode_loop import OracleCache, decode_step
    from paper_2509_04377_amd import synth

    sub = wl.with_(num_seqs=min(n_seqs, wl.num_seqs))
    lens = synth.context_lengths(sub, seed)
    S, Hk, B, D = sub.num_seqs, sub.num_kv_heads, sub.block_size, sub.head_dim

    def np32(t):
        return t.to(torch.float32).contiguous().numpy()

    caches = []
    for l in range(n_layers):
        k_in, v_in, cu = synth.prompt_kv(sub, l, lens, seed)
        layout = synth.page_layout(sub, lens, seed, steps=steps)
        kp = np.zeros((layout.num_phys_blocks, B, D), np.float32)
        vp = np.zeros_like(kp)
        table = layout.block_table.numpy().copy()
        o_lens, _ = oracle.prefill_prune(np32(k_in), np32(v_in), cu.numpy(), sub.budget, kp, vp, table)
        caches.append(OracleCache(kp, vp, table, o_lens, layout.spare.numpy().copy(), np.zeros((S, Hk), np.int32),
                                  np.full((S, Hk), -1, np.int32), sub.budget))
        del k_in, v_in
    inputs = [[tuple(np32(x) for x in synth.decode_inputs(sub, l, st, seed)) for l in range(n_layers)]
              for st in range(steps)]
    t0 = time.perf_counter()
    for st in range(steps):
        for l in range(n_layers):
            nk, nv, q = inputs[st][l]
            decode_step(caches[l], nk, nv, q)
    dt = time.perf_counter() - t0
    per_layer_step = dt / (steps * n_layers)                  # one layer, S sequences, one step
    tokens_per_s = S / (per_layer_step * wl.layers)
    return {"value": tokens_per_s, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d of %d sequences x %d of %d layers x %d consecutive decode steps from the pruned state "
                      "(an eviction every %d steps, the first at step 1), %.1f s wall; scaled to all layers"
                      % (S, wl.num_seqs, n_layers, wl.layers, steps, wl.block_size, dt),
            "ms_per_layer_step": per_layer_step * 1e3}


def kernel_breakdown(eng, wl, new_k, new_v, q, out):
    """Every kernel of the path on its own, after the timed region (not part of `value`): the loop is advanced to
    the next trigger step, which is then issued call by call (score, evict, then per layer append and attention
    as separate launches) with an event after each call."""
    import torch

    L, S, Hk, D, B = wl.layers, wl.num_seqs, wl.num_kv_heads, wl.head_dim, wl.block_size
    elem = 2 if wl.dtype == "bf16" else 4
    guard = 0
    while not any(eng._triggers()):
        eng.decode_step(new_k, new_v, q, out)
        guard += 1
        if guard > 4 * B + wl.budget:
            return None
    trig = eng._triggers()
    f = eng.folded

    def ev():
        e = torch.cuda.Event(enable_timing=True)
        e.record()
        return e

    full_pages = sum(n // B for n in eng.host_lens)
    torch.cuda.synchronize()
    e0 = ev()
    f.score_blocks()
    e1 = ev()
    f.evict_blocks()
    e2 = ev()
    eng.host_lens = [n - B if t else n for n, t in zip(eng.host_lens, trig)]
    marks = []
    for l, c in enumerate(eng.per_layer):
        a = ev()
        c.append_kv(new_k[l], new_v[l])
        b = ev()
        c.paged_decode(q[l], out[l])
        marks.append((a, b, ev()))
    eng.host_lens = [n + 1 for n in eng.host_lens]
    torch.cuda.synchronize()
    score_us = e0.elapsed_time(e1) * 1e3
    score_bytes = L * Hk * full_pages * B * D * 2 * elem
    app = sorted(a.elapsed_time(b) * 1e3 for a, b, _ in marks)
    att = sorted(b.elapsed_time(c_) * 1e3 for _, b, c_ in marks)
    att_bytes = sum(eng.host_lens) * Hk * D * 2 * elem
    med = lambda v: v[len(v) // 2]
    return {"note": "one trigger step issued call by call after the timed region; event-to-event times, each "
                    "includes its launch gap",
            "score_blocks": {"us": score_us, "bytes": score_bytes, "GBps": score_bytes / score_us / 1e3,
                             "frac_of_hbm_peak": score_bytes / score_us / 1e3 / HBM_PEAK_GBS},
            "evict_blocks": {"us": e1.elapsed_time(e2) * 1e3, "rows": L * S * Hk},
            "append_kv": {"us_median_per_layer": med(app)},
            "paged_decode": {"us_median_per_layer": med(att), "bytes": att_bytes,
                             "GBps": att_bytes / med(att) / 1e3,
                             "frac_of_hbm_peak": att_bytes / med(att) / 1e3 / HBM_PEAK_GBS}}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (rows are independent, the path shards with no collective); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2509_04377_amd import binding as pe
    from paper_2509_04377_amd import synth

    wl = synth.WORKLOADS[args.workload]
    if args.budget is not None:
        wl = wl.with_(budget=args.budget)
    if args.block_size is not None:
        wl = wl.with_(block_size=args.block_size)
    if args.q_heads is not None:
        wl = wl.with_(num_q_heads=args.q_heads)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    decode_opts = {}
    if args.splits is not None:
        decode_opts["decode_splits"] = args.splits
    if args.xcd_map is not None:
        decode_opts["decode_flat_order"] = 1 - args.xcd_map
    if args.waves is not None or args.depth is not None or args.loads is not None:
        decode_opts["decode_shape"] = (args.waves or 4) * 100 + (args.depth or 2) * 10 + (args.loads or 2)

    shared = args.layout == "shared"
    # the committed counter summary covers the workload as defined, in the per-head layout; any override of the
    # shape changes the bytes, so no measured traffic is quoted then
    overridden = any(v is not None for v in (args.budget, args.block_size, args.q_heads)) or args.stagger
    profile_key = None if overridden else wl.name + ("_shared" if shared else "")
    eng, lens, prune_ms, prune_bytes = build_engine(wl, args.seed, dev, shared, args.stagger, decode_opts)
    # shared layout: the combined call is two launches inside the library; issue them separately here so that the
    # events bracket the attention kernel alone
    eng.fused = not args.unfused and not shared
    eng.folded.cached_scores = args.cached_scores
    eng.folded.fused_evict = args.fused_evict
    L, S, Hk, Hq, D = wl.layers, wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim
    elem = 2 if wl.dtype == "bf16" else 4

    # a short ring of per-step inputs, resident before the timed region
    ring = 4
    g = torch.Generator(device=dev)
    g.manual_seed(args.seed + 99)
    new_k = (torch.randn((ring, L, S, Hk, D), generator=g, device=dev) *
             torch.exp(0.5 * torch.randn((ring, L, S, Hk, 1), generator=g, device=dev))).to(wl.torch_dtype)
    new_v = (torch.randn((ring, L, S, Hk, D), generator=g, device=dev) *
             torch.exp(0.5 * torch.randn((ring, L, S, Hk, 1), generator=g, device=dev))).to(wl.torch_dtype)
    q = torch.randn((ring, L, S, Hq, D), generator=g, device=dev).to(wl.torch_dtype)
    out = torch.empty((L, S, Hq, D), dtype=wl.torch_dtype, device=dev)

    stepper = None
    if args.graph:      # fixed input buffers, as a serving loop keeps them; warm-up also captures the graphs
        from paper_2509_04377_amd.engine import GraphedStepper
        stepper = GraphedStepper(eng, new_k[0], new_v[0], q[0], out)
    for st in range(args.warmup):
        if stepper is not None:
            stepper.step()
        else:
            eng.decode_step(new_k[st % ring], new_v[st % ring], q[st % ring], out)
    torch.cuda.synchronize()

    # ---- timed region: exactly --steps steps ---------------------------------------------------------
    # (event_start, event_end, launches between them, algorithmic bytes of those launches).  With the fused
    # append the attention launches of a step run back to back, so one event pair brackets all of them and
    # the event overhead is not charged to each launch; unfused, every attention launch gets its own pair.
    samples = []
    state = {}

    def hook(layer, phase):
        per_launch = (sum(eng.host_lens) + S) * Hk * D * 2 * elem   # host_lens is bumped after the layer loop
        if eng.fused:
            if layer == 0 and phase == 0:
                state["e0"] = torch.cuda.Event(enable_timing=True)
                state["e0"].record()
            elif layer == L - 1 and phase == 1:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                samples.append((state["e0"], e, L, per_launch * L))
        elif phase == 0:
            state["e0"] = torch.cuda.Event(enable_timing=True)
            state["e0"].record()
        else:
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            samples.append((state["e0"], e, 1, per_launch))

    sample_every = min(args.sample_every, args.steps)   # a short run still times the launches of one step
    step_events = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    n_trigger = 0        # steps on which some sequence evicts
    n_trigger_seqs = 0   # sequence-evictions over the timed region (each scores its own pages)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_events[0].record()
    for st in range(args.steps):
        i = (args.warmup + st) % ring
        sampled = sample_every > 0 and st % sample_every == sample_every // 2
        n_trigger_seqs += sum(eng._triggers())
        if stepper is not None:
            trig = stepper.step()
            if sampled and not trig and eng.fused:   # a plain step is L attention launches and nothing else
                samples.append((step_events[st], None, L, (sum(eng.host_lens)) * Hk * D * 2 * elem * L))
        else:
            trig = eng.decode_step(new_k[i], new_v[i], q[i], out, None, hook if sampled else None)
        n_trigger += bool(trig)
        step_events[st + 1].record()
        if samples and samples[-1][1] is None:
            samples[-1] = (samples[-1][0], step_events[st + 1]) + samples[-1][2:]
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # ---------------------------------------------------------------------------------------------------

    step_ms = sorted(step_events[i].elapsed_time(step_events[i + 1]) for i in range(args.steps))
    tokens_per_s = S * args.steps / elapsed
    result = {
        "metric": "decode tokens/s (score+evict+paged attn), %s shape" % SHAPE_NAMES.get(wl.name, wl.name),
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d layers, %d seqs x %d KV heads (%d q heads), head_dim %d, page %d, context %s -> "
                               "budget %d" % (wl.name, L, S, Hk, Hq, D, wl.block_size, "/".join(map(str, wl.context)),
                                              wl.budget),
                   "layout": args.layout, "stagger": args.stagger, "decode_splits": pe.pe_decode_splits(eng.per_layer[0].desc), "fused_append": eng.fused, "cached_scores": args.cached_scores, "fused_evict": args.fused_evict, "hip_graph": args.graph,
                   "trigger_steps": n_trigger, "sequence_evictions": n_trigger_seqs},
        "step_ms": {"p50": step_ms[len(step_ms) // 2], "p99": step_ms[min(len(step_ms) - 1, int(len(step_ms) * 0.99))],
                    "max": step_ms[-1]},
        # host-timed per layer (four launches and a synchronisation), against the K/V bytes the sweep reads
        "prefill_prune": {"ms_per_layer": sorted(prune_ms)[len(prune_ms) // 2],
                          "sweep_GBps": prune_bytes / (sorted(prune_ms)[len(prune_ms) // 2] * 1e-3) / 1e9,
                          "sweep_frac_of_hbm_peak": prune_bytes / (sorted(prune_ms)[len(prune_ms) // 2] * 1e-3) / 1e9
                          / HBM_PEAK_GBS},
    }
    result["roofline"] = None   # stays None when no step could be sampled (graph replay of trigger-only runs)
    if samples:
        n_launch = sum(n for _, _, n, _ in samples)
        avg_dur = sum(a.elapsed_time(b) * 1e-3 for a, b, _, _ in samples) / n_launch
        avg_bytes = sum(nb for _, _, _, nb in samples) / n_launch
        achieved = avg_bytes / avg_dur / 1e9
        result["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": achieved / HBM_PEAK_GBS, "traffic": traffic_from_profiles(profile_key),
                              "kernel": "paged_decode_kernel", "launches_timed": n_launch,
                              "avg_launch_us": avg_dur * 1e6, "algorithmic_bytes_per_launch": avg_bytes}
    # whole-step algorithmic bytes: attention every step + the score sweep on trigger steps
    result["path_GBps"] = None
    if samples:
        mean_cached = avg_bytes                                              # per layer launch
        pages_scored = 1 if args.cached_scores else wl.budget // wl.block_size     # per row per trigger
        score_bytes = L * Hk * pages_scored * wl.block_size * D * 2 * elem          # per evicting sequence
        total_bytes = mean_cached * L * args.steps + score_bytes * n_trigger_seqs
        result["path_GBps"] = total_bytes / elapsed / 1e9
        result["path_frac_of_hbm_peak"] = result["path_GBps"] / HBM_PEAK_GBS

    result["kernels"] = None if (args.graph or args.no_kernel_breakdown) else kernel_breakdown(
        eng, wl, new_k[0], new_v[0], q[0], out)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, args.seed, args.cpu_seqs, args.cpu_layers, args.cpu_steps)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
