#!/usr/bin/env python3
"""Decode throughput of the PagedEviction hot path (score + evict + paged attention) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama31_8b]

A step is one decode iteration of ALL layers over the whole batch: on steps where the newest page of
the sequences has just filled at budget, one block-score sweep and one eviction over all layers (layers
folded into the sequence dimension), then per layer the append of the new token and the paged attention,
back to back on one stream.  K/V pools, tables and the per-step inputs are resident in HBM before the
timed region.  Prints ONE JSON line: tokens/s of the whole job, the roofline object of the attention kernel
(algorithmic bytes per launch over its measured launch time, against 8 TB/s) and the CPU oracle's rate.
The headline workload is timed first; after it every other benchmark configuration (tiny, the 1B shape at its
three budgets, the 3B shape, both long-context corners) is run for a short, whole number of trigger periods and
reported under "configs" in the same line, each with its own attention roofline and its prefill-prune time
(device events).  `--no-configs` skips them.
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
    ap.add_argument("--context", type=int, default=None, help="override the prompt length (one value for all sequences)")
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
                    help="score + evict of a trigger step in one pass over the pages (pe_score_evict)")
    ap.add_argument("--layout", choices=("per_head", "shared"), default="per_head",
                    help="shared: one block-table row and one eviction decision per sequence, pages [B, Hk, D] "
                         "(separate append and attention launches)")
    ap.add_argument("--stagger", action="store_true",
                    help="prompts of budget - (s mod B) tokens instead of the workload's: sequences reach their page "
                         "boundaries at different steps, as in a serving batch (the prefill prune is then a plain copy)")
    ap.add_argument("--graph", action="store_true", help="replay each step from captured HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the short runs of the other configurations")
    ap.add_argument("--no-kernel-breakdown", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=32)
    ap.add_argument("--cpu-layers", type=int, default=4)
    ap.add_argument("--cpu-steps", type=int, default=97)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference dispatch for rocprofv3 --pmc scaling)")
    return ap.parse_args()


def kernel_source_hash():
    """sha256 over the sources that make up the attention kernel; a committed counter summary names the hash of
    the sources it was measured on, and is only quoted while they are unchanged."""
    import hashlib
    h = hashlib.sha256()
    for name in ("paged_decode.hip", "pe_device.h", "pe_launch.h"):
        with open(os.path.join(ROOT, "paper_2509_04377_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def traffic_from_profiles(workload):
    """HBM bytes per attention launch from the committed rocprofv3 --pmc summary of this workload, with where it
    came from.  Not measured in this run: (None, reason) when there is no summary or it was taken on other
    kernel sources."""
    if workload is None:
        return None, "no counter summary for an overridden workload"
    rel = os.path.join("profiles", "paged_decode_%s_pmc.md" % workload)
    val, src_hash = None, None
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch:"):
                val = float(line.split(":")[1])
            if line.startswith("kernel_source_sha256:"):
                src_hash = line.split(":")[1].strip()
    except OSError:
        return None, "no committed counter summary"
    if val is None:
        return None, "no committed counter summary"
    if src_hash != kernel_source_hash():
        return None, "%s was measured on other kernel sources (%s, now %s)" % (rel, src_hash, kernel_source_hash())
    return val, "committed rocprofv3 --pmc summary %s (FETCH_SIZE + WRITE_SIZE, copy-calibrated), not this run" % rel


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
    # one warm-up prune of layer 0 (it is pruned again below), then every layer between two events
    k_in, v_in, cu = synth.prompt_kv(wl, 0, lens, seed, device=dev)
    eng.prefill_prune_layer(0, k_in, v_in, cu, max(lens), None, ws)
    marks = []
    for l in range(wl.layers):
        k_in, v_in, cu = synth.prompt_kv(wl, l, lens, seed, device=dev)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        eng.prefill_prune_layer(l, k_in, v_in, cu, max(lens), None, ws)
        e1.record()
        marks.append((e0, e1))
        del k_in, v_in
    torch.cuda.synchronize()
    prune_ms = sorted(a.elapsed_time(b) for a, b in marks)
    eng.set_host_lens(lens)
    elem = 2 if wl.dtype == "bf16" else 4
    row_bytes = wl.num_kv_heads * wl.head_dim * elem
    kept = sum(min(n, wl.budget) for n in lens)
    # per layer: the K and V sweep of the whole prompt, the gather's reads of the kept rows and its writes
    prune_bytes = {"sweep": 2 * total * row_bytes, "gather_read": 2 * kept * row_bytes,
                   "gather_write": 2 * kept * row_bytes}
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


def workload_label(wl):
    return ("%s: %d layers, %d seqs x %d KV heads (%d q heads), head_dim %d, page %d, context %s -> budget %d"
            % (wl.name, wl.layers, wl.num_seqs, wl.num_kv_heads, wl.num_q_heads, wl.head_dim, wl.block_size,
               "/".join(map(str, wl.context)), wl.budget))


def run_workload(wl, args, dev, steps, warmup, shared=False, stagger=False, decode_opts=None, sample_every=8,
                 breakdown=False, profile_key=None, graph=None):
    """Prune all layers (device-event timed), then `warmup` untimed and exactly `steps` timed decode steps.
    Returns the measurements of this workload as a dict."""
    import torch
    from paper_2509_04377_amd import binding as pe

    graph = args.graph if graph is None else graph
    eng, lens, prune_ms, prune_bytes = build_engine(wl, args.seed, dev, shared, stagger, decode_opts)
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
    if graph:           # fixed input buffers, as a serving loop keeps them; warm-up also captures the graphs
        from paper_2509_04377_amd.engine import GraphedStepper
        stepper = GraphedStepper(eng, new_k[0], new_v[0], q[0], out)
    for st in range(warmup):
        if stepper is not None:
            stepper.step()
        else:
            eng.decode_step(new_k[st % ring], new_v[st % ring], q[st % ring], out)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps -----------------------------------------------------------
    # (event_start, event_end, launches between them, algorithmic bytes of those launches).  With the fused
    # append the attention launches of a step run back to back, so one event pair brackets all of them and
    # the event overhead is not charged to each launch; unfused, every attention launch gets its own pair.
    # A launch is the whole attention call: on split rows the partial kernel and the merge kernel together.
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

    sample_every = min(sample_every, steps)   # a short run still times the launches of one step
    step_events = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    n_trigger = 0        # steps on which some sequence evicts
    n_trigger_seqs = 0   # sequence-evictions over the timed region (each scores its own pages)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_events[0].record()
    for st in range(steps):
        i = (warmup + st) % ring
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

    step_ms = sorted(step_events[i].elapsed_time(step_events[i + 1]) for i in range(steps))
    prune_med = prune_ms[len(prune_ms) // 2]
    moved = sum(prune_bytes.values())
    r = {
        "tokens_per_s": S * steps / elapsed, "ms_per_step": elapsed / steps * 1e3, "steps": steps, "warmup": warmup,
        "step_ms": {"p50": step_ms[len(step_ms) // 2], "p99": step_ms[min(len(step_ms) - 1, int(len(step_ms) * 0.99))],
                    "max": step_ms[-1]},
        "decode_splits": pe.pe_decode_splits(eng.per_layer[0].desc), "fused_append": eng.fused,
        "trigger_steps": n_trigger, "sequence_evictions": n_trigger_seqs,
        # device events around the four launches of each layer's prune; bytes: the K/V sweep of the whole prompt
        # plus the gather's reads and writes of the kept rows
        "prefill_prune": {"ms_per_layer": prune_med, "timing": "HIP events, median over layers",
                          "bytes_per_layer": prune_bytes, "GBps": moved / (prune_med * 1e-3) / 1e9,
                          "frac_of_hbm_peak": moved / (prune_med * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "sweep_GBps": prune_bytes["sweep"] / (prune_med * 1e-3) / 1e9},
        "roofline": None,   # stays None when no step could be sampled (graph replay of trigger-only runs)
        "path_GBps": None,
    }
    if samples:
        n_launch = sum(n for _, _, n, _ in samples)
        avg_dur = sum(a.elapsed_time(b) * 1e-3 for a, b, _, _ in samples) / n_launch
        avg_bytes = sum(nb for _, _, _, nb in samples) / n_launch
        achieved = avg_bytes / avg_dur / 1e9
        traffic, traffic_source = traffic_from_profiles(profile_key)
        r["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                         "kernel": "paged_decode_kernel" + (" + paged_decode_reduce_kernel" if r["decode_splits"] > 1
                                                            else ""),
                         "launches_timed": n_launch, "avg_launch_us": avg_dur * 1e6,
                         "algorithmic_bytes_per_launch": avg_bytes}
        # whole-step algorithmic bytes: attention every step + the score sweep on trigger steps
        pages_scored = 1 if args.cached_scores else wl.budget // wl.block_size     # per row per trigger
        score_bytes = L * Hk * pages_scored * wl.block_size * D * 2 * elem          # per evicting sequence
        total_bytes = avg_bytes * L * steps + score_bytes * n_trigger_seqs
        r["path_GBps"] = total_bytes / elapsed / 1e9
        r["path_frac_of_hbm_peak"] = r["path_GBps"] / HBM_PEAK_GBS
    r["kernels"] = kernel_breakdown(eng, wl, new_k[0], new_v[0], q[0], out) if breakdown else None
    del eng, new_k, new_v, q, out
    torch.cuda.empty_cache()
    return r


def other_configs(synth):
    """The benchmark configurations besides the headline one, each for a whole number of trigger periods."""
    long_ = synth.LONG_8B
    return [("tiny_f32", synth.TINY, 32),
            ("llama32_1b_C512", synth.LLAMA32_1B.with_(budget=512), 64),
            ("llama32_1b_C1024", synth.LLAMA32_1B, 64),
            ("llama32_1b_C2048", synth.LLAMA32_1B.with_(budget=2048), 64),
            ("llama32_3b", synth.LLAMA32_3B, 64),
            ("llama31_8b_long_L65536_B16_C4096", long_, 64),
            ("llama31_8b_long_L131072_B32_C8192", long_.with_(context=(131072,), block_size=32, budget=8192), 64)]


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (rows are independent, the path shards with no collective); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2509_04377_amd import synth

    wl = synth.WORKLOADS[args.workload]
    if args.budget is not None:
        wl = wl.with_(budget=args.budget)
    if args.block_size is not None:
        wl = wl.with_(block_size=args.block_size)
    if args.context is not None:
        wl = wl.with_(context=(args.context,))
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
    overridden = any(v is not None for v in (args.budget, args.block_size, args.q_heads, args.context)) or args.stagger
    profile_key = None if overridden else wl.name + ("_shared" if shared else "")
    m = run_workload(wl, args, dev, args.steps, args.warmup, shared, args.stagger, decode_opts, args.sample_every,
                     breakdown=not (args.graph or args.no_kernel_breakdown), profile_key=profile_key)
    result = {
        "metric": "decode tokens/s (score+evict+paged attn), %s shape" % SHAPE_NAMES.get(wl.name, wl.name),
        "value": m["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": workload_label(wl), "layout": args.layout, "stagger": args.stagger,
                   "decode_splits": m["decode_splits"], "fused_append": m["fused_append"],
                   "cached_scores": args.cached_scores, "fused_evict": args.fused_evict, "hip_graph": args.graph,
                   "trigger_steps": m["trigger_steps"], "sequence_evictions": m["sequence_evictions"]},
        "step_ms": m["step_ms"], "prefill_prune": m["prefill_prune"], "roofline": m["roofline"],
        "path_GBps": m["path_GBps"], "path_frac_of_hbm_peak": m.get("path_frac_of_hbm_peak"), "kernels": m["kernels"],
    }

    if not args.no_configs:
        # every other configuration, same driver, default launch shape, a whole number of trigger periods
        configs = {}
        for key, cwl, csteps in other_configs(synth):
            try:   # a side configuration that fails is reported as such; it must not take the headline line with it
                cm = run_workload(cwl, args, dev, csteps, cwl.block_size, False, False, None, 4, graph=False)
                # the same steps replayed from captured HIP graphs (no host launch cost at all)
                gm = run_workload(cwl, args, dev, csteps, 2 * cwl.block_size, False, False, None, 4, graph=True)
            except Exception as exc:   # noqa: BLE001
                configs[key] = {"workload": workload_label(cwl), "error": "%s: %s" % (type(exc).__name__, exc)}
                torch.cuda.empty_cache()
                continue
            rf = cm["roofline"] or {}
            configs[key] = {"workload": workload_label(cwl), "dtype": cwl.dtype, "tokens_per_s": cm["tokens_per_s"],
                            "tokens_per_s_hip_graph": gm["tokens_per_s"], "ms_per_step_hip_graph": gm["ms_per_step"],
                            "ms_per_step": cm["ms_per_step"], "step_ms_p50": cm["step_ms"]["p50"],
                            "step_ms_p99": cm["step_ms"]["p99"], "steps": csteps, "trigger_steps": cm["trigger_steps"],
                            "decode_splits": cm["decode_splits"],
                            "attention_launch_us": rf.get("avg_launch_us"),
                            "attention_bytes_per_launch": rf.get("algorithmic_bytes_per_launch"),
                            "attention_GBps": rf.get("achieved"), "attention_frac_of_hbm_peak": rf.get("frac"),
                            "path_frac_of_hbm_peak": cm.get("path_frac_of_hbm_peak"),
                            "prune_ms_per_layer": cm["prefill_prune"]["ms_per_layer"],
                            "prune_GBps": cm["prefill_prune"]["GBps"],
                            "prune_frac_of_hbm_peak": cm["prefill_prune"]["frac_of_hbm_peak"]}
        result["configs"] = configs

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        try:
            result["cpu_baseline"] = cpu_baseline(wl, args.seed, args.cpu_seqs, args.cpu_layers, args.cpu_steps)
        except Exception as exc:   # noqa: BLE001  (the GPU figures above stand on their own)
            result["cpu_baseline"] = {"value": None, "unit": "tokens/s", "kind": "oracle",
                                      "error": "%s: %s" % (type(exc).__name__, exc)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
