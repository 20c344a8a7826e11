#!/usr/bin/env python3
"""Benchmark of the LASER-KV prefill-compression hot path on one MI355X.

A step is one pass of the whole path (score + LSH + top-k + gather-append) over one layer of one
synthetic context: every block of the workload, issued back to back on one stream with no host
synchronisation, inputs resident in HBM.  Prints ONE JSON line: context tokens per second per layer,
the roofline position of the dominant kernel (timed live with HIP events around every kernel launch)
and the CPU oracle's rate on the same box as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # dense bf16 MFMA, MI355X
PEAK_MFMA_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def algorithmic_work(wl, B):
    """Per-launch algorithmic work of every kernel: (bound, amount, unit). One launch = one block, all KV heads.
    flops: 2*d*rows*S per contraction (look-back keys and the query projections are extras, not counted);
    bytes: what the step must move at least once."""
    d, s, hk = wl.head_dim, wl.s_block, wl.n_kv_heads
    es = 2 if wl.dtype == "bf16" else 4
    m = wl.group * wl.window
    lk = wl.lsh_tables * wl.lsh_bits
    score = 2.0 * d * m * hk * s
    return {
        # sweep 1 = the score contraction (priced once per sweep kernel) + the projection of the keys
        "sweep1": ("mfma", score + 2.0 * d * lk * hk * s),
        "sweep2": ("mfma", score),
        # the one sweep of --lse complete: both contractions once
        "single": ("mfma", score + 2.0 * d * lk * hk * s),
        "count": ("hbm", hk * s * (wl.lsh_tables * 2 + 4) + wl.n_q_heads * wl.window * wl.lsh_tables * 2),
        "select": ("hbm", hk * s * 8 + hk * B * 4),
        "append": ("hbm", hk * B * (4 * d * es + 4 + 8)),
    }


def measure(wl, args, dev, cpu_seconds):
    """Times one workload: returns the fields of the JSON line that depend on the workload."""
    import statistics
    import torch
    from paper_2602_02199_amd import synth
    from paper_2602_02199_amd.driver import LayerCompressor

    comp = LayerCompressor(wl, dev)
    t_gen = time.time()
    data = synth.make_layer(wl, args.layer, comp.parts[0])
    ddev = {k: v.to(dev) for k, v in data.items() if k != "needles"}
    torch.cuda.synchronize()
    print(f"[bench] workload {wl.name}: inputs generated and resident in {time.time() - t_gen:.1f}s "
          f"(B={comp.B}, parts={comp.parts})", file=sys.stderr, flush=True)

    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)   # reads n bytes, writes n bytes
        torch.cuda.synchronize()
        print(f"[bench] calibration copy: {n} bytes read and written", file=sys.stderr, flush=True)
        del src, dst
    lse = None
    if args.lse == "complete":
        # stand-in for the model's attention kernel: every window row's log-sum-exp over the look-back keys and
        # the block keys it sees, computed once here (outside the timed region) with plain torch ops
        lse = []
        s, w, g, nl = wl.s_block, wl.window, wl.group, comp.parts[1]
        vis = torch.arange(s, device=dev)[None, :] <= (s - w + torch.arange(w, device=dev))[:, None]
        for t in range(wl.n_blocks):
            lo = t * s
            kk = ddev["k"][:, max(lo - nl, 0) if t else lo:lo + s].float()
            q = ddev["q_win"][t].float().view(wl.n_kv_heads, g * w, wl.head_dim)
            logits = torch.einsum("hmd,hkd->hmk", q, kk) / wl.head_dim ** 0.5
            mask = torch.ones(w, kk.shape[1], dtype=torch.bool, device=dev)
            mask[:, kk.shape[1] - s:] = vis
            logits = logits.view(wl.n_kv_heads, g, w, -1).masked_fill(~mask, float("-inf"))
            lse.append(torch.logsumexp(logits, dim=-1).reshape(wl.n_q_heads, w).contiguous())
        torch.cuda.synchronize()
    plan = comp.plan_layer(ddev, fused=not args.unfused, row_lse_complete=lse)
    stream = torch.cuda.Stream()
    graph = None
    with torch.cuda.stream(stream):
        for _ in range(args.warmup):
            comp.run_plan(plan)
        stream.synchronize()
        if args.mode == "graph":
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                comp.run_plan(plan)
            graph.replay()
            stream.synchronize()
        # exactly `steps` timed steps between two synchronisations; an event on the launch stream after every
        # step gives the per-step times, whose median is the reported step time
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record(stream)
        for i in range(args.steps):
            if graph is not None:
                graph.replay()
            else:
                comp.run_plan(plan)
            marks[i + 1].record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]
        ms_mean = (t1 - t0) * 1e3 / args.steps
        ms_per_step = statistics.median(per_step)
        # which kernels one layer launches, and how often: one pass with an event pair around every launch
        comp.lib.laserkv_profile_begin()
        comp.run_plan(plan)
        prof = comp.lib.laserkv_profile_end()
        torch.cuda.synchronize()
        # per-kernel durations: the layer's launches of ONE kernel kind, back to back (graph replays in
        # graph mode), between two events on the launch stream; average = elapsed / launches.  Event pairs
        # between consecutive kernels would add about 2 us to each.
        kern = {}
        for name, (_, n_launch) in prof.items():
            if not n_launch or not args.profile_steps:
                kern[name] = dict(avg_us=0.0, launches=0)
                continue
            comp.lib.laserkv_profile_isolate(name)
            comp.run_plan(plan)
            stream.synchronize()
            g1 = None
            if args.mode == "graph":
                g1 = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g1, stream=stream):
                    comp.run_plan(plan)
                g1.replay()
                stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(args.profile_steps):
                if g1 is not None:
                    g1.replay()
                else:
                    comp.run_plan(plan)
            e1.record(stream)
            e1.synchronize()
            kern[name] = dict(avg_us=1e3 * e0.elapsed_time(e1) / (args.profile_steps * n_launch), launches=n_launch)
            del g1
        comp.lib.laserkv_profile_isolate(None)
        comp.run_plan(plan)   # leave the workspace and the cache in the state of a complete pass
        torch.cuda.synchronize()
    tokens = ddev["k"].shape[1] * args.batch
    value = tokens / (ms_per_step * 1e-3)
    res = dict(value=round(value, 1), ms_per_step=round(ms_per_step, 4), ms_per_step_mean=round(ms_mean, 4),
               ms_per_step_min=round(min(per_step), 4), ms_per_step_max=round(max(per_step), 4),
               config=dict(workload=wl.name, l_ctx=wl.l_ctx, s_block=wl.s_block, window=wl.window, n=wl.n_div,
                           lsh_tables=wl.lsh_tables, lsh_bits=wl.lsh_bits, n_q_heads=wl.n_q_heads,
                           n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim, budget_per_block=comp.B,
                           blocks=wl.n_blocks, layers_timed=1, launch=args.mode, sequences=args.batch,
                           step_time="median of the timed steps", row_statistics=args.lse,
                           entry="laserkv_select_block+laserkv_append" if args.unfused else "laserkv_compress_block"),
               roofline=None, cpu_baseline=None)

    work = algorithmic_work(wl, comp.B)
    if not args.unfused:  # the last kernel selects and appends
        work["select"] = ("hbm", work["select"][1] + work["append"][1])
    if args.attend:
        res["attend_cache"] = measure_attend(wl, comp, ddev, dev, cases=args.attend_case.split(","))
    if args.pipeline and args.batch == 1 and args.lse == "own":
        res["model_pipeline"] = measure_model_pipeline(wl, comp, ddev, dev)
    if not any(v["launches"] for v in kern.values()):
        return res
    peak_mfma = PEAK_MFMA_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_MFMA_F32_TFLOPS
    per_kernel = {}
    for name, v in kern.items():
        if not v["launches"]:
            continue
        bound, amount = work[name]
        dur_s = v["avg_us"] * 1e-6
        if bound == "mfma":
            peak, achieved, unit = peak_mfma, amount / dur_s / 1e12, "TFLOP/s"
        else:
            peak, achieved, unit = PEAK_HBM_GBS, amount / dur_s / 1e9, "GB/s"
        per_kernel[name] = dict(bound=bound, avg_us=round(v["avg_us"], 2), achieved=round(achieved, 3), peak=peak,
                                unit=unit, frac=round(achieved / peak, 4), launches_per_step=v["launches"])
    dom = max(per_kernel, key=lambda k: per_kernel[k]["avg_us"])
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{wl.name}{'-lse-complete' if args.lse == 'complete' else ''}.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(dom)
    d = per_kernel[dom]
    roofline = dict(bound=d["bound"], kernel=dom, achieved=d["achieved"], peak=d["peak"], unit=d["unit"],
                    frac=d["frac"], traffic=traffic, avg_us=d["avg_us"], kernels=per_kernel,
                    targets="score/projection kernels >= 0.50 of bf16 MFMA peak, hash/select/gather >= 0.60 of HBM peak: "
                            + ("met" if all(v["frac"] >= (0.5 if v["bound"] == "mfma" else 0.6) for v in per_kernel.values())
                               else "NOT met"))
    # whole-path roofline: serial sum of the contraction time at MFMA peak and the byte time at HBM peak
    es = 2 if wl.dtype == "bf16" else 4
    flops_blk = work["sweep1"][1]   # score + key projection once: the same figure with one sweep or two
    bytes_blk = wl.n_kv_heads * wl.s_block * wl.head_dim * es + wl.n_q_heads * wl.window * wl.head_dim * es \
        + work["append"][1]
    t_roof = (flops_blk / (peak_mfma * 1e12) + bytes_blk / (PEAK_HBM_GBS * 1e9)) * wl.n_blocks
    roofline["path_frac_of_roofline"] = round(t_roof / (ms_per_step * 1e-3), 4)
    res["roofline"] = roofline
    if cpu_seconds > 0:
        res["cpu_baseline"] = cpu_baseline(wl, data, comp.B, cpu_seconds)
    del comp, ddev, data
    torch.cuda.empty_cache()
    return res


def measure_model_pipeline(wl, comp, ddev, dev, steps=3):
    """One layer the way a model runs it: per block laserkv_attend_block over the compacted cache and the
    block (all of the block's rows: queries are seeded N(0,1) except the window rows, which are the
    workload's), the window rows' log-sum-exp handed to the selection (laserkv_set_row_lse_complete), then
    select + append.  Step time from graph replays; the split between attention and selection from one eager
    pass with an event pair around every kernel launch."""
    import torch
    s, d, w, nb = wl.s_block, wl.head_dim, wl.window, wl.n_blocks
    gen = torch.Generator(device=dev).manual_seed(4321)
    dt = ddev["k"].dtype
    q_blocks = []
    for t in range(nb):
        q = torch.randn(wl.n_q_heads, s, d, generator=gen, device=dev).to(dt)
        q[:, s - w:] = ddev["q_win"][t]
        q_blocks.append(q)
    out = torch.empty(wl.n_q_heads, s, d, dtype=torch.float32, device=dev)
    lse = torch.empty(wl.n_q_heads, s, dtype=torch.float32, device=dev)
    lse_win = torch.empty(wl.n_q_heads, w, dtype=torch.float32, device=dev)
    n_last = (nb - 1) * min(comp.B, s)
    ws = torch.empty(max(comp.lib.laserkv_attend_block_workspace_bytes(s, n, s) for n in (0, n_last)), dtype=torch.uint8, device=dev)
    run = lambda: comp.run_layer_with_attention(ddev, q_blocks, out, lse, lse_win, ws)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        run()
        stream.synchronize()
        comp.lib.laserkv_profile_begin()
        run()
        prof = comp.lib.laserkv_profile_end()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            run()
        graph.replay()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            graph.replay()
        e1.record(stream)
        e1.synchronize()
    ms = e0.elapsed_time(e1) / steps
    att = prof["attend"][0]
    sel = sum(v[0] for k, v in prof.items() if k != "attend")
    pairs = sum(s * t * min(comp.B, s) + s * (s + 1) // 2 for t in range(nb))
    tfl = 4 * wl.n_q_heads * pairs * d / (att * 1e-3) / 1e12
    peak = PEAK_MFMA_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_MFMA_F32_TFLOPS
    return dict(ms_per_layer=round(ms, 3), tokens_per_s_per_layer=round(wl.l_ctx / (ms * 1e-3), 1),
                attention_ms=round(att, 3), attention_tflops=round(tfl, 1), attention_mfma_frac=round(tfl / peak, 4),
                selection_ms=round(sel, 3), selection_share=round(sel / (att + sel), 4),
                launches={k: v[1] for k, v in prof.items() if v[1]})


def measure_attend(wl, comp, ddev, dev, reps=10, cases=("decode", "window")):
    """laserkv_attend_cache over the layer's finished cache (the rows the timed steps kept): one decode query
    per head (bound by reading the cached K and V once) and the next block's window rows (bound by the two
    contractions QK^T and PV), with and without the output; and laserkv_attend_block for the last block (case
    "prefill").  Event times on the launch stream, average of `reps` launches after two."""
    import torch
    n = wl.n_blocks * min(comp.B, wl.s_block)
    es = 2 if wl.dtype == "bf16" else 4
    out = {}
    stream = torch.cuda.current_stream()
    for label, n_q in (("decode", 1), ("window", wl.window), ("window_normaliser_only", wl.window)):
        if label.split("_")[0] not in cases:
            continue
        q = ddev["q_win"][-1][:, :n_q].contiguous()
        o = None if label.endswith("only") else torch.empty(wl.n_q_heads, n_q, wl.head_dim, dtype=torch.float32, device=dev)
        lse = torch.empty(wl.n_q_heads, n_q, dtype=torch.float32, device=dev)
        ws = torch.empty(comp.lib.laserkv_attend_workspace_bytes(n_q, n), dtype=torch.uint8, device=dev)
        run = lambda: comp.lib.laserkv_attend_cache(q, comp.k_cache, comp.v_cache, cache_len=n, out=o, out_lse=lse, workspace=ws)
        run(); run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            run()
        e1.record(stream)
        e1.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / reps
        both = 1 if o is None else 2   # contractions per (query, key) pair; tensors of the cache read
        nbytes = both * wl.n_kv_heads * n * wl.head_dim * es
        flops = 2 * both * wl.n_q_heads * n_q * n * wl.head_dim
        gbs, tfl = nbytes / us / 1e3, flops / us / 1e6
        peak_mfma = PEAK_MFMA_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_MFMA_F32_TFLOPS
        out[label] = dict(n_q=n_q, cache_rows_per_head=n, avg_us=round(us, 2), hbm_gbs=round(gbs, 1),
                          hbm_frac=round(gbs / PEAK_HBM_GBS, 4), tflops=round(tfl, 1), mfma_frac=round(tfl / peak_mfma, 4),
                          bound="hbm" if gbs / PEAK_HBM_GBS > tfl / peak_mfma else "mfma")
    if "prefill" in cases:
        # laserkv_attend_block: the last block's own attention, every row of the block over the cache of the
        # earlier blocks and, causally, over the block itself (the model's attention call; its log-sum-exp of
        # the window rows is what laserkv_set_row_lse_complete takes).  Queries: seeded N(0,1).
        s, d = wl.s_block, wl.head_dim
        n_c = (wl.n_blocks - 1) * min(comp.B, s)
        lo = (wl.n_blocks - 1) * s
        gen = torch.Generator(device=dev).manual_seed(1234)
        q = torch.randn(wl.n_q_heads, s, d, generator=gen, device=dev).to(ddev["k"].dtype)
        kb, vb = ddev["k"][:, lo:lo + s], ddev["v"][:, lo:lo + s]
        o = torch.empty(wl.n_q_heads, s, d, dtype=torch.float32, device=dev)
        lse = torch.empty(wl.n_q_heads, s, dtype=torch.float32, device=dev)
        ws = torch.empty(comp.lib.laserkv_attend_block_workspace_bytes(s, n_c, s), dtype=torch.uint8, device=dev)
        run = lambda: comp.lib.laserkv_attend_block(q, comp.k_cache, comp.v_cache, kb, vb, cache_len=n_c, block_pos0=lo,
                                                    out=o, out_lse=lse, workspace=ws)
        run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(3):
            run()
        e1.record(stream)
        e1.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / 3
        pairs = s * n_c + s * (s + 1) // 2   # (query, visible key) pairs per query head
        flops = 4 * wl.n_q_heads * pairs * d
        tfl = flops / us / 1e6
        peak_mfma = PEAK_MFMA_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_MFMA_F32_TFLOPS
        out["prefill_block"] = dict(n_q=s, cache_rows_per_head=n_c, block_keys=s, avg_us=round(us, 1), tflops=round(tfl, 1),
                                    mfma_frac=round(tfl / peak_mfma, 4), bound="mfma")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b-128k")
    ap.add_argument("--secondary", default="gqa8-128k",
                    help="a second workload timed the same way and reported as the `secondary` object of the JSON line "
                         "('none' skips it); not run with --batch, --calibrate-copy or --profile-steps 0")
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph")
    ap.add_argument("--profile-steps", type=int, default=5, help="replays per kernel kind for the per-kernel durations; 0 skips them")
    ap.add_argument("--unfused", action="store_true", help="laserkv_select_block + laserkv_append instead of laserkv_compress_block")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="also run one plain device copy of this many MiB (a known-size reference for HBM byte counters)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="lower bound of oracle work for cpu_baseline; 0 skips")
    ap.add_argument("--policy", choices=["per-head", "consensus"], default="per-head",
                    help="consensus: the global-consensus variant (scores summed over --layers layers and all heads, one "
                         "selection per block); prints its own JSON line, not the headline metric")
    ap.add_argument("--layers", type=int, default=4, help="layers summed by --policy consensus")
    ap.add_argument("--lse", choices=["own", "complete"], default="own",
                    help="complete: the window rows' complete log-sum-exp is handed to the library (as the model's "
                         "attention kernel would report it), so the first sweep only hashes; not the headline configuration")
    ap.add_argument("--no-complete", dest="with_complete", action="store_false",
                    help="skip the extra measurement of the workload with complete row statistics from the caller")
    ap.add_argument("--attend-case", default="decode,window,prefill", help="which attention cases to time (profiling one at a time)")
    ap.add_argument("--no-attend", dest="attend", action="store_false",
                    help="skip the timing of laserkv_attend_cache over the finished cache")
    ap.add_argument("--no-pipeline", dest="pipeline", action="store_false",
                    help="skip the layer run with the library's own block attention in front of every selection")
    ap.add_argument("--layer-sweep", type=int, default=0, metavar="N",
                    help="time layers 0..N-1 of the workload one at a time (each generated with its own seed, one resident "
                         "at a time) and print mean / min / max of the step time over the layers instead of the headline line")
    ap.add_argument("--batch", type=int, default=1,
                    help="fold this many independent sequences into the head axis (heads x batch per call); the rate then "
                         "counts batch x context tokens. 1 is the headline configuration")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        return 2
    if args.steps < 1:
        print("bench.py: --steps must be at least 1", file=sys.stderr)
        return 2

    from paper_2602_02199_amd import synth

    wl = synth.WORKLOADS[args.workload]
    if args.batch > 1:
        wl = synth.shrink(wl, name=f"{wl.name}-x{args.batch}", n_q_heads=wl.n_q_heads * args.batch,
                          n_kv_heads=wl.n_kv_heads * args.batch)
    dev = "cuda:0"
    if args.policy == "consensus":
        return bench_consensus(args, wl, dev)
    if args.layer_sweep > 0:
        import statistics
        import torch
        l_args = argparse.Namespace(**vars(args))
        l_args.attend = l_args.pipeline = False
        l_args.profile_steps = 0
        per_layer = []
        for layer in range(args.layer_sweep):
            l_args.layer = layer
            per_layer.append(measure(wl, l_args, dev, 0.0)["ms_per_step"])
            torch.cuda.empty_cache()
        mean = statistics.mean(per_layer)
        print(json.dumps(dict(metric="prefill-compression tokens/s/layer, every layer timed by itself", workload=wl.name,
                              layers=args.layer_sweep, ms_per_layer_mean=round(mean, 4), ms_per_layer_min=min(per_layer),
                              ms_per_layer_max=max(per_layer), value=round(wl.l_ctx / (mean * 1e-3), 1), unit="tokens/s/layer",
                              steps=args.steps, warmup=args.warmup, data="synthetic", dtype=wl.dtype)), flush=True)
        return 0
    res = measure(wl, args, dev, args.cpu_seconds)
    if res["roofline"] is None:
        print(json.dumps(dict(value=res["value"], unit="tokens/s/layer", ms_per_step=res["ms_per_step"],
                              note="no per-kernel timing requested: roofline omitted",
                              attend_cache=res.get("attend_cache"), model_pipeline=res.get("model_pipeline"))), flush=True)
        return 0
    secondary = None
    if args.secondary not in ("none", args.workload) and args.batch == 1 and not args.calibrate_copy:
        sec_args = argparse.Namespace(**vars(args))
        sec_args.attend = False
        sec_args.pipeline = False
        sec = measure(synth.WORKLOADS[args.secondary], sec_args, dev, 0.0)
        r = sec["roofline"]
        secondary = dict(workload=args.secondary, value=sec["value"], unit="tokens/s/layer", ms_per_step=sec["ms_per_step"],
                         ms_per_step_mean=sec["ms_per_step_mean"], budget_per_block=sec["config"]["budget_per_block"],
                         blocks=sec["config"]["blocks"], dominant_kernel=r["kernel"], bound=r["bound"], frac=r["frac"],
                         avg_us=r["avg_us"], traffic=r["traffic"], kernels=r["kernels"],
                         path_frac_of_roofline=r["path_frac_of_roofline"])
    # the same workload with the window rows' complete log-sum-exp supplied by the caller (one sweep per block)
    complete = None
    if args.lse == "own" and args.with_complete and args.batch == 1 and not args.calibrate_copy:
        c_args = argparse.Namespace(**vars(args))
        c_args.attend = False
        c_args.pipeline = False
        c_args.lse = "complete"
        cm = measure(wl, c_args, dev, 0.0)
        r = cm["roofline"]
        complete = dict(row_statistics="complete, from the caller (stand-in for the model's attention kernel, outside the timed region)",
                        value=cm["value"], unit="tokens/s/layer", ms_per_step=cm["ms_per_step"],
                        ms_per_step_mean=cm["ms_per_step_mean"], dominant_kernel=r["kernel"], bound=r["bound"],
                        frac=r["frac"], avg_us=r["avg_us"], traffic=r["traffic"], kernels=r["kernels"],
                        path_frac_of_roofline=r["path_frac_of_roofline"])
    out = dict(metric="prefill-compression tokens/s/layer (score+LSH+top-k+gather) @128k; % roofline",
               value=res["value"], unit="tokens/s/layer", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=res["ms_per_step"], higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype=wl.dtype, data="synthetic", config=res["config"], roofline=res["roofline"],
               cpu_baseline=res["cpu_baseline"], ms_per_step_mean=res["ms_per_step_mean"],
               ms_per_step_min=res["ms_per_step_min"], ms_per_step_max=res["ms_per_step_max"], secondary=secondary,
               attend_cache=res.get("attend_cache"), complete_statistics=complete,
               model_pipeline=res.get("model_pipeline"))
    print(json.dumps(out), flush=True)
    return 0


def bench_consensus(args, wl, dev):
    """Global-consensus variant: per block, every layer is scored into shared accumulators, one selection
    is made, and every layer appends the shared rows.  A step covers all blocks of --layers layers; the
    rate is context tokens per second per layer (step time divided by the layer count)."""
    import torch
    from paper_2602_02199_amd import binding, synth
    B = binding.laserkv_budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    na, nl, ke, kl = binding.laserkv_partition(B, wl.n_div, wl.alpha, wl.s_block)
    b_t, s, nb, nl_layers = na + nl + ke + kl, wl.s_block, wl.n_blocks, args.layers
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=wl.window, max_ctx_keys=nl)
    data = []
    for layer in range(nl_layers):
        d = synth.make_layer(wl, layer, na)
        data.append({k: v.to(dev) for k, v in d.items() if k != "needles"})
    cap = nb * b_t
    caches = [dict(k=torch.zeros(wl.n_kv_heads, cap, wl.head_dim, dtype=wl.torch_dtype, device=dev),
                   v=torch.zeros(wl.n_kv_heads, cap, wl.head_dim, dtype=wl.torch_dtype, device=dev),
                   pos=torch.full((wl.n_kv_heads, cap), -1, dtype=torch.int64, device=dev)) for _ in range(nl_layers)]
    score = torch.empty(s, dtype=torch.float32, device=dev)
    count = torch.empty(s, dtype=torch.int32, device=dev)
    keep = torch.empty(b_t, dtype=torch.int32, device=dev)

    def step():
        cache_len = 0
        for t in range(nb):
            lo = t * s
            n_ctx = nl if t else 0
            for li in range(nl_layers):
                k_ctx = caches[li]["k"][:, cache_len - n_ctx:cache_len] if n_ctx else None
                lib.laserkv_score_block(data[li]["q_win"][t], data[li]["k"][:, lo:lo + s], k_ctx, data[li]["planes"],
                                        block_pos0=lo, score_acc=score, count_acc=count, accumulate=li > 0)
            lib.laserkv_select_consensus(score, count, s_t=s, n_anchor=na, n_local=nl, k_exact=ke, k_lsh=kl, keep_idx=keep)
            for li in range(nl_layers):
                lib.laserkv_append_shared(data[li]["k"][:, lo:lo + s], data[li]["v"][:, lo:lo + s], keep, b_t=b_t,
                                          block_pos0=lo, k_cache=caches[li]["k"], v_cache=caches[li]["v"],
                                          cache_pos=caches[li]["pos"], cache_len=cache_len)
            cache_len += b_t

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for _ in range(max(args.warmup, 1)):
            step()
        stream.synchronize()
        graph = None
        if args.mode == "graph":
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                step()
            graph.replay()
            stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay() if graph is not None else step()
        stream.synchronize()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
    print(json.dumps(dict(metric="global-consensus variant: context tokens/s/layer (score over all layers and heads, one "
                                 "selection per block, shared append)",
                          value=round(wl.l_ctx / (ms * 1e-3 / nl_layers), 1), unit="tokens/s/layer", n_gpus=1,
                          steps=args.steps, warmup=args.warmup, ms_per_step=round(ms, 4), higher_is_better=True,
                          dtype=wl.dtype, data="synthetic",
                          config=dict(workload=wl.name, layers=nl_layers, blocks=nb, budget_per_block=B, launch=args.mode))),
          flush=True)
    return 0


def cpu_baseline(wl, data, B, min_seconds):
    """The CPU oracle, as it stands, on the first blocks of the same inputs (bounded sample)."""
    import numpy as np
    import torch
    from oracle import laserkv_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    s = wl.s_block
    planes = data["planes"].double().numpy()
    cap = wl.n_blocks * B
    ck = cv = cp = None
    clen, prev_local, nblk = 0, 0, 0
    t0 = time.perf_counter()
    while nblk < wl.n_blocks and (time.perf_counter() - t0 < min_seconds or nblk < 1):
        lo = nblk * s
        k = data["k"][:, lo:lo + s].double().numpy()
        v = data["v"][:, lo:lo + s].double().numpy()
        q = data["q_win"][nblk].double().numpy()
        if ck is None:
            ck = np.zeros((wl.n_kv_heads, cap, wl.head_dim)); cv = np.zeros_like(ck)
            cp = np.full((wl.n_kv_heads, cap), -1, dtype=np.int64)
        parts = O.partition(B, wl.n_div, wl.alpha, k.shape[1])
        k_ctx = ck[:, clen - prev_local:clen] if clen and prev_local else None
        st = O.select_block(q, k, k_ctx, planes, wl.lsh_tables, wl.lsh_bits, *parts, block_pos0=lo)
        clen = O.append(ck, cv, cp, clen, k, v, st["keep"], lo)
        prev_local = parts[1]
        nblk += 1
    dt = time.perf_counter() - t0
    return dict(value=round(nblk * s / dt, 1), unit="tokens/s/layer", cores=int(threads), kind="oracle",
                sample=f"first {nblk} of {wl.n_blocks} blocks of the same layer ({nblk * s} tokens) in {dt:.1f}s, "
                       f"NumPy float64, affinity {len(os.sched_getaffinity(0))} cores")


if __name__ == "__main__":
    sys.exit(main())
