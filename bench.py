#!/usr/bin/env python3
"""Weight-gradient phase benchmark on one MI355X.

A step is one pass of the whole hot path over one synthetic batch of a conv stack:
the exact weight gradient of every layer, then the approximated one (Algorithm 1),
then the zero and the random gradient, each enqueued through
conv_wgrad_schedule_run on torch's current stream.  Inputs are resident in HBM
before the timed region; distinct input sets are rotated so that a step does not
find its operands in the 256 MB last-level cache.

Prints one JSON line: metric/value (ms per step), phase_ms per method, `roofline` (exact phase against the
matrix-core peak, with measured HBM traffic), `roofline_approx` (approximation phase against HBM bandwidth),
`cpu_baseline` (the fp64 oracle on the host cores), `per_layer` (single-layer calls).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"fp32": 157.3, "bf16": 2500.0}   # dense matrix-core peaks of MI355X


def approx_algorithmic_bytes(l, N, e):
    """dY once + the distinct X elements the patches can touch + dW once."""
    return (N * l.K * l.Ho * l.Wo * e + min(N * l.C * l.H * l.W, N * l.K * l.C * l.R * l.S) * e
            + l.K * l.C * l.R * l.S * 4)


def exact_min_bytes(l, N, e):
    return (N * l.C * l.H * l.W + N * l.K * l.Ho * l.Wo) * e + l.K * l.C * l.R * l.S * 4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="resnet20_n128_fp32")
    ap.add_argument("--copies", type=int, default=0, help="distinct input sets to rotate (0 = enough for 1 GB)")
    ap.add_argument("--layer-reps", type=int, default=20, help="back-to-back launches per layer in the per-layer pass")
    ap.add_argument("--cpu-budget-s", type=float, default=20.0, help="CPU seconds to spend on the oracle baseline (0 = skip)")
    ap.add_argument("--event-every", type=int, default=5,
                    help="timed steps between two steps whose phases are bracketed by HIP events (an event pair "
                         "drains the stream: five per step cost 25 us of a 205 us step)")
    ap.add_argument("--scale", type=float, default=1.0 / 128)
    ap.add_argument("--topk", type=int, default=4, help="k of the top-k column of the per-layer pass (0 = skip)")
    ap.add_argument("--no-layouts", action="store_true",
                    help="skip the channel-last columns of the per-layer pass (the paper's kernel layout and its two transposes)")
    ap.add_argument("--phases", default="exact,approx,zero,random",
                    help="phases a step enqueues; anything but the default is for counter runs that must "
                         "attribute every dispatch to one phase, and the printed line then says so")
    ap.add_argument("--sweep-batches", type=int, default=0,
                    help="distinct resident mini-batches of a schedule sweep (workloads *_schedule_sweep); "
                         "0 = 100 for ResNet-20, 24 for VGG-19")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 256 MiB device copy 10 times and exit (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path has no multi-GPU part); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1908_05460_amd import binding as B, inputs, schedule as sch

    B.load()   # raises if libwgrad.so is missing: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        a = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")   # 256 MiB read + 256 MiB written
        b = torch.empty_like(a)
        for _ in range(10):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": a.numel() * 4, "bytes_written": a.numel() * 4, "launches": 10}}))
        return
    cfg, stack_fn, N, dtype = inputs.WORKLOADS[args.workload]
    stack = stack_fn()
    e = 2 if dtype == "bf16" else 4
    nl = len(stack)
    if args.workload.endswith("_schedule_sweep"):
        if args.sweep_batches <= 0:
            args.sweep_batches = 100 if args.workload.startswith("resnet20") else 24
        run_sweep(args, B, inputs, sch, torch, np, cfg, stack, N, dtype)
        return
    set_bytes = sum(exact_min_bytes(l, N, e) for l in stack)
    copies = args.copies or max(2, min(8, math.ceil(1e9 / set_bytes)))

    def to_gpu(a):
        t = torch.from_numpy(a)
        if a.dtype == np.uint16:
            t = t.view(torch.bfloat16)
        return t.cuda()

    descs = [B.desc_for(l, N, dtype) for l in stack]
    sets, host0 = [], None
    for b in range(copies):
        data = [inputs.make_layer_inputs(l, N, config=cfg, batch=b, layer_index=i, dtype=dtype)
                for i, l in enumerate(stack)]
        if b == 0:
            host0 = data
        Xs = [to_gpu(x) for x, _ in data]
        dYs = [to_gpu(y) for _, y in data]
        dWs = [torch.empty((l.K, l.C, l.R, l.S), device="cuda") for l in stack]
        sets.append(B.Schedule(descs, Xs, dYs, dWs))
        del data
    m_exact = np.full(nl, sch.EXACT, np.uint8)
    m_approx = np.full(nl, sch.APPROX, np.uint8)
    m_zero = np.full(nl, sch.ZERO, np.uint8)
    m_random = np.full(nl, sch.RANDOM, np.uint8)
    ws = B.alloc_workspace(max(sets[0].workspace_bytes(m_exact), sets[0].workspace_bytes(m_approx)))
    dw_total = sum(l.K * l.C * l.R * l.S for l in stack)

    phases = ("exact", "approx", "zero", "random")
    on = set(args.phases.split(","))
    assert on <= set(phases) and on, "--phases takes a comma list of exact,approx,zero,random"
    every = max(1, args.event_every)
    ev = {i: [torch.cuda.Event(enable_timing=True) for _ in range(5)] for i in range(0, args.steps, every)}

    def step(i, events=None):
        s = sets[i % copies]
        if events: events[0].record()
        if "exact" in on: s.run(m_exact, ws)
        if events: events[1].record()
        if "approx" in on: s.run(m_approx, ws, scale=args.scale)
        if events: events[2].record()
        if "zero" in on: s.run(m_zero, ws)
        if events: events[3].record()
        if "random" in on: s.run(m_random, ws, sigma=1.0 / 128, seed=inputs.ROOT_SEED, offset=i * dw_total)
        if events: events[4].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, ev.get(i))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    phase_ms = {p: float(np.median([e[j].elapsed_time(e[j + 1]) for e in ev.values()]))
                for j, p in enumerate(phases)}

    # ---- per-layer pass: groups of back-to-back launches of one layer between one event pair,
    #      rotating the input sets, same launch configuration as above ----
    reps = args.layer_reps
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    per_layer = []
    ws_l = ws

    def time_layer(fn):
        for r in range(3):
            fn(r)
        torch.cuda.synchronize()
        a0.record()
        for r in range(reps):
            fn(r)
        a1.record()
        torch.cuda.synchronize()
        return a0.elapsed_time(a1) * 1e3 / reps     # us per launch

    tot = {"exact_us": 0.0, "approx_us": 0.0, "flops": 0.0, "approx_bytes": 0.0}
    for i, l in enumerate(stack):
        d = descs[i]
        if reps <= 0:       # counter runs: no single-layer calls; keep the sums defined
            tot["flops"] += l.flops(N); tot["approx_bytes"] += approx_algorithmic_bytes(l, N, e)
            continue
        t_ex = time_layer(lambda r: B.conv_wgrad_exact(d, sets[r % copies]._keep[0][i], sets[r % copies]._keep[1][i],
                                                       dW=sets[r % copies]._keep[2][i], ws=ws_l))
        t_ap = time_layer(lambda r: B.conv_wgrad_approx(d, sets[r % copies]._keep[0][i], sets[r % copies]._keep[1][i],
                                                        scale=args.scale, dW=sets[r % copies]._keep[2][i], ws=ws_l))
        topk = min(args.topk, d.Ho * d.Wo)
        t_tk = None
        if topk > 0:
            ws_k = B.alloc_workspace(B.topk_workspace_bytes(d, topk))
            t_tk = time_layer(lambda r: B.conv_wgrad_approx_topk(d, sets[r % copies]._keep[0][i], sets[r % copies]._keep[1][i],
                                                                 topk, scale=args.scale, dW=sets[r % copies]._keep[2][i], ws=ws_k))
        lay = {}
        if not args.no_layouts:
            # the paper's route inside an NCHW framework: transpose X, channel-last kernel (OHWI result), transpose dW
            Xn = [B.conv_wgrad_transpose_x(d, sets[c]._keep[0][i], True) for c in range(min(copies, 2))]
            ws_n = B.alloc_workspace(B.nhwc_workspace_bytes(d, B.APPROX))
            ohwi = torch.empty(B.dw_shape(d, B.DW_OHWI), dtype=torch.float32, device="cuda")
            hwio = torch.empty(B.dw_shape(d, B.DW_HWIO), dtype=torch.float32, device="cuda")
            t_k = time_layer(lambda r: B.conv_wgrad_approx_nhwc(d, Xn[r % len(Xn)], sets[r % copies]._keep[1][i], B.DW_OHWI,
                                                               scale=args.scale, dW=ohwi, ws=ws_n))
            t_x = time_layer(lambda r: B.conv_wgrad_transpose_x(d, sets[r % copies]._keep[0][i], True, out=Xn[r % len(Xn)]))
            t_w = time_layer(lambda r: B.conv_wgrad_permute_dw(d, ohwi, B.DW_OHWI, B.DW_HWIO, out=hwio))
            lay = {"nhwc_kernel_us": round(t_k, 2), "transpose_x_us": round(t_x, 2), "transpose_dw_us": round(t_w, 2),
                   "nhwc_total_us": round(t_k + t_x + t_w, 2)}
            del Xn, ws_n
        fl, ab = l.flops(N), approx_algorithmic_bytes(l, N, e)
        per_layer.append({"layer": l.name, "shape": f"{l.C}->{l.K}@{l.H}s{l.stride}",
                          "exact_us": round(t_ex, 2), "approx_us": round(t_ap, 2),
                          "exact_tflops": round(fl / t_ex / 1e6, 2),
                          "exact_frac_mfma": round(fl / t_ex / 1e6 / MFMA_PEAK_TFLOPS[dtype], 4),
                          "approx_gbs": round(ab / t_ap / 1e3, 1),
                          "approx_frac_hbm": round(ab / t_ap / 1e3 / HBM_PEAK_GBS, 4),
                          "speedup": round(t_ex / t_ap, 2),
                          "topk": topk, "topk_us": round(t_tk, 2) if t_tk else None, **lay})
        tot["exact_us"] += t_ex; tot["approx_us"] += t_ap; tot["flops"] += fl; tot["approx_bytes"] += ab

    # Roofline of the dominant kernel, in the launch configuration timed above: the exact phase
    # (conv_wgrad_schedule_run folds layers of one shape into one wgrad_exact_stream launch plus one
    # combine_partials launch), bracketed by HIP events on the launch stream inside the timed region.
    traffic = None
    tpath = os.path.join(ROOT, "paper_1908_05460_amd", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(args.workload)
    phase_ms = {k: max(v, 1e-6) for k, v in phase_ms.items()}
    single = reps > 0
    achieved_tf = tot["flops"] / phase_ms["exact"] / 1e9
    roofline = {"kernel": "exact phase = wgrad_exact_multi | wgrad_exact_stream | wgrad_exact_bf16_multi (layer groups folded into launches) + combine_table",
                "bound": "mfma", "achieved": round(achieved_tf, 3), "peak": MFMA_PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                "frac": round(achieved_tf / MFMA_PEAK_TFLOPS[dtype], 4),
                "traffic": traffic["exact_phase_bytes"] if traffic else None,
                "algorithmic_flops": tot["flops"], "algorithmic_min_bytes": sum(exact_min_bytes(l, N, e) for l in stack),
                "layers": nl, "phase_us": round(phase_ms["exact"] * 1e3, 1),
                "single_layer_calls": {"sum_us": round(tot["exact_us"], 1),
                                       "tflops": round(tot["flops"] / tot["exact_us"] / 1e6, 2)} if single else None}
    achieved_gbs = tot["approx_bytes"] / phase_ms["approx"] / 1e6
    roofline_approx = {"kernel": "approx phase = approx_fused_multi | approx_select + (approx_gather_lds_multi | approx_gather_direct | wgrad_exact_bf16_multi<SPARSE>) | sparsify_small + wgrad_exact_stream, + combine_table",
                       "bound": "hbm", "achieved": round(achieved_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(achieved_gbs / HBM_PEAK_GBS, 4),
                       "traffic": traffic["approx_phase_bytes"] if traffic else None,
                       "algorithmic_bytes": tot["approx_bytes"], "layers": nl,
                       "phase_us": round(phase_ms["approx"] * 1e3, 1),
                       "single_layer_calls": {"sum_us": round(tot["approx_us"], 1),
                                              "gbs": round(tot["approx_bytes"] / tot["approx_us"] / 1e3, 1)} if single else None}

    # ---- the oracle on the host cores, bounded sample of the same workload ----
    cpu = None
    if args.cpu_budget_s > 0:
        import oracle
        spent, done_flops, t_exact, t_approx, names = 0.0, 0.0, 0.0, 0.0, []
        order = sorted(range(nl), key=lambda i: stack[i].flops(N))       # cheapest layers first
        for i in order:
            l = stack[i]
            est = l.flops(N) / 2 / 0.5e9 / max(1, oracle.num_threads())  # ~0.5 GMAC/s/thread
            if names and spent + est > args.cpu_budget_s:
                continue
            g = oracle.shape(N, l.C, l.H, l.W, l.K, l.R, l.S, l.stride, l.pad)
            X, dY = host0[i]
            c0 = time.perf_counter(); oracle.wgrad_exact(g, X, dY); c1 = time.perf_counter()
            oracle.wgrad_approx(g, X, dY, scale=args.scale); c2 = time.perf_counter()
            t_exact += c1 - c0; t_approx += c2 - c1; spent += c2 - c0
            done_flops += l.flops(N); names.append(l.name)
        frac = done_flops / tot["flops"]
        cpu = {"value": round((t_exact + t_approx) * 1e3 / frac, 1), "unit": "ms",
               "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{len(names)} of {nl} layers of one batch ({100 * frac:.0f}% of the exact FLOPs), "
                         f"exact+approx, scaled to the whole stack by FLOPs",
               "exact_ms": round(t_exact * 1e3 / frac, 1), "approx_ms": round(t_approx * 1e3 / frac, 1)}

    out = {
        "metric": "weight-grad ms/iter (exact vs approx)", "value": round(ms_per_step, 4), "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if dtype == "fp32" else "bf16 in, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": args.workload, "layers": nl, "batch": N, "input_sets_rotated": copies,
                   "step": " + ".join(p for p in phases if p in on) + " gradient of every layer"
                           + ("" if len(on) == 4 else "  (PARTIAL STEP: not a benchmark result)")},
        "phase_ms": {k: round(v, 4) for k, v in phase_ms.items()},
        "speedup_approx_vs_exact": round(phase_ms["exact"] / phase_ms["approx"], 3),
        "roofline": roofline, "roofline_approx": roofline_approx, "cpu_baseline": cpu,
        "per_layer": per_layer,
        "paper_context": "paper: approx kernel incl. transposes >= 3x faster than cuDNN 7.4.2 backward-filter "
                         "on a Titan Xp for most layers; end-to-end training speedup 3.5% (ResNet-20) to ~7%",
    }
    print(json.dumps(out))


def run_sweep(args, B, inputs, sch, torch, np, cfg, stack, N, dtype):
    """Approximation-schedule sweep: every mini-batch of a resident set runs the weight-gradient phase
    with the per-layer methods its schedule mask gives (one conv_wgrad_schedule_run per batch)."""
    nl, nb = len(stack), args.sweep_batches
    descs = [B.desc_for(l, N, dtype) for l in stack]
    sets = []
    for b in range(nb):
        data = [inputs.make_layer_inputs(l, N, config=cfg, batch=b, layer_index=i, dtype=dtype)
                for i, l in enumerate(stack)]
        sets.append(B.Schedule(descs, [torch.from_numpy(x).cuda() for x, _ in data],
                               [torch.from_numpy(y).cuda() for _, y in data],
                               [torch.empty((l.K, l.C, l.R, l.S), device="cuda") for l in stack]))
    masks = dict(sch.SWEEP_MASKS); masks.update(sch.PAPER_SCHEDULES)
    rows = {name: [fn(nl, b) for b in range(nb)] for name, fn in masks.items()}
    ws = B.alloc_workspace(max(sets[0].workspace_bytes(r) for rr in rows.values() for r in rr[:4]))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    result = {}
    t_start = time.perf_counter()
    for name, rr in rows.items():
        for b in range(min(nb, 8)):                       # warm-up
            sets[b].run(rr[b], ws, scale=args.scale)
        torch.cuda.synchronize()
        e0.record()
        for b in range(nb):
            sets[b].run(rr[b], ws, scale=args.scale)
        e1.record()
        torch.cuda.synchronize()
        result[name] = {"ms_per_iter": round(e0.elapsed_time(e1) / nb, 4),
                        "fraction_approximated": round(sch.fraction_approximated(masks[name], nl, nb), 4)}
    wall = time.perf_counter() - t_start
    base = result["all_exact"]["ms_per_iter"]
    for v in result.values():
        v["vs_all_exact"] = round(v["ms_per_iter"] / base, 4)
    flops = sum(l.flops(N) for l in stack)
    print(json.dumps({
        "metric": "weight-grad ms/iter (exact vs approx)", "value": base, "unit": "ms", "n_gpus": 1,
        "steps": nb, "warmup": min(nb, 8), "ms_per_step": base, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "layers": nl, "batch": N, "resident_batches": nb,
                   "step": "one conv_wgrad_schedule_run per mini-batch; value = the all-exact mask"},
        "sweep": result,
        "roofline": {"kernel": "all-exact mask: exact phase of every batch", "bound": "mfma",
                     "achieved": round(flops / base / 1e9, 3), "peak": MFMA_PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                     "frac": round(flops / base / 1e9 / MFMA_PEAK_TFLOPS[dtype], 4), "traffic": None},
        "cpu_baseline": None, "timed_wall_s": round(wall, 2),
        "paper_context": "paper: schedules approximate 25% of (layer, batch) pairs; its end-to-end bound for that is ~8%",
    }))


if __name__ == "__main__":
    main()
