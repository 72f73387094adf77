#!/usr/bin/env python3
"""Weight-gradient phase benchmark on one MI355X.

A step is one pass of the whole hot path over one synthetic batch of a conv stack:
the exact weight gradient of every layer, then the approximated one (Algorithm 1),
then the zero and the random gradient, each enqueued through
conv_wgrad_schedule_run on torch's current stream.  Inputs are resident in HBM
before the timed region; distinct input sets are rotated so that a step does not
find its operands in the 256 MB last-level cache.

Prints ONE JSON line.  Top level: the headline workload (default: the VGG-19 stack at
batch 128 in fp32, the largest fp32 configuration) with metric/value (ms per step),
phase_ms per method (median; phase_ms_min beside it), `roofline` (exact phase against the
matrix-core peak), `roofline_approx` (approximation phase against HBM bandwidth),
`cpu_baseline` (the fp64 oracle on the host cores), `per_layer` (single-layer calls, each
against the roof that binds it).  `machine`: ceilings measured in this run by plain kernels
(copy and read bandwidth, matrix-core loops, LDS reads).  `configs`: the same phase figures
for every other configuration of the benchmark definition (single layer, ResNet-20,
VGG-19 at batch 512 in bf16, the approximation-schedule sweep).
"""
import argparse
import ctypes
import json
import math
import os
import sys
import time
import zlib

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"fp32": 157.3, "bf16": 2500.0}   # dense matrix-core peaks of MI355X
LDS_PEAK_GBS = 256 * 128 * 2.4                       # 256 CUs x 128 B/clk x 2.4 GHz
HEADLINE = "vgg19_n128_fp32"
OTHER_CONFIGS = ("single3x3_n16_fp32", "resnet20_n128_fp32", "vgg19_n512_bf16", "resnet20_schedule_sweep")


def approx_algorithmic_bytes(l, N, e):
    """dY once + the distinct X elements the patches can touch + dW once."""
    return (N * l.K * l.Ho * l.Wo * e + min(N * l.C * l.H * l.W, N * l.K * l.C * l.R * l.S) * e
            + l.K * l.C * l.R * l.S * 4)


def exact_min_bytes(l, N, e):
    return (N * l.C * l.H * l.W + N * l.K * l.Ho * l.Wo) * e + l.K * l.C * l.R * l.S * 4


def gather_bytes(l, N, e):
    """Operand bytes the patch gather reads (out of LDS or cache): one patch per map."""
    return N * l.K * l.C * l.R * l.S * e


def measure_machine(torch):
    """Ceilings a plain HIP kernel reaches on this device, measured now: HBM copy and read bandwidth over
    1 GiB (beyond the last-level cache), matrix-core loops without memory traffic, conflict-free LDS reads."""
    from paper_1908_05460_amd import binding as B
    path = os.path.join(ROOT, "paper_1908_05460_amd", "libwgrad_roofs.so")
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with __graft_entry__.build()")
    B.load()
    R = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    R.roofs_copy.argtypes = [vp, vp, ctypes.c_long, vp]
    R.roofs_read.argtypes = [vp, vp, ctypes.c_long, vp]
    R.roofs_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]
    R.roofs_lds_read.argtypes = [ctypes.c_int, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]
    st = vp(torch.cuda.current_stream().cuda_stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=5):
        fn(); torch.cuda.synchronize()
        best = float("inf")
        for _ in range(reps):
            e0.record(); fn(); e1.record(); torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best * 1e-3                                   # seconds, best of reps

    nbytes = 1 << 30
    a = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    out = {}
    t = timed(lambda: R.roofs_copy(vp(a.data_ptr()), vp(b.data_ptr()), nbytes, st))
    out["hbm_copy_gbs"] = round(2 * nbytes / t / 1e9, 1)
    t = timed(lambda: R.roofs_read(vp(a.data_ptr()), vp(sink.data_ptr()), nbytes, st))
    out["hbm_read_gbs"] = round(nbytes / t / 1e9, 1)
    del a, b
    fl = ctypes.c_double()
    for which, name in ((0, "mfma_f32_16x16x4_tflops"), (1, "mfma_bf16_16x16x32_tflops"), (2, "mfma_bf16_32x32x16_tflops")):
        t = timed(lambda: R.roofs_mfma(which, 256 * 8, 2000, vp(sink.data_ptr()), ctypes.byref(fl), st))
        out[name] = round(fl.value / t / 1e12, 1)
    by = ctypes.c_double()
    t = timed(lambda: R.roofs_lds_read(256 * 4, 4000, vp(sink.data_ptr()), ctypes.byref(by), st))
    out["lds_read_b32_gbs"] = round(by.value / t / 1e9, 1)
    out["nominal"] = {"hbm_gbs": HBM_PEAK_GBS, "mfma_f32_tflops": MFMA_PEAK_TFLOPS["fp32"],
                      "mfma_bf16_tflops": MFMA_PEAK_TFLOPS["bf16"], "lds_gbs": round(LDS_PEAK_GBS, 1)}
    out["how"] = ("best of 5 launches each: 1 GiB grid-stride copy / read with 16-byte accesses; 2048 workgroups x 4 "
                  "wavefronts x 16 (4 for 32x32x16) independent accumulators, no memory traffic; 512-thread workgroups "
                  "reading 3x3 windows of per-lane planes (odd pitch) with 4-byte LDS reads, one FMA per read")
    return out


def run_workload(args, name, machine, steps, warmup, headline):
    import numpy as np
    import torch
    from paper_1908_05460_amd import binding as B, inputs, schedule as sch

    cfg, stack_fn, N, dtype = inputs.WORKLOADS[name]
    stack = stack_fn()
    e = 2 if dtype == "bf16" else 4
    nl = len(stack)
    set_bytes = sum(exact_min_bytes(l, N, e) for l in stack)
    copies = args.copies or max(2, min(8, math.ceil(1e9 / set_bytes)))

    def to_gpu(a):
        t = torch.from_numpy(a)
        if a.dtype == np.uint16:
            t = t.view(torch.bfloat16)
        return t.cuda()

    descs = [B.desc_for(l, N, dtype) for l in stack]
    sets, host0, checksums = [], None, []
    for b in range(copies):
        data = [inputs.make_layer_inputs(l, N, config=cfg, batch=b, layer_index=i, dtype=dtype)
                for i, l in enumerate(stack)]
        if b == 0:
            host0 = data if headline else None
            checksums = [[f"{zlib.crc32(x.tobytes()):08x}", f"{zlib.crc32(y.tobytes()):08x}"] for x, y in data]
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

    def step(i, events=None, rotate=True):
        s = sets[i % copies if rotate else 0]
        if events: events[0].record()
        if "exact" in on: s.run(m_exact, ws)
        if events: events[1].record()
        if "approx" in on: s.run(m_approx, ws, scale=args.scale)
        if events: events[2].record()
        if "zero" in on: s.run(m_zero, ws)
        if events: events[3].record()
        if "random" in on: s.run(m_random, ws, sigma=1.0 / 128, seed=inputs.ROOT_SEED, offset=i * dw_total)
        if events: events[4].record()

    def timed_region(nsteps, rotate):
        ev = {i: [torch.cuda.Event(enable_timing=True) for _ in range(5)] for i in range(0, nsteps, every)}
        for i in range(warmup):
            step(i, rotate=rotate)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(nsteps):
            step(warmup + i, ev.get(i), rotate)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        samples = {p: [x[j].elapsed_time(x[j + 1]) for x in ev.values()] for j, p in enumerate(phases)}
        return (t1 - t0) * 1e3 / nsteps, samples

    ms_per_step, samples = timed_region(steps, True)
    phase_ms = {p: max(float(np.median(v)), 1e-6) for p, v in samples.items()}
    phase_min = {p: max(float(np.min(v)), 1e-6) for p, v in samples.items()}
    # the same steps on ONE input set: operands of a step that fit the 256 MB last-level cache are found there
    _, warm_samples = timed_region(max(10, steps // 2), False)
    phase_warm = {p: max(float(np.median(v)), 1e-6) for p, v in warm_samples.items()}

    # ---- per-layer pass: groups of back-to-back launches of one layer between one event pair,
    #      rotating the input sets, same launch configuration as the single-layer entry points ----
    reps = args.layer_reps
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    per_layer = []

    def time_layer(fn):
        """us per call: `reps` back-to-back calls between one event pair, issued from the host and replayed from a
        captured HIP graph (which takes the host's launch cost out); the smaller of the two."""
        for r in range(3):
            fn(r)
        torch.cuda.synchronize()
        a0.record()
        for r in range(reps):
            fn(r)
        a1.record()
        torch.cuda.synchronize()
        best = a0.elapsed_time(a1)
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for r in range(reps):
                    fn(r)
            graph.replay()
            torch.cuda.synchronize()
            for _ in range(3):
                a0.record(); graph.replay(); a1.record()
                torch.cuda.synchronize()
                best = min(best, a0.elapsed_time(a1))
            del graph
        return best * 1e3 / reps

    lds_roof = machine["lds_read_b32_gbs"] if machine else None
    tot = {"exact_us": 0.0, "approx_us": 0.0, "flops": 0.0, "valid_flops": 0.0, "approx_bytes": 0.0,
           "hbm_set_bytes": 0.0, "hbm_set_us": 0.0, "roof_us": 0.0, "exact_roof_us": 0.0, "exact_hbm_layers": []}
    seen_shapes = {}
    for i, l in enumerate(stack):
        d = descs[i]
        fl, vfl, ab = l.flops(N), l.valid_flops(N), approx_algorithmic_bytes(l, N, e)
        tot["flops"] += fl; tot["valid_flops"] += vfl; tot["approx_bytes"] += ab
        # the roof that binds the exact gradient of this layer: the matrix core for its nominal FLOPs, or HBM for its
        # operands where those take longer (few channels: 3->64, and 64->64 with bf16 inputs)
        t_ex_mm, t_ex_hbm = fl / (MFMA_PEAK_TFLOPS[dtype] * 1e6), exact_min_bytes(l, N, e) / (HBM_PEAK_GBS * 1e3)
        tot["exact_roof_us"] += max(t_ex_mm, t_ex_hbm)
        if t_ex_hbm > t_ex_mm: tot["exact_hbm_layers"].append(l.name)
        if reps <= 0:       # counter runs: no single-layer calls
            continue
        key = (l.C, l.K, l.H, l.stride)
        if not headline and key in seen_shapes:     # nested configurations: one row per distinct layer shape
            seen_shapes[key]["layers"].append(l.name)
            row = seen_shapes[key]
            tot["exact_us"] += row["exact_us"]; tot["approx_us"] += row["approx_us"]; tot["roof_us"] += row["approx_roof_us"]
            continue
        X_ = lambda r: sets[r % copies]._keep[0][i]
        dY_ = lambda r: sets[r % copies]._keep[1][i]
        dW_ = lambda r: sets[r % copies]._keep[2][i]
        t_ex = time_layer(lambda r: B.conv_wgrad_exact(d, X_(r), dY_(r), dW=dW_(r), ws=ws))
        t_ap = time_layer(lambda r: B.conv_wgrad_approx(d, X_(r), dY_(r), scale=args.scale, dW=dW_(r), ws=ws))
        idx_t = torch.empty((N, l.K), dtype=torch.int32, device="cuda")
        sum_t = torch.empty((N, l.K), dtype=torch.float32, device="cuda")
        t_sel = time_layer(lambda r: B.conv_wgrad_select(d, dY_(r), idx_t, sum_t))
        sel_bytes = N * l.K * l.Ho * l.Wo * e
        # The roof that binds the approximation of this layer: HBM for its algorithmic bytes; or, where that takes
        # longer, the cheaper of the two ways to apply the patches -- the gathered operand read out of LDS (measured
        # LDS rate of this run) or the matrix core contracting the sparsified dY (Section 2.4's identity; valid-tap
        # FLOPs at the published peak).
        t_hbm = ab / (HBM_PEAK_GBS * 1e3)                    # us
        t_lds = gather_bytes(l, N, 4) / (lds_roof * 1e3) if lds_roof else float("inf")
        t_mm = vfl / (MFMA_PEAK_TFLOPS[dtype] * 1e6)
        t_apply = min(t_lds, t_mm)
        bound = "hbm" if t_hbm >= t_apply else ("lds" if t_lds <= t_mm else "mfma")
        t_roof = max(t_hbm, t_apply)
        row = {"layer": l.name, "layers": [l.name], "shape": f"{l.C}->{l.K}@{l.H}s{l.stride}",
               "exact_us": round(t_ex, 2), "approx_us": round(t_ap, 2), "select_us": round(t_sel, 2),
               "exact_tflops": round(fl / t_ex / 1e6, 2), "exact_valid_tflops": round(vfl / t_ex / 1e6, 2),
               "exact_frac_mfma": round(fl / t_ex / 1e6 / MFMA_PEAK_TFLOPS[dtype], 4),
               "exact_bound": "hbm" if t_ex_hbm > t_ex_mm else "mfma", "exact_roof_us": round(max(t_ex_mm, t_ex_hbm), 2),
               "approx_gbs": round(ab / t_ap / 1e3, 1),
               "approx_frac_hbm": round(ab / t_ap / 1e3 / HBM_PEAK_GBS, 4),
               "approx_bound": bound, "approx_roof_us": round(t_roof, 2),
               "approx_frac_of_binding_roof": round(t_roof / t_ap, 4),
               "select_gbs": round(sel_bytes / t_sel / 1e3, 1),
               "select_frac_hbm": round(sel_bytes / t_sel / 1e3 / HBM_PEAK_GBS, 4),
               "speedup": round(t_ex / t_ap, 2)}
        if headline:
            topk = min(args.topk, d.Ho * d.Wo)
            if topk > 0:
                ws_k = B.alloc_workspace(B.topk_workspace_bytes(d, topk))
                t_tk = time_layer(lambda r: B.conv_wgrad_approx_topk(d, X_(r), dY_(r), topk, scale=args.scale, dW=dW_(r), ws=ws_k))
                row["topk"] = topk; row["topk_us"] = round(t_tk, 2)
            if not args.no_layouts:
                # the paper's route inside an NCHW framework: transpose X, channel-last kernel (OHWI result), transpose dW
                Xn = [B.conv_wgrad_transpose_x(d, sets[c]._keep[0][i], True) for c in range(min(copies, 2))]
                ws_n = B.alloc_workspace(B.nhwc_workspace_bytes(d, B.APPROX))
                ohwi = torch.empty(B.dw_shape(d, B.DW_OHWI), dtype=torch.float32, device="cuda")
                hwio = torch.empty(B.dw_shape(d, B.DW_HWIO), dtype=torch.float32, device="cuda")
                t_k = time_layer(lambda r: B.conv_wgrad_approx_nhwc(d, Xn[r % len(Xn)], dY_(r), B.DW_OHWI,
                                                                   scale=args.scale, dW=ohwi, ws=ws_n))
                t_x = time_layer(lambda r: B.conv_wgrad_transpose_x(d, X_(r), True, out=Xn[r % len(Xn)]))
                t_w = time_layer(lambda r: B.conv_wgrad_permute_dw(d, ohwi, B.DW_OHWI, B.DW_HWIO, out=hwio))
                row.update({"nhwc_kernel_us": round(t_k, 2), "transpose_x_us": round(t_x, 2),
                            "transpose_dw_us": round(t_w, 2), "nhwc_total_us": round(t_k + t_x + t_w, 2)})
                del Xn, ws_n
        seen_shapes[key] = row
        per_layer.append(row)
        tot["exact_us"] += t_ex; tot["approx_us"] += t_ap; tot["roof_us"] += t_roof
    # which layers' approximation is bound by HBM (the set on which a fraction of HBM bandwidth means something)
    for row in per_layer:
        if row["approx_bound"] == "hbm":
            for lname in row["layers"]:
                l = next(x for x in stack if x.name == lname)
                tot["hbm_set_bytes"] += approx_algorithmic_bytes(l, N, e)
                tot["hbm_set_us"] += row["approx_us"]

    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        traffic = tj.get(name)
        traffic_src = tj.get("provenance")
    single = reps > 0
    achieved_tf = tot["flops"] / phase_ms["exact"] / 1e9
    mfma_measured = None
    if machine:
        mfma_measured = machine["mfma_f32_16x16x4_tflops"] if dtype == "fp32" else machine["mfma_bf16_16x16x32_tflops"]
    roofline = {"kernel": "exact phase = wgrad_exact_multi (fp32: all layer groups in one launch) | wgrad_exact_stream | wgrad_exact_bf16_multi + wgrad_exact_bf16_planes (bf16), + combine_table",
                "bound": "mfma", "achieved": round(achieved_tf, 3), "peak": MFMA_PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                "frac": round(achieved_tf / MFMA_PEAK_TFLOPS[dtype], 4),
                "traffic": traffic["exact_phase_bytes"] if traffic else None, "traffic_source": traffic_src if traffic else None,
                "peak_measured": mfma_measured,
                "frac_of_measured": round(achieved_tf / mfma_measured, 4) if mfma_measured else None,
                "achieved_valid_taps": round(tot["valid_flops"] / phase_ms["exact"] / 1e9, 3),
                "frac_valid_taps": round(tot["valid_flops"] / phase_ms["exact"] / 1e9 / MFMA_PEAK_TFLOPS[dtype], 4),
                "note": "achieved counts nominal FLOPs (padding taps included, the usual convention); the fp32 kernels leave out "
                        "matrix instructions whose taps meet only padding, so the matrix core's own rate is bounded by "
                        "achieved_valid_taps (products that do not multiply padding) from below and achieved from above",
                "achieved_best": round(tot["flops"] / phase_min["exact"] / 1e9, 3),
                "algorithmic_flops": tot["flops"], "valid_tap_flops": tot["valid_flops"],
                "algorithmic_min_bytes": sum(exact_min_bytes(l, N, e) for l in stack),
                "binding_roofs": {"note": "sum over the layers of max(nominal FLOPs / matrix-core peak, minimal bytes / HBM peak) against the phase time",
                                  "sum_roof_us": round(tot["exact_roof_us"], 1), "hbm_bound_layers": tot["exact_hbm_layers"],
                                  "frac": round(tot["exact_roof_us"] / (phase_ms["exact"] * 1e3), 4)},
                "layers": nl, "phase_us": round(phase_ms["exact"] * 1e3, 1), "phase_us_min": round(phase_min["exact"] * 1e3, 1),
                "single_layer_calls": {"sum_us": round(tot["exact_us"], 1),
                                       "tflops": round(tot["flops"] / tot["exact_us"] / 1e6, 2)} if single else None}
    achieved_gbs = tot["approx_bytes"] / phase_ms["approx"] / 1e6
    read_measured = machine["hbm_read_gbs"] if machine else None
    roofline_approx = {"kernel": "approx phase = approx_fused_multi | approx_select_multi + (approx_gather_lds_multi | approx_gather_direct | wgrad_exact_bf16_multi<SPARSE>) | sparsify_small + wgrad_exact_plane2, + combine_table",
                       "bound": "hbm", "achieved": round(achieved_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(achieved_gbs / HBM_PEAK_GBS, 4),
                       "traffic": traffic["approx_phase_bytes"] if traffic else None, "traffic_source": traffic_src if traffic else None,
                       "peak_measured": read_measured,
                       "frac_of_measured": round(achieved_gbs / read_measured, 4) if read_measured else None,
                       "algorithmic_bytes": tot["approx_bytes"], "layers": nl,
                       "phase_us": round(phase_ms["approx"] * 1e3, 1), "phase_us_min": round(phase_min["approx"] * 1e3, 1),
                       "binding_roofs": {"note": "sum over the layers of each layer's binding roof (HBM, or LDS reads / matrix core where "
                                                 "applying the patches takes longer than streaming the bytes) against the phase time",
                                         "sum_roof_us": round(tot["roof_us"], 1),
                                         "frac": round(tot["roof_us"] / (phase_ms["approx"] * 1e3), 4)} if single else None,
                       "hbm_bound_layers": {"note": "single-layer calls of the layers whose binding roof is HBM, not the LDS reads of the gather",
                                            "layers": [n_ for r_ in per_layer if r_["approx_bound"] == "hbm" for n_ in r_["layers"]],
                                            "gbs": round(tot["hbm_set_bytes"] / tot["hbm_set_us"] / 1e3, 1),
                                            "frac": round(tot["hbm_set_bytes"] / tot["hbm_set_us"] / 1e3 / HBM_PEAK_GBS, 4)}
                                           if single and tot["hbm_set_us"] > 0 else None,
                       "single_layer_calls": {"sum_us": round(tot["approx_us"], 1),
                                              "gbs": round(tot["approx_bytes"] / tot["approx_us"] / 1e3, 1)} if single else None}

    # ---- the oracle on the host cores, bounded sample of the same workload ----
    cpu = None
    if headline and args.cpu_budget_s > 0:
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

    res = {
        "ms_per_step": round(ms_per_step, 4), "steps": steps, "warmup": warmup,
        "dtype": "f32" if dtype == "fp32" else "bf16 in, f32 accumulate",
        "config": {"workload": name, "layers": nl, "batch": N, "input_sets_rotated": copies,
                   "step": " + ".join(p for p in phases if p in on) + " gradient of every layer"
                           + ("" if len(on) == 4 else "  (PARTIAL STEP: not a benchmark result)")},
        "phase_ms": {k: round(v, 4) for k, v in phase_ms.items()},
        "phase_ms_min": {k: round(v, 4) for k, v in phase_min.items()},
        "phase_ms_warm_cache": {"note": "one input set reused by every step: operands that fit the 256 MB last-level cache are found there",
                                **{k: round(v, 4) for k, v in phase_warm.items()}},
        "speedup_approx_vs_exact": round(phase_ms["exact"] / phase_ms["approx"], 3),
        "roofline": roofline, "roofline_approx": roofline_approx, "cpu_baseline": cpu,
        "per_layer": per_layer,
        "input_checksums_crc32": {"note": "input set 0, per layer [X, dY]", "values": checksums},
    }
    del sets, ws
    torch.cuda.empty_cache()
    return res


def run_sweep(args, name):
    """Approximation-schedule sweep: every mini-batch of a resident set runs the weight-gradient phase
    with the per-layer methods its schedule mask gives (one conv_wgrad_schedule_run per batch)."""
    import numpy as np
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from paper_1908_05460_amd import binding as B, inputs, schedule as sch

    cfg, stack_fn, N, dtype = inputs.WORKLOADS[name]
    stack = stack_fn()
    nl = len(stack)
    nb = args.sweep_batches or (100 if name.startswith("resnet20") else 24)
    descs = [B.desc_for(l, N, dtype) for l in stack]

    def make(b):
        return [inputs.make_layer_inputs(l, N, config=cfg, batch=b, layer_index=i, dtype=dtype) for i, l in enumerate(stack)]

    sets = []
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:     # numpy's generators release the GIL
        for lo in range(0, nb, 16):
            for data in ex.map(make, range(lo, min(nb, lo + 16))):
                sets.append(B.Schedule(descs, [torch.from_numpy(x).cuda() for x, _ in data],
                                       [torch.from_numpy(y).cuda() for _, y in data],
                                       [torch.empty((l.K, l.C, l.R, l.S), device="cuda") for l in stack]))
    masks = dict(sch.SWEEP_MASKS); masks.update(sch.PAPER_SCHEDULES)
    rows = {mname: [fn(nl, b) for b in range(nb)] for mname, fn in masks.items()}
    ws = B.alloc_workspace(max(sets[0].workspace_bytes(r) for rr in rows.values() for r in rr[:4]))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    result = {}
    t_start = time.perf_counter()
    for mname, rr in rows.items():
        for b in range(min(nb, 8)):                       # warm-up
            sets[b].run(rr[b], ws, scale=args.scale)
        torch.cuda.synchronize()
        e0.record()
        for b in range(nb):
            sets[b].run(rr[b], ws, scale=args.scale)
        e1.record()
        torch.cuda.synchronize()
        result[mname] = {"ms_per_iter": round(e0.elapsed_time(e1) / nb, 4),
                         "fraction_approximated": round(sch.fraction_approximated(masks[mname], nl, nb), 4)}
    wall = time.perf_counter() - t_start
    base = result["all_exact"]["ms_per_iter"]
    for v in result.values():
        v["vs_all_exact"] = round(v["ms_per_iter"] / base, 4)
    flops = sum(l.flops(N) for l in stack)
    res = {"ms_per_step": base, "steps": nb, "warmup": min(nb, 8), "dtype": "f32",
           "config": {"workload": name, "layers": nl, "batch": N, "resident_batches": nb,
                      "step": "one conv_wgrad_schedule_run per mini-batch; ms_per_step = the all-exact mask"},
           "sweep": result,
           "roofline": {"kernel": "all-exact mask: exact phase of every batch", "bound": "mfma",
                        "achieved": round(flops / base / 1e9, 3), "peak": MFMA_PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                        "frac": round(flops / base / 1e9 / MFMA_PEAK_TFLOPS[dtype], 4), "traffic": None},
           "timed_wall_s": round(wall, 2),
           "paper_context": "paper: schedules approximate 25% of (layer, batch) pairs; its end-to-end bound for that is ~8%"}
    del sets, ws
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline workload: no machine ceilings and no nested results of the other configurations")
    ap.add_argument("--copies", type=int, default=0, help="distinct input sets to rotate (0 = enough for 1 GB)")
    ap.add_argument("--layer-reps", type=int, default=20, help="back-to-back launches per layer in the per-layer pass")
    ap.add_argument("--cpu-budget-s", type=float, default=20.0, help="CPU seconds to spend on the oracle baseline (0 = skip)")
    ap.add_argument("--event-every", type=int, default=5,
                    help="timed steps between two steps whose phases are bracketed by HIP events (an event pair "
                         "drains the stream: five per step cost 25 us of a 205 us step)")
    ap.add_argument("--no-graph", action="store_true",
                    help="per-layer pass: time host-issued launches only (no replay from a captured HIP graph)")
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
    from paper_1908_05460_amd import binding as B, inputs

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
    t_begin = time.perf_counter()
    counter_run = args.layer_reps <= 0 or args.phases != "exact,approx,zero,random"
    extras = not args.no_extras and not counter_run
    machine = measure_machine(torch) if extras else None
    if args.workload.endswith("_schedule_sweep"):
        head = run_sweep(args, args.workload)
    else:
        head = run_workload(args, args.workload, machine, args.steps, args.warmup, headline=True)
    configs = {}
    if extras:
        for name in OTHER_CONFIGS + (HEADLINE,):
            if name == args.workload:
                continue
            if name.endswith("_schedule_sweep"):
                configs[name] = run_sweep(args, name)
            else:
                configs[name] = run_workload(args, name, machine, max(20, args.steps // 2), args.warmup, headline=False)
    out = {
        "metric": "weight-grad ms/iter (exact vs approx)", "value": head["ms_per_step"], "unit": "ms",
        "n_gpus": 1, "steps": head["steps"], "warmup": head["warmup"], "ms_per_step": head["ms_per_step"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"],
        "data": "synthetic",
    }
    out.update({k: v for k, v in head.items() if k not in ("ms_per_step", "steps", "warmup", "dtype")})
    out.setdefault("cpu_baseline", None)
    out["machine"] = machine
    out["configs"] = configs
    out["numpy_version"] = np.__version__
    out["inputs"] = ("numpy.random.default_rng(SeedSequence([%d, config, batch, layer, tensor])).standard_normal(float32): "
                     "X = max(z, 0), dY = 0.01 z; bf16 = one round-to-nearest-even of those" % inputs.ROOT_SEED)
    out["wall_s"] = round(time.perf_counter() - t_begin, 1)
    out["paper_context"] = ("paper: approx kernel incl. transposes >= 3x faster than cuDNN 7.4.2 backward-filter "
                            "on a Titan Xp for most layers; end-to-end training speedup 3.5% (ResNet-20) to ~7%")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
