#!/usr/bin/env python3
"""Benchmark of the W4A16 linear-layer hot path on one MI355X.

One step = one pass of the quantised linear layers (Eq. 3 of arXiv 2312.03788) of a whole
Code Llama-34B-shaped decoder stack at decode batch M=16: 48 layers x 4 merged linears
(8192->10240, 8192->8192, 8192->44032, 22016->8192), every layer with its own packed
int4 weights (17.3 GB resident in HBM, so each GEMM streams from HBM, not from cache).
The weights are produced on the GPU by the library's own smoothing + quantise/pack
kernels from seeded synthetic fp16 weights (N(0, 0.02)) and activations with 1 % outlier
channels (x50); the timed region contains only sqp_w4a16_gemm launches.

Prints ONE JSON line: whole-job GB/s of algorithmic bytes (4-bit codes + fp16 step +
4-bit zero point per group + fp16 X and Y), a `roofline` object for the decode kernel and a
`cpu_baseline` object (the CPU oracle timed on a bounded sample of the same workload).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2516.6

# HBM bytes per decode launch (averaged over the four shapes of the sweep) from the rocprofv3
# FETCH_SIZE / WRITE_SIZE runs summarised in the profile file below (34B shapes, M=16).  The
# figure belongs to the launch plans listed with it: if the library picks another plan for one
# of these shapes the figure is stale and the run stops, so that the profile gets refreshed.
TRAFFIC_PROFILE = "profiles/w4a16_decode_34b_m16_hbm_traffic.md"
TRAFFIC_BYTES_PER_LAUNCH = 103.1e6
TRAFFIC_PLANS = {(8192, 10240): (2, 3), (8192, 8192): (2, 4), (8192, 44032): (4, 4), (22016, 8192): (2, 4)}  # (strips, K parts)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--model", default="34b", choices=["7b", "13b", "34b"])
    ap.add_argument("--m", type=int, default=16, help="decode rows")
    ap.add_argument("--layers", type=int, default=0, help="0 = the model's layer count")
    ap.add_argument("--no-graph", action="store_true", help="launch from Python instead of replaying a HIP graph")
    ap.add_argument("--no-extra", action="store_true", help="skip the M=1 / prefill / companion side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (known size: calibrates the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2312_03788_amd as sqp
    import workloads as wl

    sqp.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    shapes = wl.MODEL_SHAPES[args.model]
    nlayers = args.layers or wl.MODEL_LAYERS[args.model]
    M = args.m
    G = wl.GROUP

    # ---- resident quantised model, built with the library's own kernels
    gen = torch.Generator(device=dev)
    outl = {K: torch.from_numpy(wl.outlier_channels(K)).to(dev) for K, _ in shapes}

    def activation(m, K, seed):
        gen.manual_seed(seed)
        x = torch.randn((m, K), device=dev, generator=gen, dtype=torch.float32)
        x[:, outl[K]] *= 50.0
        return x.half()

    t_build = time.time()
    layers = []      # per layer: list of (packed, scales, zeros)
    s_first = {}     # smoothing factors of layer 0, per shape (for the activations)
    for layer in range(nlayers):
        per = []
        for si, (K, N) in enumerate(shapes):
            gen.manual_seed(1000 + 16 * layer + si)
            w = (torch.randn((K, N), device=dev, generator=gen, dtype=torch.float32) * 0.02).half()
            xcal = activation(wl.T_CAL, K, 3000)
            s = sqp.smooth_scales(xcal, w, wl.ALPHA)
            sqp.smooth_apply_w(w, s, out=w)
            per.append(sqp.quantize_pack(w, G))
            if layer == 0:
                s_first[si] = s
            del w, xcal
        layers.append(per)
    xs = []
    for si, (K, N) in enumerate(shapes):
        xs.append(sqp.smooth_apply_x(activation(M, K, 2000 + M), s_first[si]))
    ys = [torch.empty((M, N), device=dev, dtype=torch.float16) for (K, N) in shapes]
    torch.cuda.synchronize()
    t_build = time.time() - t_build

    traffic = None
    if args.model == "34b" and M == 16:
        import ctypes
        L = sqp.lib()
        for (K, N) in shapes:
            nw, split, kspg = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
            L.sqp_debug_decode_plan(M, N, K, G, ctypes.byref(nw), ctypes.byref(split), ctypes.byref(kspg))
            if (nw.value, split.value) != TRAFFIC_PLANS[(K, N)]:
                sys.exit("bench.py: the launch plan of %d->%d is now %s, but %s was taken with %s: refresh the profile and "
                         "TRAFFIC_* in bench.py" % (K, N, (nw.value, split.value), TRAFFIC_PROFILE, TRAFFIC_PLANS[(K, N)]))
        traffic = TRAFFIC_BYTES_PER_LAUNCH

    launches_per_step = nlayers * len(shapes)
    bytes_per_step = nlayers * sum(wl.algorithmic_bytes(M, N, K, G) for (K, N) in shapes)

    def step():
        for per in layers:
            for si, (p, sc, z) in enumerate(per):
                sqp.w4a16_gemm(xs[si], p, sc, z, G, out=ys[si])

    if args.calib_copy:
        import ctypes
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        L = sqp.lib()
        L.sqp_debug_plain_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        for _ in range(3):
            rc = L.sqp_debug_plain_copy(src.data_ptr(), dst.data_ptr(), src.numel() * 4,
                                        torch.cuda.current_stream().cuda_stream)
            assert rc == 0
        torch.cuda.synchronize()
        del src, dst

    # the library allocates nothing: hand it a workspace for its split launches that covers
    # every shape of this run (decode rows of the sweep, the side measurements' M = 1 and 2048)
    ws_need = max(sqp.workspace_bytes(m, N, K, G) for (K, N) in shapes for m in (1, M, 16, 32, 64, 65, 128, 256, 2048, 4096))
    sqp.set_workspace(max(ws_need, 64 << 20))
    torch.cuda.synchronize()
    graph = None
    if not args.no_graph:
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                step()
        torch.cuda.synchronize()
    run = graph.replay if graph is not None else step

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = wall * 1e3 / args.steps
    value = bytes_per_step / (wall / args.steps) / 1e9

    # dominant kernel: the decode GEMM; average launch duration from the HIP events
    avg_launch_s = ev_ms * 1e-3 / (args.steps * launches_per_step)
    bytes_per_launch = bytes_per_step / launches_per_step
    achieved = bytes_per_launch / avg_launch_s / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": TRAFFIC_PROFILE if traffic else None,
                "kernel": "w4a16_decode_kernel", "avg_launch_us": round(avg_launch_s * 1e6, 2),
                "algorithmic_bytes_per_launch": round(bytes_per_launch)}

    extra, roofline_prefill = {}, None
    if not args.no_extra:
        extra, roofline_prefill = side_measurements(torch, sqp, wl, dev, shapes, layers, s_first, activation, G, M)

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(np, torch, wl, shapes, layers, xs, M, G)
        if not args.no_extra:
            cpu["other_kernels"] = cpu_baseline_other(np, torch, sqp, wl, dev, shapes, layers, s_first, activation, G, extra)

    out = {
        "metric": "W4A16 GEMM: HBM GB/s at M<=16 (% of peak); TFLOP/s at M=2048 (% MFMA)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 x int4 -> f32 accumulate", "data": "synthetic",
        "config": {"workload": "Code Llama-%s-shaped decode sweep, M=%d, %d layers x 4 linears, group 128, "
                               "weights resident (%.2f GB algorithmic per step)" % (args.model.upper(), M, nlayers, bytes_per_step / 1e9),
                   "launch": "hip-graph replay" if graph is not None else "python launches",
                   "build_s": round(t_build, 1)},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
        "roofline": roofline,
        "roofline_prefill": roofline_prefill,
        "cpu_baseline": cpu,
        "extra": extra,
    }
    print(json.dumps(out))


def _time(torch, fn, iters):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / iters


def _graph_time(torch, fn, iters):
    """Seconds per call of fn when fn's launches are replayed from a HIP graph."""
    fn()
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            fn()
    torch.cuda.synchronize()
    return _time(torch, graph.replay, iters)


def side_measurements(torch, sqp, wl, dev, shapes, layers, s_first, activation, G, M_decode):
    """Context figures outside the headline: the decode sweep by layer shape and at M=1, the
    tiled path at M=2048 and 4096 (TFLOP/s against the fp16 MFMA peak: the second half of the
    metric, returned as its own roofline object), the row counts around the switch between the
    two paths, on-chip reference rates (plain copy, plain read, MFMA-only loop) and the
    companion kernels on the 22016x8192 weight."""
    import ctypes
    extra = {}
    L = sqp.lib()
    # the headline sweep, one layer shape at a time (graph replay over the resident layers)
    by_shape = {}
    for si, (K, N) in enumerate(shapes):
        x = sqp.smooth_apply_x(activation(M_decode, K, 2000 + M_decode), s_first[si])
        y = torch.empty((M_decode, N), device=dev, dtype=torch.float16)

        def sweep_one():
            for per in layers:
                p, sc, z = per[si]
                sqp.w4a16_gemm(x, p, sc, z, G, out=y)
        t = _graph_time(torch, sweep_one, 5) / len(layers)
        b = wl.algorithmic_bytes(M_decode, N, K, G)
        by_shape["%dx%d" % (K, N)] = {"us": round(t * 1e6, 2), "gbs": round(b / t / 1e9, 1), "pct_hbm_peak": round(100 * b / t / 1e9 / HBM_PEAK_GBS, 1)}
    extra["decode_m%d_by_shape" % M_decode] = by_shape
    # decode with fewer rows (up to 8 rows take the column-slice kernel) over all resident layers,
    # and by layer shape at M = 1
    for M in (1, 8):
        xs = [sqp.smooth_apply_x(activation(M, K, 2000 + M), s_first[si]) for si, (K, N) in enumerate(shapes)]
        ys = [torch.empty((M, N), device=dev, dtype=torch.float16) for (K, N) in shapes]

        def sweep():
            for per in layers:
                for si, (p, sc, z) in enumerate(per):
                    sqp.w4a16_gemm(xs[si], p, sc, z, G, out=ys[si])
        t = _graph_time(torch, sweep, 3)
        b = len(layers) * sum(wl.algorithmic_bytes(M, N, K, G) for (K, N) in shapes)
        extra["decode_m%d_gbs" % M] = round(b / t / 1e9, 1)
        extra["decode_m%d_pct_hbm_peak" % M] = round(100 * b / t / 1e9 / HBM_PEAK_GBS, 2)
        if M == 1:
            by_shape = {}
            for si, (K, N) in enumerate(shapes):
                def sweep_one():
                    for per in layers:
                        p, sc, z = per[si]
                        sqp.w4a16_gemm(xs[si], p, sc, z, G, out=ys[si])
                t1 = _graph_time(torch, sweep_one, 5) / len(layers)
                b1 = wl.algorithmic_bytes(M, N, K, G)
                by_shape["%dx%d" % (K, N)] = {"us": round(t1 * 1e6, 2), "gbs": round(b1 / t1 / 1e9, 1),
                                              "pct_hbm_peak": round(100 * b1 / t1 / 1e9 / HBM_PEAK_GBS, 1),
                                              "kernel": ("strips", "slices of 32 columns", "slices of 64 columns")[1 + L.sqp_debug_decode_slice_choice(M, N, K, G)]}
            extra["decode_m1_by_shape"] = by_shape
    # the tiled path at M = 2048 and 4096, the four shapes, rotating over resident layers; the
    # average launch duration comes from HIP events around the timed launches
    roofline_prefill = None
    for M in (2048, 4096):
        pre = {}
        flops_total, t_total = 0.0, 0.0
        for si, (K, N) in enumerate(shapes):
            x = sqp.smooth_apply_x(activation(M, K, 2000 + M), s_first[si])
            y = torch.empty((M, N), device=dev, dtype=torch.float16)
            nl = min(len(layers), 8)
            state = {"i": 0}

            def one():
                p, sc, z = layers[state["i"] % nl][si]
                state["i"] += 1
                sqp.w4a16_gemm(x, p, sc, z, G, out=y)
            t = _time(torch, one, nl)
            fl = wl.gemm_flops(M, N, K)
            pre["%dx%d" % (K, N)] = {"tflops": round(fl / t / 1e12, 1), "avg_launch_us": round(t * 1e6, 1),
                                     "pct_mfma_peak": round(100 * fl / t / 1e12 / MFMA_F16_PEAK_TFLOPS, 1)}
            flops_total += fl
            t_total += t
            del x, y
        agg = flops_total / t_total / 1e12
        obj = {"bound": "mfma", "achieved": round(agg, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
               "frac": round(agg / MFMA_F16_PEAK_TFLOPS, 4), "traffic": None, "kernel": "w4a16_prefill_kernel",
               "workload": "34B shapes at M=%d, one call per shape and layer, flops 2MNK" % M, "by_shape": pre}
        if M == 2048:
            roofline_prefill = obj
            extra["prefill_m2048_tflops"] = round(agg, 1)
            extra["prefill_m2048_pct_mfma_peak"] = round(100 * agg / MFMA_F16_PEAK_TFLOPS, 2)
        else:
            roofline_prefill["m4096"] = {k: obj[k] for k in ("achieved", "frac", "by_shape")}
    # where the two paths meet: one 34B shape (8192 -> 8192) at row counts around the switch at 64
    K, N = shapes[1]
    cross = {}
    for M in (16, 32, 64, 65, 128, 256):
        x = sqp.smooth_apply_x(activation(M, K, 2000 + M), s_first[1])
        y = torch.empty((M, N), device=dev, dtype=torch.float16)

        def sweep_m():
            for per in layers[:16]:
                p, sc, z = per[1]
                sqp.w4a16_gemm(x, p, sc, z, G, out=y)
        cross["m%d_us" % M] = round(_graph_time(torch, sweep_m, 5) / 16 * 1e6, 2)
    extra["crossover_8192x8192_us"] = cross
    # the fallback for group sizes the matrix-core kernels do not cover (one thread per output
    # element): group 24 on a 3072 -> 4096 layer at M = 16, random codes
    Kg, Ng, Gg = 3072, 4096, 24
    gen_g = torch.Generator(device=dev)
    gen_g.manual_seed(5)
    pg = torch.randint(-2**31, 2**31 - 1, (Kg // 8, Ng), dtype=torch.int32, device=dev, generator=gen_g)
    scg = (torch.rand((Kg // Gg, Ng), device=dev, generator=gen_g) * 0.004 + 0.003).half()
    zg = torch.randint(0, 16, (Kg // Gg, Ng), dtype=torch.uint8, device=dev, generator=gen_g)
    xg24 = torch.randn((16, Kg), device=dev, generator=gen_g).half()
    yg24 = torch.empty((16, Ng), device=dev, dtype=torch.float16)
    t = _time(torch, lambda: sqp.w4a16_gemm(xg24, pg, scg, zg, Gg, out=yg24), 10)
    extra["generic_kernel_group24_3072x4096_m16_us"] = round(t * 1e6, 1)
    del pg, scg, zg, xg24, yg24
    # on-chip reference rates: the plain copy kernel that calibrates the traffic counters and a
    # plain streaming read with and without the non-temporal hint, 2 GiB each
    L.sqp_debug_plain_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.sqp_debug_read_probe.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    big = torch.zeros(1 << 29, dtype=torch.float32, device=dev)
    dst = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    sink4 = torch.zeros(4, dtype=torch.int32, device=dev)
    stq = torch.cuda.current_stream().cuda_stream

    def copy1():
        assert L.sqp_debug_plain_copy(big.data_ptr(), dst.data_ptr(), dst.numel() * 4, stq) == 0
    t = _time(torch, copy1, 5)
    extra["plain_copy_gbs_read_plus_write"] = round(2.0 * dst.numel() * 4 / t / 1e9, 1)
    for nt in (0, 1):  # 768 workgroups = three per compute unit: the grid that reads fastest
        def read1():
            assert L.sqp_debug_read_probe(big.data_ptr(), big.numel() * 4, nt, 768, sink4.data_ptr(), stq) == 0
        t = _time(torch, read1, 5)
        extra["read_probe_%s_gbs" % ("nt" if nt else "plain")] = round(big.numel() * 4 / t / 1e9, 1)
    del big, dst
    # what the matrix cores sustain on this chip with nothing else to do: a loop of independent
    # 32x32x16 fp16 MFMAs on one of the activations above (the clock settles under the power limit)
    L.sqp_debug_mfma_ceiling.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    data = sqp.smooth_apply_x(activation(16, shapes[0][0], 2016), s_first[0])  # >= 64 KiB of smoothed activations
    blocks, iters = 256, 20000
    sink = torch.empty(blocks * 256, device=dev, dtype=torch.float32)
    st = torch.cuda.current_stream().cuda_stream

    def mf():
        rc = L.sqp_debug_mfma_ceiling(data.data_ptr(), sink.data_ptr(), blocks, iters, st)
        assert rc == 0
    t = _time(torch, mf, 3)
    extra["mfma_only_loop_tflops"] = round(blocks * 4 * iters * 16 * 32768.0 / t / 1e12, 1)
    del data, sink
    # companion kernels on the largest weight (22016 x 8192)
    K, N = shapes[3]
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    w = (torch.randn((K, N), device=dev, generator=gen, dtype=torch.float32) * 0.02).half()
    xcal = activation(wl.T_CAL, K, 3000)
    s = torch.empty(K, device=dev, dtype=torch.float32)
    t = _time(torch, lambda: sqp.smooth_scales(xcal, w, wl.ALPHA, out=s), 5)
    extra["smooth_scales_22016x8192_us"] = round(t * 1e6, 1)
    extra["smooth_scales_gbs"] = round((2.0 * K * N + 2.0 * wl.T_CAL * K) / t / 1e9, 1)
    out = sqp.quantize_pack(w, G)
    t = _time(torch, lambda: sqp.quantize_pack(w, G, out=out), 5)
    extra["quantize_pack_22016x8192_us"] = round(t * 1e6, 1)
    extra["quantize_pack_gbs"] = round((2.0 * K * N + K * N * (0.5 + 3.0 / G)) / t / 1e9, 1)
    # single-layer search for the smoothing strength (Eq. 4 over 21 values of alpha) on the
    # 8192 -> 8192 linear with the 512 calibration rows
    K2, N2 = shapes[1]
    w2 = (torch.randn((K2, N2), device=dev, generator=gen, dtype=torch.float32) * 0.02).half()
    xcal2 = activation(wl.T_CAL, K2, 3000)
    s2 = torch.empty(K2, device=dev, dtype=torch.float32)
    sqp.smooth_scales(xcal2, w2, wl.ALPHA, out=s2)
    xh2 = sqp.smooth_apply_x(xcal2, s2)
    q2 = sqp.quantize_pack(sqp.smooth_apply_w(w2, s2), G)
    lo = torch.empty(1, device=dev, dtype=torch.float64)
    t = _time(torch, lambda: sqp.quant_loss(xcal2, w2, xh2, q2[0], q2[1], q2[2], G, out=lo), 5)
    extra["quant_loss_%dx%dx%d_us" % (wl.T_CAL, K2, N2)] = round(t * 1e6, 1)
    extra["quant_loss_tflops"] = round(4.0 * wl.T_CAL * K2 * N2 / t / 1e12, 1)
    t0 = time.time()
    best, curve = sqp.alpha_search(xcal2, w2, G)
    torch.cuda.synchronize()
    extra["alpha_search_21_ms"] = round((time.time() - t0) * 1e3, 1)
    extra["alpha_search_best"] = round(best, 2)
    # the merged gate/up projection with SiLU(gate) * up fused into the store, against the plain
    # GEMM on the same weights (8192 -> 44032, M = 16, rotating over the resident layers)
    Kg, Ng = shapes[2]
    xg = sqp.smooth_apply_x(activation(16, Kg, 2016), s_first[2])
    yg = torch.empty((16, Ng), device=dev, dtype=torch.float16)
    hg = torch.empty((16, Ng // 2), device=dev, dtype=torch.float16)
    nlg = len(layers)
    stg = {"i": 0}

    def plain():
        pq, scq, zq = layers[stg["i"] % nlg][2]
        stg["i"] += 1
        sqp.w4a16_gemm(xg, pq, scq, zq, G, out=yg)

    def fused():
        pq, scq, zq = layers[stg["i"] % nlg][2]
        stg["i"] += 1
        sqp.w4a16_gemm_silu_mul(xg, pq, scq, zq, G, out=hg)
    extra["gate_up_m16_plain_us"] = round(_time(torch, plain, nlg) * 1e6, 1)
    extra["gate_up_m16_silu_fused_us"] = round(_time(torch, fused, nlg) * 1e6, 1)
    xn = activation(2048, Kg, 4048)
    gm = torch.ones(Kg, device=dev, dtype=torch.float16)
    yn = torch.empty_like(xn)
    t = _time(torch, lambda: sqp.rmsnorm(xn, gm, 1e-5, out=yn), 5)
    extra["rmsnorm_2048x%d_us" % Kg] = round(t * 1e6, 1)
    extra["rmsnorm_gbs"] = round(4.0 * 2048 * Kg / t / 1e9, 1)
    del xg, yg, hg, xn, yn
    # context: the loss of plain round-to-nearest (no smoothing) on the same layer
    qr = sqp.quantize_pack(w2, G)
    e_rtn = float(sqp.quant_loss(xcal2, w2, xcal2, qr[0], qr[1], qr[2], G)[0])
    e_best = min(v for _, v in curve)
    extra["loss_rtn_over_best_alpha"] = round(e_rtn / e_best, 2)
    del w2, xcal2, xh2, q2, qr
    # the other two model sizes the configurations name (context: same kernel, same plan rule),
    # M = 16 sweeps over random codes/steps/zero points, replayed from a graph like the headline
    by_model = {}
    for model in ("7b", "13b"):
        if model not in wl.MODEL_SHAPES:
            continue
        mshapes, nl = wl.MODEL_SHAPES[model], wl.MODEL_LAYERS[model]
        gen.manual_seed(77)
        mlayers = []
        for _ in range(nl):
            per = []
            for (Km, Nm) in mshapes:
                p = torch.randint(-2**31, 2**31 - 1, (Km // 8, Nm), dtype=torch.int32, device=dev, generator=gen)
                sc = (torch.rand((Km // G, Nm), device=dev, generator=gen) * 0.004 + 0.003).half()
                z = torch.randint(0, 16, (Km // G, Nm), dtype=torch.uint8, device=dev, generator=gen)
                per.append((p, sc, z))
            mlayers.append(per)
        mx = [torch.randn((16, Km), device=dev, generator=gen, dtype=torch.float32).half() for (Km, Nm) in mshapes]
        my = [torch.empty((16, Nm), device=dev, dtype=torch.float16) for (Km, Nm) in mshapes]

        def msweep():
            for per in mlayers:
                for si, (p, sc, z) in enumerate(per):
                    sqp.w4a16_gemm(mx[si], p, sc, z, G, out=my[si])
        msweep()
        torch.cuda.synchronize()
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            mgraph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(mgraph, stream=stream):
                msweep()
        torch.cuda.synchronize()
        t = _time(torch, mgraph.replay, 5)
        b = nl * sum(wl.algorithmic_bytes(16, Nm, Km, G) for (Km, Nm) in mshapes)
        by_model[model] = {"gbs": round(b / t / 1e9, 1), "us_per_launch": round(t * 1e6 / (nl * len(mshapes)), 2)}
        del mgraph, mlayers, mx, my
    extra["decode_m16_other_models"] = by_model
    # context only (never a target): dense fp16 x fp16 GEMM of the vendor library through
    # torch.matmul at the same shapes, weights rotating over >= 1.5 GB so that they stream from HBM
    dense = {}
    for (Kd, Nd) in shapes:
        nl = max(2, int(1.5e9 / (2.0 * Kd * Nd)) + 1)
        ws = [(torch.randn((Kd, Nd), device=dev, generator=gen, dtype=torch.float32) * 0.02).half() for _ in range(nl)]
        for Md in (16, 2048):
            xd = activation(Md, Kd, 2000 + Md)
            yd = torch.empty((Md, Nd), device=dev, dtype=torch.float16)
            state = {"i": 0}

            def one():
                torch.matmul(xd, ws[state["i"] % nl], out=yd)
                state["i"] += 1
            t = _time(torch, one, 2 * nl)
            dense["%dx%d_m%d_us" % (Kd, Nd, Md)] = round(t * 1e6, 1)
        del ws
    extra["dense_fp16_vendor_gemm"] = dense
    return extra, roofline_prefill


def cpu_baseline(np, torch, wl, shapes, layers, xs, M, G):
    """The CPU oracle (fp32-accumulate variant, as it stands) on a bounded sample of the
    same workload: layer 0, the 8192->8192 and 8192->10240 linears, at the same M."""
    import oracle
    oracle.lib()
    nl = min(len(layers), 12)
    t_total, b_total = 0.0, 0.0
    for layer in range(nl):
        for si, (K, N) in enumerate(shapes):
            p, sc, z = layers[layer][si]
            x = xs[si].cpu().numpy()
            pn = p.cpu().numpy().view(np.uint32)
            scn = sc.cpu().numpy()
            zn = z.cpu().numpy()
            t0 = time.perf_counter()
            oracle.w4a16_gemm_f32(x, pn, scn, zn, G)
            t_total += time.perf_counter() - t0
            b_total += wl.algorithmic_bytes(M, N, K, G)
    return {"value": round(b_total / t_total / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "layers 0..%d of the same sweep (all 4 linears, M=%d), one call each: %.1f s of CPU time" %
                      (nl - 1, M, t_total)}


def cpu_baseline_other(np, torch, sqp, wl, dev, shapes, layers, s_first, activation, G, extra):
    """The oracle's companion functions on the same 22016 x 8192 weight the GPU figures in
    `extra` are quoted on, and its GEMM on 32 sampled rows of the M = 2048 call of 8192 -> 8192
    (extrapolated to 2048 rows: every row costs the same)."""
    import oracle
    out = {}
    K, N = shapes[3]
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    w = (torch.randn((K, N), device=dev, generator=gen, dtype=torch.float32) * 0.02).half().cpu().numpy()
    xcal = activation(wl.T_CAL, K, 3000).cpu().numpy()
    t0 = time.perf_counter()
    oracle.smooth_scales(xcal, w, wl.ALPHA)
    t = time.perf_counter() - t0
    out["smooth_scales_22016x8192"] = {"oracle_s": round(t, 2), "gpu_us": extra.get("smooth_scales_22016x8192_us"),
                                       "oracle_gbs": round((2.0 * K * N + 2.0 * wl.T_CAL * K) / t / 1e9, 2)}
    t0 = time.perf_counter()
    oracle.quantize_pack(w, G)
    t = time.perf_counter() - t0
    out["quantize_pack_22016x8192"] = {"oracle_s": round(t, 2), "gpu_us": extra.get("quantize_pack_22016x8192_us"),
                                       "oracle_gbs": round((2.0 * K * N + K * N * (0.5 + 3.0 / G)) / t / 1e9, 2)}
    del w
    K, N = shapes[1]
    p, sc, z = layers[0][1]
    rows = 32
    x = sqp.smooth_apply_x(activation(2048, K, 2000 + 2048), s_first[1])[:rows].contiguous().cpu().numpy()
    pn, scn, zn = p.cpu().numpy().view(np.uint32), sc.cpu().numpy(), z.cpu().numpy()
    t0 = time.perf_counter()
    oracle.w4a16_gemm_f32(x, pn, scn, zn, G)
    t = time.perf_counter() - t0
    out["gemm_8192x8192_m2048"] = {"oracle_s_for_32_rows": round(t, 2), "oracle_tflops_extrapolated": round(wl.gemm_flops(rows, N, K) / t / 1e12, 5),
                                   "sample": "32 of 2048 rows, time x 64"}
    out["cores"] = oracle.num_threads()
    return out


if __name__ == "__main__":
    main()
