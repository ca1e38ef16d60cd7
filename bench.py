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

# HBM bytes per decode launch (averaged over the four shapes of the sweep) from the
# rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in
# profiles/w4a16_decode_34b_m16_hbm_traffic.md (34B shapes, M=16, default plan).
TRAFFIC_BYTES_PER_LAUNCH = 109.4e6


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
    ws_need = max(sqp.workspace_bytes(m, N, K, G) for (K, N) in shapes for m in (1, M, 16, 2048, 4096))
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
                "traffic": TRAFFIC_BYTES_PER_LAUNCH if (args.model == "34b" and M == 16) else None,
                "kernel": "w4a16_decode_kernel", "avg_launch_us": round(avg_launch_s * 1e6, 2),
                "algorithmic_bytes_per_launch": round(bytes_per_launch)}

    extra = {}
    if not args.no_extra:
        extra = side_measurements(torch, sqp, wl, dev, shapes, layers, s_first, activation, G)

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(np, torch, wl, shapes, layers, xs, M, G)

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


def side_measurements(torch, sqp, wl, dev, shapes, layers, s_first, activation, G):
    """Context figures outside the headline: M=1 decode sweep, prefill at M=2048 (TFLOP/s
    against the fp16 MFMA peak) and the companion kernels on the 22016x8192 weight."""
    extra = {}
    # decode at M=1 over all resident layers
    M = 1
    xs = [sqp.smooth_apply_x(activation(M, K, 2000 + M), s_first[si]) for si, (K, N) in enumerate(shapes)]
    ys = [torch.empty((M, N), device=dev, dtype=torch.float16) for (K, N) in shapes]

    def sweep():
        for per in layers:
            for si, (p, sc, z) in enumerate(per):
                sqp.w4a16_gemm(xs[si], p, sc, z, G, out=ys[si])
    t = _time(torch, sweep, 3)
    b = len(layers) * sum(wl.algorithmic_bytes(M, N, K, G) for (K, N) in shapes)
    extra["decode_m1_gbs"] = round(b / t / 1e9, 1)
    extra["decode_m1_pct_hbm_peak"] = round(100 * b / t / 1e9 / HBM_PEAK_GBS, 2)
    # prefill, M = 2048, the four shapes, rotating over the resident layers
    M = 2048
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
        pre["%dx%d" % (K, N)] = round(fl / t / 1e12, 1)
        flops_total += fl
        t_total += t
        del x, y
    extra["prefill_m2048_tflops_by_shape"] = pre
    extra["prefill_m2048_tflops"] = round(flops_total / t_total / 1e12, 1)
    extra["prefill_m2048_pct_mfma_peak"] = round(100 * flops_total / t_total / 1e12 / MFMA_F16_PEAK_TFLOPS, 2)
    # what the matrix cores sustain on this chip with nothing else to do: a loop of independent
    # 32x32x16 fp16 MFMAs on one of the activations above (the clock settles under the power limit)
    import ctypes
    L = sqp.lib()
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
    return extra


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


if __name__ == "__main__":
    main()
