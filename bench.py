#!/usr/bin/env python3
"""Benchmark of the binarized forward hot path on one MI355X.

One step = one forward pass of the fully binarized MNIST-shaped MLP
(784 -> 4096 -> 4096 -> 4096 -> 10, batch 10000) through the library:
Sign+pack of the real input, four XNOR-popcount GEMMs, three BatchNorm+Sign
epilogues.  Inputs, weights and thresholds are resident in HBM before the timed
region; the value is images/s.  The same run also reports, outside the timed
region, the 8192^3 binary GEMM (XNOR kernel and int8-MFMA variant) in binary
TOP/s (2*M*N*K per second), the streaming kernels in GB/s, the conv layers,
and the CPU oracle timed on the host cores on a bounded sample.

Prints exactly one JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Peak 32-bit integer vector-ALU rate: 256 compute units x 64 lanes x 2.4 GHz
# lane-operations per second.  One 32-bit word of K per output costs two lane
# operations (xor, popcount-accumulate) and is 64 binary operations in the
# 2*M*N*K count, so the ceiling of the XNOR kernel is 32 x the lane-op rate.
PEAK_LANE_OPS = 256 * 64 * 2.4e9
PEAK_BINARY_TOPS = PEAK_LANE_OPS / 2 * 64 / 1e12          # ~1258.3
PEAK_HBM_GBS = 8000.0
PEAK_I8_MFMA_TOPS = 5000.0                                # dense int8, 2*M*N*K counting
PEAK_FP4_MFMA_TFLOPS = 10100.0                            # dense fp4/fp6 MFMA, 2*M*N*K counting
# HBM bytes per launch of the dominant kernel (fetched + written), from the FETCH_SIZE / WRITE_SIZE counter
# runs summarised in profiles/xnor_gemm_mfma_mlp_batch10000.txt and profiles/xnor_gemm_tiled128_mlp_batch10000.txt.
WARM_SECONDS = 0.05
PROFILED_TRAFFIC_BYTES = {("mfma", True): 23.1e6 + 5.2e6, ("valu", False): 32.9e6 + 166.4e6}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_launches(fn, iters, warmup=2):
    """Average duration in ms of fn(): `iters` back-to-back launches bracketed by one pair of events on
    the current stream (an event pair around every single launch adds several microseconds to each,
    which is a large share of the short kernels here).  Returns (average, average) for callers that
    also report a minimum."""
    import torch
    # The clocks need some tens of milliseconds of load to settle after an idle spell (host-side set-up):
    # warm up for `warmup` launches and at least WARM_SECONDS.
    for _ in range(warmup):
        fn()
    t_end = time.perf_counter() + WARM_SECONDS
    while time.perf_counter() < t_end:
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(iters):
        fn()
    e.record()
    torch.cuda.synchronize()
    t = s.elapsed_time(e) / iters
    return float(t), float(t)


def gemm_only(args, bnn, torch, dev):
    """One GEMM shape, one kernel: W warm-up launches, K timed launches, one JSON line."""
    M, N, K = (int(v) for v in args.gemm.split(","))
    kw = (K + 31) // 32
    ld = (kw + 3) // 4 * 4
    g = torch.Generator(device=dev)
    g.manual_seed(160202830)
    a = torch.randint(-2 ** 31, 2 ** 31 - 1, (M, ld), dtype=torch.int32, device=dev, generator=g)[:, :kw]
    b = torch.randint(-2 ** 31, 2 ** 31 - 1, (N, ld), dtype=torch.int32, device=dev, generator=g)[:, :kw]
    kid = {"auto": bnn.KERNEL_AUTO, "naive": bnn.KERNEL_NAIVE, "tiled128": bnn.KERNEL_TILED128,
           "ksplit": bnn.KERNEL_KSPLIT, "tiled64": bnn.KERNEL_TILED64, "mfma": bnn.KERNEL_MFMA,
           "mfma128": bnn.KERNEL_MFMA128, "mfma_shortk": bnn.KERNEL_MFMA_SHORTK}.get(args.kernel)
    if args.kernel == "i8":
        a8, b8 = bnn.unpack_i8(a, K), bnn.unpack_i8(b, K)
        c = torch.empty((M, N), dtype=torch.int32, device=dev)
        fn = lambda: bnn.gemm_i8_mfma(a8, b8, out=c)
    elif args.fused:
        thr = torch.zeros(N, dtype=torch.int32, device=dev)
        flip = torch.zeros((N + 31) // 32, dtype=torch.int32, device=dev)
        out = torch.empty((M, (N + 31) // 32), dtype=torch.int32, device=dev)
        fn = lambda: bnn.xnor_gemm_bn_sign_pack(a, b, K, thr, flip, out=out, kernel=kid)
    else:
        c = torch.empty((M, N), dtype=torch.int32, device=dev)
        fn = lambda: bnn.xnor_gemm(a, b, K, out=c, kernel=kid)
    ms, ms_min = time_launches(fn, args.steps, warmup=args.warmup)
    ops = 2.0 * M * N * K
    print(json.dumps({"workload": f"xnor_gemm_{M}x{N}x{K}", "kernel": args.kernel, "fused": bool(args.fused),
                      "steps": args.steps, "warmup": args.warmup, "avg_launch_ms": ms, "min_launch_ms": ms_min,
                      "binary_tops": ops / ms / 1e9}), flush=True)


def stream_only(args, bnn, torch, dev):
    """One streaming kernel (Sign packer or BN+Sign epilogue) on a rows x cols input: one JSON line."""
    rows, cols = (int(v) for v in args.shape.split(","))
    nw = (cols + 31) // 32
    out = torch.empty((rows, nw), dtype=torch.int32, device=dev)
    if args.stream == "pack_sign":
        x = torch.empty((rows, cols), dtype=torch.float32, device=dev).normal_()
        fn = lambda: bnn.pack_sign(x, out=out)
    else:
        c = torch.randint(-cols, cols + 1, (rows, cols), dtype=torch.int32, device=dev)
        thr = torch.randint(-8, 9, (cols,), dtype=torch.int32, device=dev)
        flip = torch.randint(-2 ** 31, 2 ** 31 - 1, (nw,), dtype=torch.int32, device=dev)
        fn = lambda: bnn.bn_sign_pack(c, thr, flip, out=out)
    ms, _ = time_launches(fn, args.steps, warmup=args.warmup)
    nbytes = rows * cols * 4 + rows * nw * 4
    print(json.dumps({"workload": f"{args.stream}_{rows}x{cols}", "steps": args.steps, "warmup": args.warmup,
                      "avg_launch_ms": ms, "algorithmic_bytes": nbytes, "GBps": nbytes / ms / 1e6}), flush=True)


def conv_only(args, bnn, torch, dev, synth, eps):
    """One conv layer of the ConvNet workload (fused, no im2col matrix): one JSON line."""
    layer = args.conv
    ch, hw = synth.CONV_LAYERS[layer]
    xc, Wt, bn = synth.config_conv(layer)
    B = xc.shape[0]
    wt = torch.from_numpy(Wt.astype(np.float32)).to(dev)
    xb = bnn.pack_sign(torch.from_numpy(xc.reshape(-1, ch).astype(np.float32)).to(dev)).view(B, hw, hw, ch // 32)
    conv = bnn.BinaryConvLayer(wt, bn, eps, B, hw, hw, fused=True, implicit=True)
    ms, _ = time_launches(lambda: conv.forward(xb), args.steps, warmup=args.warmup)
    ops = 2.0 * conv.M * conv.K * conv.Cout
    print(json.dumps({"workload": f"conv_{ch}ch_{hw}x{hw}_batch{B}", "steps": args.steps, "warmup": args.warmup,
                      "avg_launch_ms": ms, "binary_tops": ops / ms / 1e9, "images_per_s": B / ms * 1e3}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # Defaults: 300 warm-up steps (~50 ms: after the host-side set-up the GPU clocks take ~35 ms of load to
    # settle, during which a step is up to 25 % slower), then 500 timed steps (~80 ms).
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--unfused", action="store_true",
                    help="hidden layers as separate GEMM and BN+Sign launches (int32 pre-activations through HBM)")
    ap.add_argument("--valu", action="store_true",
                    help="force the vector-ALU XNOR-popcount GEMM kernel in the hidden layers "
                         "(default: the library's choice, the bits-in / MFMA-inside kernel at these sizes)")
    ap.add_argument("--skip-extras", action="store_true", help="only the timed MLP region and the CPU baseline")
    ap.add_argument("--cpu-sample", type=int, default=2500, help="images the CPU oracle is timed on")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic, for scaling profiler byte counters)")
    ap.add_argument("--gemm", default=None, metavar="M,N,K",
                    help="time only bnn_xnor_gemm on random packed operands of this shape (for profiler runs)")
    ap.add_argument("--kernel", default="auto", choices=["auto", "naive", "tiled128", "ksplit", "tiled64", "mfma", "mfma128", "mfma_shortk", "i8"],
                    help="kernel for --gemm (i8 = the int8 MFMA variant on unpacked operands)")
    ap.add_argument("--fused", action="store_true", help="with --gemm: the fused BN+Sign entry point instead")
    ap.add_argument("--stream", default=None, choices=["pack_sign", "bn_sign_pack"],
                    help="time only this streaming kernel on a --shape input (for profiler runs)")
    ap.add_argument("--shape", default="32768,8192", metavar="ROWS,COLS", help="input shape for --stream")
    ap.add_argument("--conv", default=None, type=int, choices=[0, 1, 2],
                    help="time only this fused conv layer of the ConvNet workload, batch 256 (for profiler runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch

    import paper_1602_02830_amd as bnn
    from workloads import synth

    bnn.load_library()                      # raises if the HIP library is not built
    if not torch.cuda.is_available():
        raise RuntimeError("bench.py needs a GPU; there is no CPU fallback")
    dev = "cuda:0"
    eps = 1e-4

    if args.gemm:
        gemm_only(args, bnn, torch, dev)
        return
    if args.stream:
        stream_only(args, bnn, torch, dev)
        return
    if args.conv is not None:
        conv_only(args, bnn, torch, dev, synth, eps)
        return

    # ---------------- workload: MNIST-shaped MLP, batch 10000, synthetic -------------
    x, weights, bns = synth.config_mlp()
    batch = x.shape[0]
    wr = [torch.from_numpy(np.ascontiguousarray(w.T).astype(np.float32)).to(dev) for w in weights]
    fused = not args.unfused
    net = bnn.BinaryMLP(wr, bns, eps, batch, fused=fused,
                        kernel=bnn.KERNEL_TILED128 if args.valu else bnn.KERNEL_AUTO)
    del wr
    xd = torch.from_numpy(x).to(dev)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        net.forward(xd)
    torch.cuda.synchronize()
    # Dominant kernel: the two 4096 x 4096 layers (same kernel, same shape; consecutive launches when
    # the epilogue is fused).  On every EVENT_EVERY-th timed step one pair of events brackets them (only
    # the second one when a BN+Sign launch sits in between); on the other steps nothing is recorded,
    # because each event record drains the queue and costs the step several microseconds.
    dominant_layers = [1, 2] if fused else [2]
    EVENT_EVERY = 10
    pairs = []
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % EVENT_EVERY == 0:
            ev = {}
            net.forward(xd, span_events=(dominant_layers[0], dominant_layers[-1], ev))
            pairs.append(ev)
        else:
            net.forward(xd)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    images_per_s = batch / (ms_per_step * 1e-3)
    gemm_ms = float(np.mean([ev["start"].elapsed_time(ev["end"]) for ev in pairs])) / len(dominant_layers)
    M, N, K = batch, 4096, 4096
    ops_per_launch = 2.0 * M * N * K
    achieved_tops = ops_per_launch / (gemm_ms * 1e-3) / 1e12
    log(f"MLP step {ms_per_step:.3f} ms  {images_per_s:,.0f} images/s; 4096-layer GEMM {gemm_ms:.3f} ms "
        f"= {achieved_tops:.1f} binary TOP/s")
    scores = net.s[-1].cpu().numpy()

    result = {
        "metric": "images/s, 3x4096 BNN MLP forward (784-4096-4096-4096-10), batch 10000",
        "value": images_per_s,
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": "mlp_784-4096x3-10_batch10000", "batch": batch,
                   "kernels": ("pack_sign + 3 x xnor_gemm_bn_sign_pack + xnor_gemm" if fused else
                               "pack_sign + 4 x xnor_gemm + 3 x bn_sign_pack")},
    }
    kname = ("xnor_gemm_tiled_kernel<8,8,16>" if args.valu else "xnor_gemm_mfma_kernel<4,2>") + \
            (" + fused BN+Sign epilogue" if fused else "") + " M=10000 N=4096 K=4096"
    traffic = PROFILED_TRAFFIC_BYTES.get(("valu" if args.valu else "mfma", fused))
    if args.valu:
        result["roofline"] = {
            "bound": "alu", "kernel": kname, "achieved": achieved_tops, "peak": PEAK_BINARY_TOPS,
            "unit": "binary TOP/s (2*M*N*K/s; peak = 256 CU x 64 lanes x 2.4 GHz / 2 lane-ops per word x 64)",
            "frac": achieved_tops / PEAK_BINARY_TOPS, "avg_launch_ms": gemm_ms, "event_samples": len(pairs),
            "traffic": traffic}
    else:
        result["roofline"] = {
            "bound": "mfma", "kernel": kname, "achieved": achieved_tops, "peak": PEAK_FP4_MFMA_TFLOPS,
            "unit": "TFLOP/s (fp4 MFMA, 2*M*N*K per launch)",
            "frac": achieved_tops / PEAK_FP4_MFMA_TFLOPS, "avg_launch_ms": gemm_ms, "event_samples": len(pairs),
            "traffic": traffic}

    if args.calibration_copy:
        src = torch.zeros(256 * 1024 * 1024, dtype=torch.int32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- CPU oracle on the host cores, bounded sample --------------------
    import oracle
    n_cpu = min(args.cpu_sample, batch)
    rows = np.arange(n_cpu)
    c0 = time.perf_counter()
    tr = oracle.mlp_forward(x[rows], weights, bns, eps=eps)
    c1 = time.perf_counter()
    parity = bool((tr["s"][-1] == scores[rows]).all())
    result["cpu_baseline"] = {
        "value": n_cpu / (c1 - c0),
        "unit": "images/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"first {n_cpu} of the {batch} images, whole MLP forward, {c1 - c0:.2f} s wall",
        "scores_equal_gpu": parity,
    }
    log(f"oracle: {n_cpu} images in {c1 - c0:.2f} s on {oracle.num_threads()} threads; scores equal GPU: {parity}")
    if not parity:
        raise RuntimeError("GPU scores differ from the oracle")

    # ---------------- extras, outside the timed region --------------------------------
    if not args.skip_extras:
        del net
        extras = {}
        n = synth.GEMM_LARGE
        rng = np.random.default_rng(synth.seed_for(4, 0))
        a_f = torch.from_numpy(rng.standard_normal((n, n), dtype=np.float32)).to(dev)
        b_f = torch.from_numpy(rng.standard_normal((n, n), dtype=np.float32)).to(dev)
        a_bits, b_bits = bnn.pack_sign(a_f), bnn.pack_sign(b_f)
        c = torch.empty((n, n), dtype=torch.int32, device=dev)
        ops = 2.0 * n * n * n
        ms, ms_min = time_launches(lambda: bnn.xnor_gemm(a_bits, b_bits, n, out=c), 20)
        extras["xnor_gemm_8192"] = {"kernel": "auto (bits-in / MFMA-inside)", "ms": ms, "ms_min": ms_min,
                                    "binary_tops": ops / ms / 1e9,
                                    "frac_of_fp4_mfma_peak": ops / ms / 1e9 / PEAK_FP4_MFMA_TFLOPS,
                                    "vs_valu_roof": ops / ms / 1e9 / PEAK_BINARY_TOPS}
        log(f"xnor_gemm 8192^3 (auto = MFMA-inside): {ms:.3f} ms = {ops / ms / 1e9:.1f} binary TOP/s "
            f"({ops / ms / 1e9 / PEAK_FP4_MFMA_TFLOPS:.1%} of fp4 MFMA peak)")
        c_valu = torch.empty((n, n), dtype=torch.int32, device=dev)
        ms, ms_min = time_launches(lambda: bnn.xnor_gemm(a_bits, b_bits, n, out=c_valu, kernel=bnn.KERNEL_TILED128), 20)
        extras["xnor_gemm_8192_valu"] = {"kernel": "tiled128 (v_xor + v_bcnt)", "ms": ms, "ms_min": ms_min,
                                         "binary_tops": ops / ms / 1e9,
                                         "frac_of_valu_peak": ops / ms / 1e9 / PEAK_BINARY_TOPS,
                                         "equal_to_auto": bool(torch.equal(c, c_valu))}
        log(f"xnor_gemm 8192^3 (vector-ALU XNOR-popcount): {ms:.3f} ms = {ops / ms / 1e9:.1f} binary TOP/s "
            f"({ops / ms / 1e9 / PEAK_BINARY_TOPS:.1%} of VALU peak); equal: {extras['xnor_gemm_8192_valu']['equal_to_auto']}")
        del c_valu
        a8, b8 = bnn.unpack_i8(a_bits, n), bnn.unpack_i8(b_bits, n)
        c2 = torch.empty((n, n), dtype=torch.int32, device=dev)
        ms, ms_min = time_launches(lambda: bnn.gemm_i8_mfma(a8, b8, out=c2), 20)
        extras["gemm_i8_mfma_8192"] = {"ms": ms, "ms_min": ms_min, "binary_tops": ops / ms / 1e9,
                                       "frac_of_i8_mfma_peak": ops / ms / 1e9 / PEAK_I8_MFMA_TOPS,
                                       "equal_to_xnor": bool(torch.equal(c, c2))}
        log(f"gemm_i8_mfma 8192^3: {ms:.3f} ms = {ops / ms / 1e9:.1f} TOP/s; equal to xnor result: "
            f"{extras['gemm_i8_mfma_8192']['equal_to_xnor']}")
        del a8, b8, c2
        del a_f, b_f, c, a_bits, b_bits

        # Streaming kernels on 32768 x 8192 inputs (1 GiB: four times the last-level cache, so the rate is HBM's).
        rows_s = 4 * n
        x_s = torch.empty((rows_s, n), dtype=torch.float32, device=dev).normal_()
        bits_s = torch.empty((rows_s, n // 32), dtype=torch.int32, device=dev)
        bytes_ = rows_s * n * 4 + rows_s * n / 8
        ms, _ = time_launches(lambda: bnn.pack_sign(x_s, out=bits_s), 20)
        extras["pack_sign_32768x8192"] = {"ms": ms, "GBps": bytes_ / ms / 1e6, "frac_of_hbm_peak": bytes_ / ms / 1e6 / PEAK_HBM_GBS}
        log(f"pack_sign 32768x8192: {ms:.3f} ms = {bytes_ / ms / 1e6:.0f} GB/s")
        c_s = x_s.view(torch.int32)                       # any int32 values do for the compare
        thr = torch.zeros(n, dtype=torch.int32, device=dev)
        flip = torch.zeros(n // 32, dtype=torch.int32, device=dev)
        ms, _ = time_launches(lambda: bnn.bn_sign_pack(c_s, thr, flip, out=bits_s), 20)
        extras["bn_sign_pack_32768x8192"] = {"ms": ms, "GBps": bytes_ / ms / 1e6, "frac_of_hbm_peak": bytes_ / ms / 1e6 / PEAK_HBM_GBS}
        log(f"bn_sign_pack 32768x8192: {ms:.3f} ms = {bytes_ / ms / 1e6:.0f} GB/s")
        del x_s, c_s, bits_s

        # The small dense layer (64 x 1024 x 1024) and the ragged sweep: launch-latency bound, time only.
        A0, Bm0, bn0 = synth.config_dense()
        a0 = bnn.pack_sign(torch.from_numpy(A0.astype(np.float32)).to(dev))
        b0 = bnn.pack_sign(torch.from_numpy(np.ascontiguousarray(Bm0.T).astype(np.float32)).to(dev))
        thr0, flip0 = bnn.bn_fold(*bn0, eps, 1024)
        thr0, flip0 = torch.from_numpy(thr0).to(dev), torch.from_numpy(flip0.view(np.int32)).to(dev)
        out0 = torch.empty((64, 32), dtype=torch.int32, device=dev)
        ms, _ = time_launches(lambda: bnn.xnor_gemm_bn_sign_pack(a0, b0, 1024, thr0, flip0, out=out0), 200)
        extras["dense_64x1024x1024_fused_layer"] = {"us": ms * 1e3, "note": "launch-latency bound; includes the host-side launch cost"}
        log(f"dense layer 64x1024x1024 (fused GEMM + BN + Sign): {ms * 1e3:.1f} us per launch")
        cases = []
        for idx, (Mr, Nr, Kr, _p) in enumerate(synth.ragged_cases()):
            Ar, Br = synth.config_ragged(idx)
            cases.append((bnn.pack_sign(torch.from_numpy(Ar.astype(np.float32)).to(dev)),
                          bnn.pack_sign(torch.from_numpy(np.ascontiguousarray(Br.T).astype(np.float32)).to(dev)), Kr,
                          torch.empty((Mr, Nr), dtype=torch.int32, device=dev)))
        def sweep():
            for ar, br, Kr, cr in cases:
                bnn.xnor_gemm(ar, br, Kr, out=cr)
        ms, _ = time_launches(sweep, 5, warmup=1)
        extras["ragged_sweep_336_cases"] = {"ms_total": ms, "us_per_case": ms * 1e3 / len(cases)}
        log(f"ragged sweep, {len(cases)} GEMMs: {ms:.3f} ms in total ({ms * 1e3 / len(cases):.1f} us per case)")
        del cases

        conv = {}
        for layer, (ch, hw) in enumerate(synth.CONV_LAYERS):
            xc, Wt, bn = synth.config_conv(layer)
            B = xc.shape[0]
            wt = torch.from_numpy(Wt.astype(np.float32)).to(dev)
            xb = bnn.pack_sign(torch.from_numpy(xc.reshape(-1, ch).astype(np.float32)).to(dev)).view(B, hw, hw, ch // 32)
            imp = bnn.BinaryConvLayer(wt, bn, eps, B, hw, hw, fused=True, implicit=True)
            low = bnn.BinaryConvLayer(wt, bn, eps, B, hw, hw, fused=True, implicit=False)
            ms_imp, _ = time_launches(lambda: imp.forward(xb), 20)
            ms_low, _ = time_launches(lambda: low.forward(xb), 20)
            ms_i, _ = time_launches(lambda: bnn.conv_im2col_pack(xb, ch, out=low.cols), 20)
            same = bool(torch.equal(imp.out_bits, low.out_bits))
            ops_c = 2.0 * imp.M * imp.K * imp.Cout
            conv[f"{ch}ch_{hw}x{hw}"] = {
                "implicit_fused_layer_ms": ms_imp, "images_per_s": B / ms_imp * 1e3,
                "binary_tops": ops_c / ms_imp / 1e9, "im2col_then_fused_gemm_layer_ms": ms_low,
                "im2col_ms": ms_i, "im2col_write_GBps": imp.M * imp.K / 8 / ms_i / 1e6, "paths_equal": same}
            log(f"conv {ch}ch {hw}x{hw} batch {B}: implicit fused layer {ms_imp:.3f} ms ({ops_c / ms_imp / 1e9:.0f} TOP/s, "
                f"{B / ms_imp * 1e3:,.0f} images/s); im2col + fused GEMM {ms_low:.3f} ms (im2col {ms_i:.3f}); equal: {same}")
            del imp, low, xb
        extras["conv_layers_batch256"] = conv

        # The binary body of the paper's CIFAR-10 ConvNet (Sec. 2.2): five 3x3 convolutions with three
        # poolings and three dense layers, batch 256, from the first layer's output bits to the scores.
        xn, convs, fcs, fc_bns = synth.config_convnet()
        Bn = xn.shape[0]
        net = bnn.BinaryConvNet(
            [(torch.from_numpy(Wt.astype(np.float32)).to(dev), bn, pooled)
             for (Wt, bn), (_ci, _co, _hw, pooled) in zip(convs, synth.CONVNET_CONVS)],
            [torch.from_numpy(np.ascontiguousarray(Bm.T).astype(np.float32)).to(dev) for Bm in fcs], fc_bns, eps, Bn, 32, 32)
        xnb = bnn.pack_sign(torch.from_numpy(xn.reshape(-1, 128).astype(np.float32)).to(dev)).view(Bn, 32, 32, 4)
        ms_net, _ = time_launches(lambda: net.forward(xnb), 50)
        ops_net = sum(2.0 * Bn * hw * hw * 9 * ci * co for ci, co, hw, _p in synth.CONVNET_CONVS) + \
            sum(2.0 * Bn * synth.CONVNET_FCS[l] * synth.CONVNET_FCS[l + 1] for l in range(3))
        extras["convnet_body_batch256"] = {"ms": ms_net, "images_per_s": Bn / ms_net * 1e3,
                                           "binary_tops": ops_net / ms_net / 1e9, "launches": 8}
        log(f"ConvNet body (128C3-MP2-256C3-256C3-MP2-512C3-512C3-MP2-1024FC-1024FC-10) batch {Bn}: {ms_net:.3f} ms "
            f"({Bn / ms_net * 1e3:,.0f} images/s, {ops_net / ms_net / 1e9:.0f} TOP/s)")
        del net, xnb
        result["extras"] = extras

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
