#!/usr/bin/env python3
"""Benchmark of the binarized forward hot path on one MI355X.

One step = one forward pass of the fully binarized MNIST-shaped MLP
(784 -> 4096 -> 4096 -> 4096 -> 10, batch 10000) through the library:
Sign+pack of the real input, four XNOR-popcount GEMMs, three BatchNorm+Sign
epilogues.  Inputs, weights and thresholds are resident in HBM before the timed
region; the value is images/s over exactly --steps steps between two device
synchronisations.

Protocol: --warmup steps, then steps keep running until the step time has
settled (at least 50 ms, two 10-step windows within 2 %), so that a short run
measures the same clocks as a long one.  The dominant kernel is timed inside
the timed region by at least 10 pre-created pairs of HIP events (created
without the system-scope fence, so that recording them costs the step nothing)
spread over the steps; the roofline uses the median pair.  A one-wavefront
probe reads the shader clock while that kernel runs, for the fraction at the
clock the box actually held.  Outside the timed region the same run reports
the 8192^3 binary GEMM (matrix-engine and vector-ALU kernels, int8-MFMA
variant) in binary TOP/s (2*M*N*K per second), the streaming kernels in GB/s,
the conv layers, and the CPU oracle timed on the host cores: the whole batch
of the step, and the 8192^3 product with every element compared.

Single workloads: --gemm M,N,K [--fused] [--kernel ...], --stream NAME,
--conv LAYER (back-to-back launches, 10 batches of --steps, median batch).

Prints exactly one JSON line on stdout; progress goes to stderr.  With
--results FILE every workload's figures are also appended to FILE, one JSON
line each, as soon as they are measured.
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
WARM_SECONDS = 0.05
# HBM bytes per launch of the dominant kernel (fetched + written): rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this script, scaled by the same counters over a plain 1 GiB copy.  They cannot be read from inside the run, so the
# figure is carried here together with the file that holds the counter run it comes from.
PROFILED_TRAFFIC = {
    ("mfma", True): (19.18e6 + 5.12e6, "profiles/xnor_gemm_mfma_mlp_batch10000.txt"),
    ("valu", False): (32.9e6 + 166.4e6, "profiles/xnor_gemm_tiled128_mlp_batch10000.txt"),
    "xnor_gemm_8192_mfma": (50.5e6 + 268.4e6, "profiles/xnor_gemm_8192_mfma_vs_valu.txt"),
    "xnor_gemm_8192_valu": (82.4e6 + 272.6e6, "profiles/xnor_gemm_8192_mfma_vs_valu.txt"),
}
NOMINAL_CLOCK_HZ = 2.4e9


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def settle(fn, min_seconds=WARM_SECONDS, window=10, tol=0.02, max_seconds=1.0):
    """Warm-up by time, not by count: the clocks need some tens of milliseconds of load to settle after an
    idle spell (host-side set-up), and a launch is up to 25 % slower until then.  Runs fn() back to back for
    at least min_seconds, then until two consecutive windows of `window` calls agree within `tol` (bounded
    by max_seconds).  Returns (seconds spent, calls made, settled)."""
    import torch
    t_start = time.perf_counter()
    calls = 0
    prev = None
    settled = False
    while True:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(window):
            fn()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        calls += window
        cur = t1 - t0
        spent = t1 - t_start
        if spent >= min_seconds and prev is not None and abs(cur - prev) <= tol * prev:
            settled = True
            break
        if spent >= max_seconds:
            break
        prev = cur
    return time.perf_counter() - t_start, calls, settled


def time_launches(fn, iters, warmup=2, batches=10):
    """Duration in ms of one fn(): after a warm-up by time (settle), `batches` batches of `iters` back-to-back
    launches, each batch bracketed by its own pair of events on the current stream (an event pair around every
    single launch adds several microseconds to each, a large share of the short kernels here); the batches
    follow each other without a synchronisation.  Returns {"mean", "median", "min"} over the batches' averages."""
    import torch
    for _ in range(warmup):
        fn()
    settle(fn)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(batches + 1)]
    evs[0].record()
    for b in range(batches):
        for _ in range(iters):
            fn()
        evs[b + 1].record()
    torch.cuda.synchronize()
    t = np.array([evs[b].elapsed_time(evs[b + 1]) / iters for b in range(batches)])
    return {"mean": float(t.mean()), "median": float(np.median(t)), "min": float(t.min()), "batches": batches,
            "launches_per_batch": iters}


class HipEvent:
    """A HIP event created without the system-scope release that a default event record carries
    (hipEventDisableSystemFence): timing events inside the timed region then cost the step less.  Recorded
    on the raw stream handle torch launches on.  record()/elapsed_time() mirror torch.cuda.Event."""
    _hip = None
    DISABLE_SYSTEM_FENCE = 0x20000000

    def __init__(self):
        import ctypes
        if HipEvent._hip is None:
            hip = ctypes.CDLL("libamdhip64.so")
            hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
            hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
            hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
            hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
            hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
            HipEvent._hip = hip
        self._ct = ctypes
        self.handle = ctypes.c_void_p()
        rc = HipEvent._hip.hipEventCreateWithFlags(ctypes.byref(self.handle), HipEvent.DISABLE_SYSTEM_FENCE)
        if rc != 0:
            raise RuntimeError(f"hipEventCreateWithFlags failed: {rc}")

    def record(self):
        import torch
        rc = HipEvent._hip.hipEventRecord(self.handle, self._ct.c_void_p(torch.cuda.current_stream().cuda_stream))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed: {rc}")

    def elapsed_time(self, end):
        ms = self._ct.c_float()
        HipEvent._hip.hipEventSynchronize(end.handle)
        rc = HipEvent._hip.hipEventElapsedTime(self._ct.byref(ms), self.handle, end.handle)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def __del__(self):
        try:
            HipEvent._hip.hipEventDestroy(self.handle)
        except Exception:
            pass


_clock_probe = None


def measured_clock_hz(fn, torch, dev, span_ms=8.0):
    """Shader clock while fn() runs back to back: a one-wavefront probe kernel on a second stream (same priority)
    samples the shader-clock counter against the constant 100 MHz counter for about span_ms while the main
    stream keeps launching fn().  Returns the median clock over the samples of the middle 80 %, or None if
    the probe library is not built."""
    global _clock_probe
    if _clock_probe is None:
        import ctypes
        path = os.path.join(ROOT, "paper_1602_02830_amd", "libbnn_clock_probe.so")
        if not os.path.exists(path):
            return None
        _clock_probe = ctypes.CDLL(path)
        _clock_probe.bnn_clock_probe.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        _clock_probe.bnn_clock_probe.restype = ctypes.c_int
    n, sleeps = 400, 6                       # one sample every 6 x s_sleep(127) ~ 20 us: ~8 ms in all
    n = max(50, int(n * span_ms / 8.0))
    samples = torch.zeros(2 * n, dtype=torch.int64, device=dev)
    side = torch.cuda.Stream()
    for _ in range(8):
        fn()
    settle(fn)
    for _ in range(4):                       # the probe starts while launches of fn are already queued
        fn()
    rc = _clock_probe.bnn_clock_probe(samples.data_ptr(), n, sleeps, side.cuda_stream)
    if rc != 0:
        raise RuntimeError(f"clock probe launch failed: hipError {rc}")
    t_end = time.perf_counter() + 4.0
    while not side.query() and time.perf_counter() < t_end:
        for _ in range(8):
            fn()
    torch.cuda.synchronize()
    v = samples.cpu().numpy().reshape(-1, 2).astype(np.float64)
    d = np.diff(v, axis=0)
    lo, hi = len(d) // 10, len(d) - len(d) // 10
    ratio = d[lo:hi, 0] / np.maximum(d[lo:hi, 1], 1.0)
    return float(np.median(ratio) * 1e8)


def gemm_only(args, bnn, torch, dev):
    """One GEMM shape, one kernel: warm-up by time, then 10 event-bracketed batches of --steps launches, one JSON line."""
    M, N, K = (int(v) for v in args.gemm.split(","))
    kw = (K + 31) // 32
    ld = (kw + 3) // 4 * 4
    g = torch.Generator(device=dev)
    g.manual_seed(160202830)
    a = torch.randint(-2 ** 31, 2 ** 31 - 1, (M, ld), dtype=torch.int32, device=dev, generator=g)[:, :kw]
    b = torch.randint(-2 ** 31, 2 ** 31 - 1, (N, ld), dtype=torch.int32, device=dev, generator=g)[:, :kw]
    kid = {"auto": bnn.KERNEL_AUTO, "naive": bnn.KERNEL_NAIVE, "tiled128": bnn.KERNEL_TILED128,
           "ksplit": bnn.KERNEL_KSPLIT, "tiled64": bnn.KERNEL_TILED64, "mfma": bnn.KERNEL_MFMA,
           "mfma128": bnn.KERNEL_MFMA128, "mfma_shortk": bnn.KERNEL_MFMA_SHORTK,
           "mfma_persist": bnn.KERNEL_MFMA_PERSIST, "mfma_big": bnn.KERNEL_MFMA_BIG,
           "mfma_splitk": bnn.KERNEL_MFMA_SPLITK}.get(args.kernel)
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
    t = time_launches(fn, args.steps, warmup=args.warmup)
    ops = 2.0 * M * N * K
    print(json.dumps({"workload": f"xnor_gemm_{M}x{N}x{K}", "kernel": args.kernel, "fused": bool(args.fused),
                      "steps": args.steps, "warmup": args.warmup, "avg_launch_ms": t["mean"],
                      "median_launch_ms": t["median"], "min_launch_ms": t["min"],
                      "binary_tops": ops / t["median"] / 1e9}), flush=True)


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
    t = time_launches(fn, args.steps, warmup=args.warmup)
    nbytes = rows * cols * 4 + rows * nw * 4
    print(json.dumps({"workload": f"{args.stream}_{rows}x{cols}", "steps": args.steps, "warmup": args.warmup,
                      "avg_launch_ms": t["mean"], "median_launch_ms": t["median"], "min_launch_ms": t["min"],
                      "algorithmic_bytes": nbytes, "GBps": nbytes / t["median"] / 1e6}), flush=True)


def conv_only(args, bnn, torch, dev, synth, eps):
    """One conv layer of the ConvNet workload (fused, no im2col matrix): one JSON line."""
    layer = args.conv
    ch, hw = synth.CONV_LAYERS[layer]
    xc, Wt, bn = synth.config_conv(layer)
    B = xc.shape[0]
    wt = torch.from_numpy(Wt.astype(np.float32)).to(dev)
    xb = bnn.pack_sign(torch.from_numpy(xc.reshape(-1, ch).astype(np.float32)).to(dev)).view(B, hw, hw, ch // 32)
    conv = bnn.BinaryConvLayer(wt, bn, eps, B, hw, hw, fused=True, implicit=True)
    t = time_launches(lambda: conv.forward(xb), args.steps, warmup=args.warmup)
    ops = 2.0 * conv.M * conv.K * conv.Cout
    print(json.dumps({"workload": f"conv_{ch}ch_{hw}x{hw}_batch{B}", "steps": args.steps, "warmup": args.warmup,
                      "avg_launch_ms": t["mean"], "median_launch_ms": t["median"], "min_launch_ms": t["min"],
                      "binary_tops": ops / t["median"] / 1e9, "images_per_s": B / t["median"] * 1e3}), flush=True)


def gemm_roofline(name, kind, t, ops, clock_hz, extra=None):
    """Roofline entry of one 2*M*N*K product timed by time_launches: against the fp4 MFMA peak ("mfma") or the
    integer vector-ALU ceiling of the XNOR-popcount formulation ("alu"), at the nominal and at the measured clock."""
    peak = PEAK_FP4_MFMA_TFLOPS if kind == "mfma" else PEAK_BINARY_TOPS
    achieved = ops / t["median"] / 1e9
    traffic, source = PROFILED_TRAFFIC.get(name, (None, None))
    r = {"bound": kind, "kernel": name, "achieved": achieved, "peak": peak,
         "unit": ("TFLOP/s (fp4 MFMA, 2*M*N*K per launch)" if kind == "mfma" else
                  "binary TOP/s (2*M*N*K/s; peak = 256 CU x 64 lanes x 2.4 GHz / 2 lane-ops per word x 64)"),
         "frac": achieved / peak, "median_launch_ms": t["median"], "min_launch_ms": t["min"],
         "avg_launch_ms": t["mean"], "event_samples": t["batches"], "launches_per_sample": t["launches_per_batch"],
         "traffic": traffic, "traffic_source": source}
    if clock_hz:
        r["measured_clock_ghz"] = clock_hz / 1e9
        r["frac_at_measured_clock"] = achieved / (peak * clock_hz / NOMINAL_CLOCK_HZ)
    if extra:
        r.update(extra)
    return r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # --warmup counts untimed steps, but the warm-up never ends before the clocks have settled (settle():
    # at least 50 ms of steps, then two consecutive 10-step windows within 2 %), whatever the count is.
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--unfused", action="store_true",
                    help="hidden layers as separate GEMM and BN+Sign launches (int32 pre-activations through HBM)")
    ap.add_argument("--valu", action="store_true",
                    help="force the vector-ALU XNOR-popcount GEMM kernel in the hidden layers "
                         "(default: the library's choice, the bits-in / MFMA-inside kernel at these sizes)")
    ap.add_argument("--results", default=None, metavar="FILE",
                    help="append one JSON line per workload to FILE as soon as it is measured (the MLP step, the 8192^3 "
                         "product, the streaming kernels, the dense layer, the ragged sweep, the conv layers, the "
                         "ConvNet body), so that a run cut short keeps what it has; stdout stays the one line")
    ap.add_argument("--skip-extras", action="store_true",
                    help="only the timed MLP region, the 8192^3 product and the CPU baselines")
    ap.add_argument("--cpu-sample", type=int, default=10000, help="images the CPU oracle is timed on")
    ap.add_argument("--cpu-gemm-rows", type=int, default=8192,
                    help="rows of the 8192^3 product the CPU oracle is timed on (and every element of which is compared)")
    ap.add_argument("--event-pairs", type=int, default=None,
                    help="timed steps on which the dominant kernel's launches are bracketed by events "
                         "(default: max(10, steps / 10), at most every step)")
    ap.add_argument("--torch-events", action="store_true",
                    help="bracket with torch.cuda.Event (default flags) instead of HIP events without the system fence")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic, for scaling profiler byte counters)")
    ap.add_argument("--gemm", default=None, metavar="M,N,K",
                    help="time only bnn_xnor_gemm on random packed operands of this shape (for profiler runs)")
    ap.add_argument("--kernel", default="auto", choices=["auto", "naive", "tiled128", "ksplit", "tiled64", "mfma", "mfma128", "mfma_shortk", "mfma_persist", "mfma_big", "mfma_splitk", "i8"],
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
    warm_s, warm_steps, settled = settle(lambda: net.forward(xd))
    log(f"warm-up: {args.warmup} + {warm_steps} steps, {warm_s * 1e3:.0f} ms by time, settled: {settled}")
    # Dominant kernel: the two 4096 x 4096 layers (same kernel, same shape; consecutive launches when
    # the epilogue is fused).  On at least 10 of the timed steps, spread evenly, one pair of events brackets
    # them (only the second one when a BN+Sign launch sits in between); on the other steps nothing is
    # recorded, because each event record drains the queue and costs the step several microseconds.
    dominant_layers = [1, 2] if fused else [2]
    n_pairs = max(1, min(args.steps, args.event_pairs if args.event_pairs is not None else max(10, args.steps // 10)))
    event_steps = set(int(round(v)) for v in np.linspace(0, args.steps - 1, n_pairs)) if n_pairs else set()
    # The events are created before the timed region; inside it they are only recorded.
    make_event = (lambda: torch.cuda.Event(enable_timing=True)) if args.torch_events else HipEvent
    pairs = [{"start": make_event(), "end": make_event()} for _ in range(len(event_steps))]
    next_pair = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i in event_steps:
            net.forward(xd, span_events=(dominant_layers[0], dominant_layers[-1], pairs[next_pair]))
            next_pair += 1
        else:
            net.forward(xd)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    images_per_s = batch / (ms_per_step * 1e-3)
    launch_ms = np.array([ev["start"].elapsed_time(ev["end"]) for ev in pairs]) / len(dominant_layers)
    gemm_ms = float(np.median(launch_ms))
    M, N, K = batch, 4096, 4096
    ops_per_launch = 2.0 * M * N * K
    achieved_tops = ops_per_launch / (gemm_ms * 1e-3) / 1e12
    log(f"MLP step {ms_per_step:.3f} ms  {images_per_s:,.0f} images/s; 4096-layer GEMM median {gemm_ms:.4f} ms "
        f"(min {launch_ms.min():.4f}, mean {launch_ms.mean():.4f}, {len(pairs)} event pairs) "
        f"= {achieved_tops:.1f} binary TOP/s")
    scores = net.s[-1].cpu().numpy()
    # Clock of the compute units under this kernel (outside the timed region).
    a1, w1, thr1, flip1, out1 = net.a_bits[1], net.w_bits[1], net.thr[1], net.flip[1], net.a_bits[2]
    if fused:
        dom_fn = lambda: bnn.xnor_gemm_bn_sign_pack(a1, w1, K, thr1, flip1, out=out1, kernel=net.kernel)
    else:
        dom_fn = lambda: bnn.xnor_gemm(a1, w1, K, out=net.s[1], kernel=net.kernel)
    clock_hz = measured_clock_hz(dom_fn, torch, dev)

    # What the timed kernels compute in: the hidden layers multiply 1-bit operands (packed 32 per u32 in
    # HBM and LDS) widened to fp4 (E2M1) on the matrix engine with exact fp32 accumulation; with --valu
    # everything is 32-bit integer xor / popcount.
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
        "dtype": "u32" if args.valu else "fp4",
        "data": "synthetic",
        "config": {"workload": "mlp_784-4096x3-10_batch10000", "batch": batch,
                   "kernels": ("pack_sign + 3 x xnor_gemm_bn_sign_pack + xnor_gemm" if fused else
                               "pack_sign + 4 x xnor_gemm + 3 x bn_sign_pack"),
                   "arithmetic": ("u32 xor + popcount on the vector ALU" if args.valu else
                                  "1-bit operands packed in u32, widened in registers to fp4 E2M1 for "
                                  "v_mfma_f32_32x32x64_f8f6f4, exact fp32 accumulation, integer results"),
                   "warmup_by_time_ms": warm_s * 1e3, "warmup_steps_run": args.warmup + warm_steps,
                   "clocks_settled": settled},
    }
    def emit(workload, payload):
        """One line per workload in the --results file: workload, seed of its inputs, measurements."""
        if args.results:
            with open(args.results, "a") as f:
                f.write(json.dumps({"workload": workload, "data": "synthetic (workloads/synth.py, fixed seeds)",
                                    "n_gpus": 1, **payload}) + "\n")

    kname = ("xnor_gemm_tiled_kernel<8,8,16>" if args.valu else
             "xnor_gemm_mfma_big_kernel (256x256 tiles, one wavefront per SIMD)" if fused else
             "xnor_gemm_mfma_persist_kernel<false> (256x128 tiles, tile walk)") + \
            (" + fused BN+Sign epilogue" if fused else "") + " M=10000 N=4096 K=4096"
    traffic, traffic_source = PROFILED_TRAFFIC.get(("valu" if args.valu else "mfma", fused), (None, None))
    peak = PEAK_BINARY_TOPS if args.valu else PEAK_FP4_MFMA_TFLOPS
    result["roofline"] = {
        "bound": "alu" if args.valu else "mfma", "kernel": kname, "achieved": achieved_tops, "peak": peak,
        "unit": ("binary TOP/s (2*M*N*K/s; peak = 256 CU x 64 lanes x 2.4 GHz / 2 lane-ops per word x 64)"
                 if args.valu else "TFLOP/s (fp4 MFMA, 2*M*N*K per launch)"),
        "frac": achieved_tops / peak, "avg_launch_ms": float(launch_ms.mean()), "median_launch_ms": gemm_ms,
        "min_launch_ms": float(launch_ms.min()), "event_samples": len(pairs),
        "traffic": traffic, "traffic_source": traffic_source}
    if clock_hz:
        result["roofline"]["measured_clock_ghz"] = clock_hz / 1e9
        result["roofline"]["frac_at_measured_clock"] = achieved_tops / (peak * clock_hz / NOMINAL_CLOCK_HZ)

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
    emit(result["config"]["workload"], {k: result[k] for k in ("metric", "value", "unit", "steps", "warmup", "ms_per_step",
                                                               "dtype", "roofline", "cpu_baseline")})
    if not parity:
        raise RuntimeError("GPU scores differ from the oracle")
    del tr, net, a1, w1, thr1, flip1, out1

    # ---------------- the other half of the metric: binary TOP/s of bnn_xnor_gemm at 8192^3 ------------
    # (Sec. 4 / Fig. 3 shape.)  The library's own choice (bits-in / MFMA-inside) against the fp4 MFMA peak and
    # the paper's formulation (v_xor + v_bcnt on the vector ALU) against the integer-VALU ceiling, each at the
    # nominal and at the measured clock, with the oracle timed on rows of the same product.
    n = synth.GEMM_LARGE
    A8, Bm8 = synth.config_gemm_square(n)
    a_bits = bnn.pack_sign(torch.from_numpy(A8.astype(np.float32)).to(dev))
    b_bits = bnn.pack_sign(torch.from_numpy(np.ascontiguousarray(Bm8.T).astype(np.float32)).to(dev))
    c = torch.empty((n, n), dtype=torch.int32, device=dev)
    ops = 2.0 * n * n * n
    fn_auto = lambda: bnn.xnor_gemm(a_bits, b_bits, n, out=c)
    t_auto = time_launches(fn_auto, 20)
    clk_auto = measured_clock_hz(fn_auto, torch, dev)
    c_valu = torch.empty((n, n), dtype=torch.int32, device=dev)
    fn_valu = lambda: bnn.xnor_gemm(a_bits, b_bits, n, out=c_valu, kernel=bnn.KERNEL_TILED128)
    t_valu = time_launches(fn_valu, 5)
    clk_valu = measured_clock_hz(fn_valu, torch, dev, span_ms=12.0)
    equal = bool(torch.equal(c, c_valu))
    del c_valu
    n_rows = max(1, min(args.cpu_gemm_rows, n))
    g0 = time.perf_counter()
    c_cpu = oracle.matmul_pm1(A8[:n_rows], Bm8)
    g1 = time.perf_counter()
    gemm_parity = bool((c[:n_rows].cpu().numpy() == c_cpu).all())
    del c_cpu
    other = {
        "xnor_gemm_8192_mfma": gemm_roofline(
            "xnor_gemm_8192_mfma", "mfma", t_auto, ops, clk_auto,
            {"kernel": "bnn_xnor_gemm 8192^3, int32 out, library's choice = xnor_gemm_mfma_persist_kernel<false> launched one workgroup per 256x128 tile",
             "binary_tops": ops / t_auto["median"] / 1e9,
             "vs_integer_valu_ceiling": ops / t_auto["median"] / 1e9 / PEAK_BINARY_TOPS}),
        "xnor_gemm_8192_valu": gemm_roofline(
            "xnor_gemm_8192_valu", "alu", t_valu, ops, clk_valu,
            {"kernel": "bnn_xnor_gemm_kernel 8192^3, int32 out, xnor_gemm_tiled_kernel<8,8,16> (v_xor + v_bcnt)",
             "binary_tops": ops / t_valu["median"] / 1e9, "equal_to_mfma_result": equal}),
    }
    result["roofline"]["other_kernels"] = other
    result["cpu_baseline"]["other_workloads"] = {
        "xnor_gemm_8192": {"value": 2.0 * n_rows * n * n / (g1 - g0) / 1e12, "unit": "binary TOP/s (2*M*N*K/s)",
                           "cores": oracle.num_threads(), "kind": "oracle",
                           "sample": f"first {n_rows} of the {n} rows of the 8192^3 product, {g1 - g0:.2f} s wall"
                                     + ("" if n_rows == n else " (a row slice, not extrapolated)"),
                           "equal_gpu_every_element": gemm_parity}}
    for k, v in other.items():
        log(f"{k}: median {v['median_launch_ms']:.4f} ms (min {v['min_launch_ms']:.4f}) = {v['achieved']:.1f} T, "
            f"{v['frac']:.1%} of its peak; clock {v.get('measured_clock_ghz', float('nan')):.3f} GHz -> "
            f"{v.get('frac_at_measured_clock', float('nan')):.1%}")
    log(f"oracle: {n_rows} rows of 8192^3 in {g1 - g0:.2f} s; equal GPU: {gemm_parity}; VALU == MFMA result: {equal}")
    emit("xnor_gemm_8192x8192x8192", {"kernels": other, "cpu_baseline": result["cpu_baseline"]["other_workloads"]["xnor_gemm_8192"]})
    if not (gemm_parity and equal):
        raise RuntimeError("8192^3: GPU results differ from the oracle or from each other")

    # ---------------- extras, outside the timed region --------------------------------
    if not args.skip_extras:
        extras = {}
        a8, b8 = bnn.unpack_i8(a_bits, n), bnn.unpack_i8(b_bits, n)
        c2 = torch.empty((n, n), dtype=torch.int32, device=dev)
        t = time_launches(lambda: bnn.gemm_i8_mfma(a8, b8, out=c2), 10)
        extras["gemm_i8_mfma_8192"] = {"ms": t["median"], "ms_min": t["min"], "binary_tops": ops / t["median"] / 1e9,
                                       "frac_of_i8_mfma_peak": ops / t["median"] / 1e9 / PEAK_I8_MFMA_TOPS,
                                       "equal_to_xnor": bool(torch.equal(c, c2))}
        log(f"gemm_i8_mfma 8192^3: {t['median']:.3f} ms = {ops / t['median'] / 1e9:.1f} TOP/s; equal to xnor result: "
            f"{extras['gemm_i8_mfma_8192']['equal_to_xnor']}")
        del a8, b8, c2
        thr8 = torch.zeros(n, dtype=torch.int32, device=dev)
        flip8 = torch.zeros(n // 32, dtype=torch.int32, device=dev)
        out8 = torch.empty((n, n // 32), dtype=torch.int32, device=dev)
        t = time_launches(lambda: bnn.xnor_gemm_bn_sign_pack(a_bits, b_bits, n, thr8, flip8, out=out8), 20)
        extras["xnor_gemm_bn_sign_pack_8192"] = {"ms": t["median"], "ms_min": t["min"],
                                                 "binary_tops": ops / t["median"] / 1e9,
                                                 "frac_of_fp4_mfma_peak": ops / t["median"] / 1e9 / PEAK_FP4_MFMA_TFLOPS}
        log(f"xnor_gemm_bn_sign_pack 8192^3: {t['median']:.3f} ms = {ops / t['median'] / 1e9:.1f} TOP/s")
        del thr8, flip8, out8
        emit("xnor_gemm_8192_variants", {k: extras[k] for k in ("gemm_i8_mfma_8192", "xnor_gemm_bn_sign_pack_8192")})
    del c, a_bits, b_bits, A8, Bm8

    if not args.skip_extras:
        # Streaming kernels on 32768 x 8192 inputs (1 GiB: four times the last-level cache, so the rate is HBM's).
        rows_s = 4 * n
        x_s = torch.empty((rows_s, n), dtype=torch.float32, device=dev).normal_()
        bits_s = torch.empty((rows_s, n // 32), dtype=torch.int32, device=dev)
        bytes_ = rows_s * n * 4 + rows_s * n / 8
        t = time_launches(lambda: bnn.pack_sign(x_s, out=bits_s), 20)
        ms = t["median"]
        extras["pack_sign_32768x8192"] = {"ms": ms, "ms_min": t["min"], "GBps": bytes_ / ms / 1e6,
                                          "frac_of_hbm_peak": bytes_ / ms / 1e6 / PEAK_HBM_GBS}
        log(f"pack_sign 32768x8192: {ms:.3f} ms = {bytes_ / ms / 1e6:.0f} GB/s")
        c_s = x_s.view(torch.int32)                       # any int32 values do for the compare
        thr = torch.zeros(n, dtype=torch.int32, device=dev)
        flip = torch.zeros(n // 32, dtype=torch.int32, device=dev)
        t = time_launches(lambda: bnn.bn_sign_pack(c_s, thr, flip, out=bits_s), 20)
        ms = t["median"]
        extras["bn_sign_pack_32768x8192"] = {"ms": ms, "ms_min": t["min"], "GBps": bytes_ / ms / 1e6,
                                             "frac_of_hbm_peak": bytes_ / ms / 1e6 / PEAK_HBM_GBS}
        log(f"bn_sign_pack 32768x8192: {ms:.3f} ms = {bytes_ / ms / 1e6:.0f} GB/s")
        del x_s, c_s, bits_s
        emit("streaming_kernels_32768x8192", {k: extras[k] for k in ("pack_sign_32768x8192", "bn_sign_pack_32768x8192")})

        # The small dense layer (64 x 1024 x 1024) and the ragged sweep: launch-latency bound, time only.
        A0, Bm0, bn0 = synth.config_dense()
        a0 = bnn.pack_sign(torch.from_numpy(A0.astype(np.float32)).to(dev))
        b0 = bnn.pack_sign(torch.from_numpy(np.ascontiguousarray(Bm0.T).astype(np.float32)).to(dev))
        thr0, flip0 = bnn.bn_fold(*bn0, eps, 1024)
        thr0, flip0 = torch.from_numpy(thr0).to(dev), torch.from_numpy(flip0.view(np.int32)).to(dev)
        out0 = torch.empty((64, 32), dtype=torch.int32, device=dev)
        t = time_launches(lambda: bnn.xnor_gemm_bn_sign_pack(a0, b0, 1024, thr0, flip0, out=out0), 200)
        o0 = time.perf_counter()
        for _ in range(3):
            oracle.dense_layer(A0, Bm0, bn0, eps=eps)
        o1 = time.perf_counter()
        extras["dense_64x1024x1024_fused_layer"] = {"us": t["median"] * 1e3, "us_min": t["min"] * 1e3,
                                                    "oracle_us": (o1 - o0) / 3 * 1e6,
                                                    "note": "launch-latency bound; includes the host-side launch cost"}
        log(f"dense layer 64x1024x1024 (fused GEMM + BN + Sign): {t['median'] * 1e3:.1f} us per launch "
            f"(oracle {(o1 - o0) / 3 * 1e6:.0f} us)")
        emit("dense_64x1024x1024", extras["dense_64x1024x1024_fused_layer"])
        cases, host_cases = [], []
        for idx, (Mr, Nr, Kr, _p) in enumerate(synth.ragged_cases()):
            Ar, Br = synth.config_ragged(idx)
            host_cases.append((Ar, Br))
            cases.append((bnn.pack_sign(torch.from_numpy(Ar.astype(np.float32)).to(dev)),
                          bnn.pack_sign(torch.from_numpy(np.ascontiguousarray(Br.T).astype(np.float32)).to(dev)), Kr,
                          torch.empty((Mr, Nr), dtype=torch.int32, device=dev)))
        def sweep():
            for ar, br, Kr, cr in cases:
                bnn.xnor_gemm(ar, br, Kr, out=cr)
        t = time_launches(sweep, 2, warmup=1, batches=5)
        o0 = time.perf_counter()
        for Ar, Br in host_cases:
            oracle.matmul_pm1(Ar, Br)
        o1 = time.perf_counter()
        extras["ragged_sweep_336_cases"] = {"ms_total": t["median"], "us_per_case": t["median"] * 1e3 / len(cases),
                                            "oracle_ms_total": (o1 - o0) * 1e3}
        log(f"ragged sweep, {len(cases)} GEMMs: {t['median']:.3f} ms in total ({t['median'] * 1e3 / len(cases):.1f} us "
            f"per case); oracle {(o1 - o0) * 1e3:.0f} ms")
        del cases, host_cases
        emit("ragged_sweep_336_cases", extras["ragged_sweep_336_cases"])

        conv = {}
        for layer, (ch, hw) in enumerate(synth.CONV_LAYERS):
            xc, Wt, bn = synth.config_conv(layer)
            B = xc.shape[0]
            wt = torch.from_numpy(Wt.astype(np.float32)).to(dev)
            xb = bnn.pack_sign(torch.from_numpy(xc.reshape(-1, ch).astype(np.float32)).to(dev)).view(B, hw, hw, ch // 32)
            imp = bnn.BinaryConvLayer(wt, bn, eps, B, hw, hw, fused=True, implicit=True)
            low = bnn.BinaryConvLayer(wt, bn, eps, B, hw, hw, fused=True, implicit=False)
            t_imp = time_launches(lambda: imp.forward(xb), 20)
            ms_imp = t_imp["median"]
            ms_low = time_launches(lambda: low.forward(xb), 20)["median"]
            ms_i = time_launches(lambda: bnn.conv_im2col_pack(xb, ch, out=low.cols), 20)["median"]
            same = bool(torch.equal(imp.out_bits, low.out_bits))
            ops_c = 2.0 * imp.M * imp.K * imp.Cout
            conv[f"{ch}ch_{hw}x{hw}"] = {
                "implicit_fused_layer_ms": ms_imp, "implicit_fused_layer_ms_min": t_imp["min"],
                "images_per_s": B / ms_imp * 1e3,
                "binary_tops": ops_c / ms_imp / 1e9, "frac_of_fp4_mfma_peak": ops_c / ms_imp / 1e9 / PEAK_FP4_MFMA_TFLOPS,
                "im2col_then_fused_gemm_layer_ms": ms_low,
                "im2col_ms": ms_i, "im2col_write_GBps": imp.M * imp.K / 8 / ms_i / 1e6, "paths_equal": same}
            log(f"conv {ch}ch {hw}x{hw} batch {B}: implicit fused layer {ms_imp:.3f} ms ({ops_c / ms_imp / 1e9:.0f} TOP/s, "
                f"{B / ms_imp * 1e3:,.0f} images/s); im2col + fused GEMM {ms_low:.3f} ms (im2col {ms_i:.3f}); equal: {same}")
            del imp, low, xb
        extras["conv_layers_batch256"] = conv
        emit("conv_layers_batch256", conv)

        # The binary body of the paper's CIFAR-10 ConvNet (the architecture Sec. 2.2 refers to): five 3x3
        # convolutions with three poolings and three dense layers, batch 256, from the first layer's output
        # bits to the scores.
        xn, convs, fcs, fc_bns = synth.config_convnet()
        Bn = xn.shape[0]
        net = bnn.BinaryConvNet(
            [(torch.from_numpy(Wt.astype(np.float32)).to(dev), bn, pooled)
             for (Wt, bn), (_ci, _co, _hw, pooled) in zip(convs, synth.CONVNET_CONVS)],
            [torch.from_numpy(np.ascontiguousarray(Bm.T).astype(np.float32)).to(dev) for Bm in fcs], fc_bns, eps, Bn, 32, 32)
        xnb = bnn.pack_sign(torch.from_numpy(xn.reshape(-1, 128).astype(np.float32)).to(dev)).view(Bn, 32, 32, 4)
        t_net = time_launches(lambda: net.forward(xnb), 50)
        ms_net = t_net["median"]
        ops_net = sum(2.0 * Bn * hw * hw * 9 * ci * co for ci, co, hw, _p in synth.CONVNET_CONVS) + \
            sum(2.0 * Bn * synth.CONVNET_FCS[l] * synth.CONVNET_FCS[l + 1] for l in range(3))
        extras["convnet_body_batch256"] = {"ms": ms_net, "ms_min": t_net["min"], "images_per_s": Bn / ms_net * 1e3,
                                           "binary_tops": ops_net / ms_net / 1e9,
                                           "frac_of_fp4_mfma_peak": ops_net / ms_net / 1e9 / PEAK_FP4_MFMA_TFLOPS,
                                           "launches": 8}
        log(f"ConvNet body (128C3-MP2-256C3-256C3-MP2-512C3-512C3-MP2-1024FC-1024FC-10) batch {Bn}: {ms_net:.3f} ms "
            f"({Bn / ms_net * 1e3:,.0f} images/s, {ops_net / ms_net / 1e9:.0f} TOP/s)")
        del net, xnb
        emit("convnet_body_batch256", extras["convnet_body_batch256"])
        result["extras"] = extras

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
