#!/usr/bin/env python3
"""Benchmark of the MI355X-native local GEMM / forward convolution library.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Prints ONE JSON line.  The default workload is the headline one: the FP32 NN GEMM with
M = N = K = 4096 (one GPU's local block of a block-distributed matrix), seeded synthetic inputs
already resident in HBM, one dmath_gemm call per step.  Metric: TFLOP/s (2*M*N*K per call over
the mean time per call), with the fraction of the MI355X FP32 MFMA peak in "roofline" and the
FP64 CPU oracle timed on this machine's host cores on a bounded sample of the same problem in
"cpu_baseline".  Other workloads (--workload) are the remaining benchmark configurations; they
print the same kind of line for their own shape.

Everything runs on one GPU; --gpus above 1 is refused.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Published MI355X peaks used as roofline denominators.
PEAK_FP32_MFMA_TFLOPS = 157.3   # 256 CUs x 4 SIMDs x 64 flop/clk x 2.4 GHz
PEAK_FP16_MFMA_TFLOPS = 2500.0  # dense FP16-input matrix instruction, FP32 accumulate
PEAK_FP64_MFMA_TFLOPS = 78.6
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE runs, each scaled by
# what the same counter reads for a device copy of known size); figures and commands are in
# profiles/*.md.  Keyed by workload; None where no counter run is committed.
MEASURED_HBM_TRAFFIC_BYTES = {
    # per step: sum over the kernels of a step of FETCH_SIZE KiB x 2.0 (copy factor) + WRITE_SIZE KiB x 1.0
    "gemm4096": int((196779.4 * 2.0 + 65536.5) * 1024),                         # profiles/gemm_nn_4096_tile_kernel.md
    "gemm256": int((820.7 * 2.0 + 256.2) * 1024),                               # profiles/gemm_nn_256_wavek_kernel.md
    "summa": int(16 * (231599.7 * 2.0 + 262144.5) * 1024),                      # profiles/summa_update_8192x8192x512_tile_kernel.md
    "summa_fused": int((1704078.9 * 2.0 + 262243.2) * 1024),                    # profiles/summa_fused_8192x8192x512_x16_panels_kernel.md
    "fc": int(((49207.9 + 49210.5 + 12461.6) * 2.0
               + 2 * 4096.5 + 65612.7) * 1024),                                 # profiles/fc_4096_batch256_kernels.md
    "conv": int(((97615.8 + 1815.1) * 2.0 + 137522.4 + 2304.1) * 1024),        # profiles/conv3x3_n128_c256_k256_28x28_kernels.md
    "conv_bwd_data": int(((97004.2 + 5719.1) * 2.0 + 137523.3 + 2304.1) * 1024),  # profiles/conv3x3_..._bwd_data_kernels.md
    "conv_bwd_filter": int(((156773.1 + 32274.5) * 2.0 + 64512.0 + 2304.0) * 1024),  # profiles/conv3x3_..._bwd_filter_kernels.md
    "hgemm4096": int((98398.5 * 2.0 + 32768.5) * 1024),                         # profiles/hgemm_nn_4096_half_storage_mi16_dma64_kernel.md
    "fc_half": int(((2 * 8212.6 + 33934.3 + 6248.1 + 33933.8) * 2.0
                    + 2 * 2048.0 + 2 * 16384.5 + 32768.5) * 1024),              # profiles/fc_4096_batch256_half_storage_kernels.md
    "dgemm4096": int((665503.0 * 2.0 + 131694.3) * 1024),                       # profiles/dgemm_nn_4096_tile_kernel.md
}

WORKLOADS = ("gemm4096", "gemm256", "summa", "fc", "conv", "conv_bwd_data", "conv_bwd_filter", "summa_fused",
             "fc_nn", "fc_nt", "fc_tn", "hgemm4096", "fc_half", "dgemm4096", "square")

# One-GPU column of the paper's table "Matrix Multiplication Performance" (seconds per multiply on one
# K80 GPU with cuBLAS 7.5; the larger sizes did not fit its memory).  Context only, never a target.
PAPER_TABLE_ONE_GPU_SECONDS = {4096: 0.052, 6144: 0.174, 8192: 0.413, 12288: 1.450, 16384: 3.340, 24576: 12.279}


def _device_arrays(torch, arrays):
    return {k: torch.from_numpy(v).cuda() for k, v in arrays.items()}


LAUNCH_BOUND = ("gemm256", "fc", "fc_nn", "fc_nt", "fc_tn", "fc_half")   # steps of 10 - 200 us


def _time_steps(torch, step, steps, warmup, per_step=True, before_step=None):
    """warmup untimed steps, then exactly `steps` timed ones between synchronisations.

    The timed region is bracketed by one HIP event pair on the launch stream (its span / steps is the
    mean that the benchmark reports).  Inside it an event is also recorded at every step boundary
    (per_step) or at the boundaries of five equal batches (launch-bound workloads, where an event per
    step would be a visible share of the step), which gives the spread over the region.
    before_step(i), if given, is called on the host before step i of the timed region (i < 0: warm-up).

    Returns a dict: ms (mean per step by the events), ms_host (by the host clock), per_step_ms or
    batch_ms (list), events_per ("step" | "batch")."""
    for i in range(warmup):
        if before_step is not None:
            before_step(i - warmup)
        step()
    torch.cuda.synchronize()
    if per_step:
        marks = list(range(steps + 1))
    else:
        nb = min(5, steps)
        marks = sorted(set(round(j * steps / nb) for j in range(nb + 1)))
    ev = {m: torch.cuda.Event(enable_timing=True) for m in marks}
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        if before_step is not None:
            before_step(i)
        step()
        if i + 1 in ev:
            ev[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    spans = [ev[a].elapsed_time(ev[b]) / (b - a) for a, b in zip(marks[:-1], marks[1:])]
    out = {"ms": ev[0].elapsed_time(ev[steps]) / steps, "ms_host": (t1 - t0) * 1e3 / steps,
           "events_per": "step" if per_step else "batch"}
    out["per_step_ms" if per_step else "batch_ms"] = spans
    return out


def _spread(values):
    v = sorted(values)
    n = len(v)
    med = v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])
    return {"median": med, "min": v[0], "max": v[-1]}


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _cpu_baseline_gemm(oracle, call, arrays, budget_s=15.0):
    """The oracle as it stands on a bounded sample: the first R rows of C (all N columns, full K).

    Returns (report, rows, ref, mag): the timing report, and the oracle's sums for those rows so that
    the caller can hold the GPU result against them."""
    A, B = arrays[call.A], arrays[call.B]
    C0 = arrays[call.C] if call.beta != 0.0 else None

    def run(rows):
        t0 = time.perf_counter()
        ref, mag = oracle.gemm(call.transA, call.transB, rows, call.N, call.K, call.alpha, A, call.lda, B, call.ldb,
                               call.beta, C0, call.ldc)
        return time.perf_counter() - t0, ref, mag

    threads = oracle.num_threads()
    probe_rows = min(call.M, 2 * threads)
    t_probe = max(run(probe_rows)[0], 1e-4)
    rows = int(min(call.M, max(probe_rows, probe_rows * budget_s / t_probe)))
    rows = max(threads, rows - rows % threads)
    rows = min(rows, call.M)
    t, ref, mag = run(rows)
    flop = 2.0 * rows * call.N * call.K
    return {
        "value": flop / t / 1e12, "unit": "TFLOP/s", "cores": threads, "cpu_model": _cpu_model(), "kind": "oracle",
        "seconds": t, "seconds_whole_call_extrapolated": t * call.M / rows,
        "sample": "first %d of %d rows of C (all %d columns, full K=%d), FP64 sums plus the magnitude sums, %.1f s"
                  % (rows, call.M, call.N, call.K, t),
    }, rows, ref, mag


def _cpu_baseline_conv(oracle, wl, budget_s=15.0):
    import numpy as np
    threads = oracle.num_threads()
    N, Kout, P, Q = wl.out_shape
    _, _, K = wl.gemm_view
    total = N * Kout * P * Q
    rng = np.random.default_rng(0)

    def run(npts):
        idx = rng.choice(total, size=npts, replace=False)
        t0 = time.perf_counter()
        ref, mag = oracle.conv2d_fwd_points(wl.x, wl.w, idx, pad=wl.pad, stride=wl.stride)
        return time.perf_counter() - t0, idx, ref, mag

    probe = 20000
    t_probe = max(run(probe)[0], 1e-4)
    npts = int(min(total, max(probe, probe * budget_s / t_probe)))
    t, idx, ref, mag = run(npts)
    return {
        "value": 2.0 * npts * K / t / 1e12, "unit": "TFLOP/s", "cores": threads, "cpu_model": _cpu_model(), "kind": "oracle",
        "seconds": t, "seconds_whole_call_extrapolated": t * total / npts,
        "sample": "%d random output elements of %d (all %d taps each), FP64 sums plus the magnitude sums, %.1f s"
                  % (npts, total, K, t),
    }, idx, ref, mag


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", choices=WORKLOADS, default="gemm4096")
    ap.add_argument("--size", type=int, default=16384,
                    help="--workload square: FP32 NN product of size^3, operands uniform[-1,1] drawn on the device "
                         "(the sizes of the paper's multiplication table: 4096 6144 8192 12288 16384 24576 32768 49152 65536)")
    ap.add_argument("--tile-config", type=int, default=-1, help="force a tile configuration (tuning only)")
    ap.add_argument("--split-k", type=int, default=-1, help="force a split-K factor (tuning only)")
    ap.add_argument("--hgemm-path", type=int, default=-1, help="force the dmath_hgemm kernel (see dmath_set_hgemm_path)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (for profiler runs)")
    ap.add_argument("--detail", action="store_true",
                    help="add the per-step (or per-batch) times and the shader clock of every launch to the line")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (launch-bound workloads: gemm256, fc, fc_half)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the workload, run `steps` device copies of 256 MiB (for scaling HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this library runs on one GPU; --gpus %d is not supported "
                         "(no multi-GPU path exists in this build)\n" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1604_01416_amd import dmath as dm      # fails loudly if libdmath.so is missing
    from paper_1604_01416_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    if args.copy_calibration:
        nbytes = 256 << 20
        src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        ms = _time_steps(torch, lambda: dst.copy_(src), args.steps, args.warmup, per_step=False)["ms"]
        print(json.dumps({"copy_bytes_read": nbytes, "copy_bytes_written": nbytes, "steps": args.steps,
                          "ms_per_copy": ms, "GBps": 2 * nbytes / ms / 1e6}))
        return

    ws_bytes = 128 << 20
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    dm.check(dm.dmath_set_workspace(ws, ws_bytes))
    if args.tile_config >= 0 or args.split_k >= 1:
        dm.check(dm.dmath_set_override(args.tile_config, args.split_k))
    if args.hgemm_path >= 0:
        dm.check(dm.dmath_set_hgemm_path(args.hgemm_path))

    cpu_baseline = None
    conv = None
    if args.workload in ("conv", "conv_bwd_data", "conv_bwd_filter"):
        conv = workloads.config5()
        N, Kout, P, Q = conv.out_shape
        _, C, H, W = conv.x.shape
        dx, dw = torch.from_numpy(conv.x).cuda(), torch.from_numpy(conv.w).cuda()
        dy = torch.empty((N, Kout, P, Q), device="cuda")
        bwd = args.workload == "conv_bwd_data"
        bwd_filter = args.workload == "conv_bwd_filter"
        if bwd or bwd_filter:   # gradients of the same layer: dy ~ N(0, 1e-2), seed 5
            grad = (np.random.default_rng(5).standard_normal((N, Kout, P, Q)) * 1e-2).astype(np.float32)
            dy = torch.from_numpy(grad).cuda()
        if bwd:
            dx = torch.empty((N, C, H, W), device="cuda")
        if bwd_filter:
            dw = torch.empty((Kout, C, 3, 3), device="cuda")

        def step():
            if bwd_filter:
                dm.check(dm.dmath_conv2d_bwd_filter(N, C, H, W, Kout, 3, 3, 1, 1, 1, 1, 1.0, dx, dy, 0.0, dw))
            elif bwd:
                dm.check(dm.dmath_conv2d_bwd_data(N, C, H, W, Kout, 3, 3, 1, 1, 1, 1, 1.0, dy, dw, 0.0, dx))
            else:
                dm.check(dm.dmath_conv2d_fwd(N, C, H, W, Kout, 3, 3, 1, 1, 1, 1, 1.0, dx, dw, 0.0, dy))

        flop, alg_bytes, launches = conv.flop, conv.algorithmic_bytes, 1
        wl_name = conv.name + ("_bwd_data" if bwd else "_bwd_filter" if bwd_filter else "")
    elif args.workload == "square":
        # a size of the paper's table: drawn on the device (65536^2 elements would take minutes on the host)
        n = args.size
        assert 1 <= n <= 65536
        gen = torch.Generator(device="cuda")
        gen.manual_seed(n)
        dA = torch.rand((n, n), generator=gen, device="cuda").mul_(2.0).sub_(1.0)
        dB = torch.rand((n, n), generator=gen, device="cuda").mul_(2.0).sub_(1.0)
        dC = torch.empty((n, n), device="cuda")
        call = workloads.GemmCall(0, 0, n, n, n, 1.0, "A", n, "B", n, 0.0, "C", n)

        def step():
            dm.check(dm.dmath_gemm(0, 0, n, n, n, 1.0, dA, n, dB, n, 0.0, dC, n))

        flop, alg_bytes, launches, wl_name = call.flop, call.algorithmic_bytes, 1, "gemm_nn_%d" % n
    else:
        wl = {"gemm4096": workloads.config2, "gemm256": workloads.config1, "summa": workloads.config3,
              "summa_fused": workloads.config3, "fc": workloads.config4, "fc_nn": workloads.config4,
              "fc_nt": workloads.config4, "fc_tn": workloads.config4, "hgemm4096": workloads.config2,
              "fc_half": workloads.config4, "dgemm4096": workloads.config2}[args.workload]()
        half = args.workload in ("hgemm4096", "fc_half")   # the same operands rounded to half-precision storage
        if half:
            wl.arrays = {k: v.astype(np.float16) for k, v in wl.arrays.items()}
            wl.name += "_half_storage"
        if args.workload in ("fc_nn", "fc_nt", "fc_tn"):   # one of the three products of the layer alone
            wl.calls = [wl.calls[("fc_nn", "fc_nt", "fc_tn").index(args.workload)]]
            wl.name += "_" + args.workload[3:]
        double = args.workload == "dgemm4096"          # the same operands widened to FP64
        if double:
            wl.arrays = {k: v.astype(np.float64) for k, v in wl.arrays.items()}
            wl.name += "_fp64"
        dev = _device_arrays(torch, wl.arrays)
        calls = [(c, dev[c.A], dev[c.B], dev[c.C]) for c in wl.calls]
        fused = args.workload == "summa_fused"   # the same update sequence as one multi-panel call

        def step():
            if fused:
                c = wl.calls[0]
                dm.check(dm.dmath_gemm_panels(c.transA, c.transB, c.M, c.N, c.K, c.alpha, [x[1] for x in calls], c.lda,
                                              [x[2] for x in calls], c.ldb, c.beta, calls[0][3], c.ldc))
                return
            gemm = dm.dmath_hgemm if half else dm.dmath_dgemm if double else dm.dmath_gemm
            for c, a, b, cc in calls:
                dm.check(gemm(c.transA, c.transB, c.M, c.N, c.K, c.alpha, a, c.lda, b, c.ldb, c.beta, cc, c.ldc))

        flop = wl.flop
        alg_bytes = sum(c.algorithmic_bytes for c in wl.calls) // (2 if half else 1) * (2 if double else 1)
        launches = len(wl.calls)
        wl_name = wl.name
        if fused:   # all panels read once, C read and written once
            c = wl.calls[0]
            alg_bytes = 4 * (len(wl.calls) * (c.M * c.K + c.K * c.N) + 2 * c.M * c.N)
            launches = 1
            wl_name = wl.name + "_fused"

    # Clock the tile kernel really runs at (GEMM workloads): the in-kernel stamps stay on during warm-up
    # and timed steps (four 8-byte global stores by one lane of 8 workgroups per launch), every step into
    # a row of its own, so the line can say how the clock moved over the region it timed.
    probe = None
    before_step = None
    if conv is None:
        probe = torch.zeros((args.warmup + args.steps, 32), dtype=torch.int64, device="cuda")
        rows_of_probe = [probe[i] for i in range(args.warmup + args.steps)]
        dm.check(dm.dmath_set_clock_probe(rows_of_probe[-1]))
        # (a captured launch keeps the pointer it was captured with; launch-bound workloads would notice
        # the extra host call per step: both keep the last row for every launch)
        if not args.graph and args.workload not in LAUNCH_BOUND:
            def before_step(i):
                dm.dmath_set_clock_probe(rows_of_probe[i + args.warmup])
    if args.graph:   # the same kernels, launched by one graph replay per step
        step()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        captured = torch.cuda.CUDAGraph()
        with torch.cuda.graph(captured, stream=side):
            step()
        eager_step, step = step, captured.replay
    # one event per step where a step is long enough not to notice it (an event costs about a microsecond
    # on the stream); launch-bound workloads get five batches instead
    per_step = args.workload not in LAUNCH_BOUND and not args.graph
    timing = _time_steps(torch, step, args.steps, args.warmup, per_step=per_step, before_step=before_step)
    ms_ev, ms_wall = timing["ms"], timing["ms_host"]
    tflops = flop / ms_ev / 1e9
    spans = timing.get("per_step_ms") or timing["batch_ms"]
    spread = _spread(spans)
    nb = min(5, len(spans))
    batches = [sum(spans[round(j * len(spans) / nb):round((j + 1) * len(spans) / nb)]) /
               max(1, round((j + 1) * len(spans) / nb) - round(j * len(spans) / nb)) for j in range(nb)]
    measured_clock_ghz = None
    clock_per_step = None
    kernel_us = []
    launch_floor_us = None
    if probe is not None:
        dm.check(dm.dmath_set_clock_probe(None))
        clock_per_step = []
        kernel_us = []
        for row in probe.cpu().tolist():
            p = [int(v) for v in row]
            per_die = [(p[4 * d + 2] - p[4 * d]) / (p[4 * d + 3] - p[4 * d + 1]) * 0.1
                       for d in range(8) if p[4 * d + 3] > p[4 * d + 1]]
            clock_per_step.append(sum(per_die) / len(per_die) if per_die else None)
            if launches == 1:   # span of the launch on the device: first start to last end of those workgroups
                starts = [p[4 * d + 1] for d in range(8) if p[4 * d + 3] > p[4 * d + 1]]
                ends = [p[4 * d + 3] for d in range(8) if p[4 * d + 3] > p[4 * d + 1]]
                kernel_us.append((max(ends) - min(starts)) / 100.0 if starts else None)
        timed = [c for c in clock_per_step[args.warmup:] if c is not None]
        if timed:
            measured_clock_ghz = {"mean": sum(timed) / len(timed), "min": min(timed), "max": max(timed),
                                  "first_timed_step": timed[0], "last_timed_step": timed[-1],
                                  "first_warmup_step": clock_per_step[0]}

    if args.workload == "gemm256" and not args.no_cpu_baseline:
        # what a launch costs when the kernel has next to nothing to do: a 64^3 product (one workgroup),
        # queued the same way (a reference leg like the CPU baseline, and skipped with it)
        fa, fb, fc_ = (torch.zeros((64, 64), device="cuda") for _ in range(3))
        floor = _time_steps(torch, lambda: dm.check(dm.dmath_gemm(0, 0, 64, 64, 64, 1.0, fa, 64, fb, 64, 0.0, fc_, 64)),
                            args.steps, args.warmup, per_step=False)
        launch_floor_us = floor["ms"] * 1e3
    # The oracle on this machine's host cores on a bounded sample, and the output of the timed launches held
    # against it (beta == 0 workloads recompute the same C every step; an accumulating first call is run
    # once more from the stored C0).
    check = None
    if not args.no_cpu_baseline:
        import oracle
        if args.workload in ("hgemm4096", "fc_half", "dgemm4096", "square"):
            cpu_baseline = None   # the FP32 workloads of the same shapes carry the oracle timing
        elif conv is not None and args.workload != "conv":
            cpu_baseline = None   # the forward workload carries the oracle timing of this layer
        elif conv is not None:
            cpu_baseline, idx, ref, mag = _cpu_baseline_conv(oracle, conv)
            got = dy.reshape(-1)[torch.from_numpy(idx).cuda()].cpu().numpy().astype(np.float64)
            ratio = np.abs(got - ref) / oracle.bound(conv.gemm_view[2], mag)
            check = {"max_err_over_bound": float(ratio.max()), "max_abs_err": float(np.abs(got - ref).max()),
                     "elements": int(idx.size), "passed": bool((ratio <= 1.0).all())}
        else:
            c0 = wl.calls[0]
            cpu_baseline, rows, ref, mag = _cpu_baseline_gemm(oracle, c0, wl.arrays)
            out_dev = dev[c0.C]   # (the fused update is held against its first panel's product through dmath_gemm)
            if c0.beta != 0.0:
                out_dev = torch.from_numpy(wl.arrays[c0.C]).cuda()
                dm.check(dm.dmath_gemm(c0.transA, c0.transB, c0.M, c0.N, c0.K, c0.alpha, dev[c0.A], c0.lda, dev[c0.B],
                                       c0.ldb, c0.beta, out_dev, c0.ldc))
                torch.cuda.synchronize()
            got = out_dev.reshape(-1)[:rows * c0.ldc].reshape(rows, c0.ldc)[:, :c0.N].cpu().numpy().astype(np.float64)
            ratio = np.abs(got - ref) / oracle.bound(c0.K, mag)
            check = {"max_err_over_bound": float(ratio.max()), "max_abs_err": float(np.abs(got - ref).max()),
                     "elements": int(ratio.size), "passed": bool((ratio <= 1.0).all()),
                     "what": "first call of the step, first %d rows of C, |gpu - ref| / (4*K*2^-24*mag + 1e-6)" % rows}

    # Dominant kernel: the MFMA tile kernel.  The headline workload is one launch of it per step, so its
    # mean duration is the event time per step; for multi-call workloads this is the aggregate rate.
    achieved = tflops
    # each contraction is priced against the matrix peak of its own input type
    peak, dtype = PEAK_FP32_MFMA_TFLOPS, "f32"
    if args.workload in ("hgemm4096", "fc_half"):
        peak, dtype = PEAK_FP16_MFMA_TFLOPS, "f16"     # half storage, exact products, FP32 accumulation
    elif args.workload == "dgemm4096":
        peak, dtype = PEAK_FP64_MFMA_TFLOPS, "f64"
    roofline = {
        "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
        "frac": achieved / peak,
        "traffic": MEASURED_HBM_TRAFFIC_BYTES.get(args.workload),
        "algorithmic_bytes_per_step": alg_bytes,
        "algorithmic_GBps": alg_bytes / ms_ev / 1e6,
        "hbm_frac": alg_bytes / ms_ev / 1e6 / PEAK_HBM_GBS,
    }
    line = {
        "metric": "FP32 GEMM TFLOP/s at 4096^3 on 1 MI355X; % of FP32 MFMA peak" if args.workload == "gemm4096"
                  else "%s TFLOP/s on workload %s on 1 MI355X" % ({"f32": "FP32", "f16": "FP16-storage / FP32-accumulate",
                                                                   "f64": "FP64"}[dtype], wl_name),
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_ev, "ms_per_step_median": spread["median"], "ms_per_step_min": spread["min"],
        "ms_per_step_max": spread["max"], "ms_per_step_batches": batches, "events_per": timing["events_per"],
        "value_at_median_step": flop / spread["median"] / 1e9,
        "ms_per_step_host_clock": ms_wall, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": wl_name, "launches_per_step": launches, "flop_per_step": flop, "graph_replay": bool(args.graph),
                   "tile_config": dm.dmath_config_name(args.tile_config) if args.tile_config >= 0 else "auto",
                   "library": dm.dmath_version()},
        "pct_of_fp32_mfma_peak": 100.0 * tflops / peak if dtype == "f32" else None,
        "pct_of_mfma_peak": 100.0 * tflops / peak,
        "measured_shader_clock_ghz": measured_clock_ghz,
        "kernel_us_device_stamps": (lambda t: sum(t) / len(t) if t else None)(
            [k for k in kernel_us[args.warmup:] if k is not None]),   # workgroups 0..7, 100 MHz counter
        "launch_floor_us": launch_floor_us,
        "pct_of_mfma_peak_at_measured_clock":
            None if not measured_clock_ghz
            else 100.0 * tflops / (peak * measured_clock_ghz["mean"] / 2.4),
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "check_vs_oracle": check,
        "paper_context": "dMath paper, table 'Matrix Multiplication Performance': N=4096 on one K80 GPU with "
                         "cuBLAS 7.5 took 0.052 s (about 2.64 TFLOP/s, precision not stated); other hardware, "
                         "context only",
    }
    if args.detail:
        line["per_step_ms"] = [round(v, 5) for v in spans]
        line["shader_clock_ghz_per_step_incl_warmup"] = (None if clock_per_step is None else
                                                         [None if c is None else round(c, 4) for c in clock_per_step])
    if args.workload == "square":
        line["seconds_per_multiply"] = ms_ev / 1e3
        line["paper_table_one_gpu_seconds"] = PAPER_TABLE_ONE_GPU_SECONDS.get(args.size)  # None: did not fit one K80 GPU
    print(json.dumps(line))


if __name__ == "__main__":
    main()
