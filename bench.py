#!/usr/bin/env python3
"""Benchmark of the TBIK hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--extras]

One *step* is one pass of the whole hot path over one batch of the 8B-class attention output
projection workload (X bf16 [4096,4096] ~ N(0,1), W bf16 [4096,4096] ~ N(0,0.02), leaf 256):

    RMSNorm(X)                                                   batch-invariant RMSNorm
    Y      = tbik_gemm(X, W)                                     leaf GEMM + in-kernel tree, whole K (P = 1)
    part_P = tbik_gemm_shard_partials(X, W, P), P in {2,4,8}     per-shard subtree sums (TP emulation)
    Y_P    = tbik_tree_combine(part_P)                           top of the tree + single rounding
    log-softmax over the fp32 rows of Y_8                        tree-ordered row reduction

All inputs are resident in HBM before the timed region.  `value` is the metric itself: the rate of the tree GEMM on
the whole K (tbik_gemm, P = 1, 2*M*K*N flop per call), from HIP events around that call inside every timed step.
`ms_per_step` is the wall time of the whole step and `step_tflops` the GEMM work of a step (4 products) over it: the
step also holds the HBM-bound traffic of the emulated shards, so that figure is neither the kernel's rate nor a
tensor-parallel latency.  After the timed region the outputs for P in {1,2,4,8} are compared bit for bit
(`unique_outputs` must be 1).  `kernels` carries every shape the metric names (o_proj M in {1024, 4096}, down_proj M in
{512, 4096}, weight streaming at small M with the weights rotated through more than the 256 MiB memory-side cache,
RMSNorm 8192 x {4096, 5120}, log-softmax {1, 64, 512} x 151936, tree_combine P in {2, 4, 8}); HBM-bound kernels are
timed cold (buffers rotated through more than the cache) and warm (one buffer set) side by side.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0      # MI355X dense fp8 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
CACHE_BYTES = 256 << 20        # memory-side cache: a buffer set a kernel is to find in HBM is rotated through more than this
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "bench_step_oproj_m4096_pmc.md")


def profiled_traffic():
    """HBM bytes per launch of the dominant kernel (tbik_gemm, P = 1, M = K = N = 4096) as the committed rocprofv3
    FETCH_SIZE / WRITE_SIZE summary states them (line `traffic_bytes_per_launch: N`), or None."""
    try:
        for line in open(TRAFFIC_FILE):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1].split()[0])
    except OSError:
        pass
    return None          # the summary did not travel with this copy of the tree: unmeasured here


def best_ms(fn, iters, torch, reps=3, warm=2):
    for _ in range(warm):
        fn()
    return min(time_region(fn, iters, torch) for _ in range(reps))


def rotating(calls):
    """One callable that walks through `calls` (the same kernel on distinct buffer sets) in turn."""
    state = {"i": 0}

    def fn():
        calls[state["i"] % len(calls)]()
        state["i"] += 1
    return fn


def sets_for_cold(bytes_per_set):
    """How many distinct buffer sets it takes to exceed the memory-side cache (at least 2, at most 64)."""
    return int(max(2, min(64, -(-int(1.5 * CACHE_BYTES) // max(1, bytes_per_set)))))


def time_region(fn, iters, torch):
    """Average milliseconds per call of fn over `iters` back-to-back calls, by HIP events on the current stream."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU oracle timing leg")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of the workload the CPU oracle computes (0 = auto)")
    ap.add_argument("--extras", action="store_true", help="also time each kernel on the other configured shapes")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one plain 1 GiB device-to-device copy (a known-size reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (tensor parallelism is emulated on it by per-shard "
              "partial buffers); --gpus %d is not supported." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2511_17826_amd import binding as tb
    from paper_2511_17826_amd import synthetic as syn

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    tb.lib()   # fail loudly if the HIP library is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)

    M, K, N, leaf, g = 4096, 4096, 4096, 256, 1
    c = syn.gemm_oproj(M)
    to_dev = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev)
    X, W = to_dev(c["X"]), to_dev(c["W"])
    _, wn_bits = syn.rmsnorm_inputs(1, K)
    wnorm = to_dev(wn_bits)
    Ps = (2, 4, 8)

    # every buffer of the step is allocated once, outside the timed region
    xn = torch.empty_like(X)
    y1 = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    parts = {P: torch.empty((P, M, N), dtype=torch.float32, device=dev) for P in Ps}
    yP = {P: torch.empty((M, N), dtype=torch.bfloat16, device=dev) for P in Ps}
    y8f = torch.empty((M, N), dtype=torch.float32, device=dev)
    lsm = torch.empty((M, N), dtype=torch.float32, device=dev)
    ws_gemm = torch.empty(max(256, tb.gemm_workspace_bytes(M, N, K, leaf, g)), dtype=torch.uint8, device=dev)
    ws_rr = torch.empty(max(256, int(tb.lib().tbik_row_reduce_workspace_bytes(M, N, tb.TBIK_LOGSOFTMAX))),
                        dtype=torch.uint8, device=dev)

    def step(gemm_events=None):
        tb.tbik_rmsnorm(X, wnorm, 1e-6, out=xn)
        if gemm_events is not None:
            gemm_events[0].record()
        tb.tbik_gemm(X, W, leaf, g, out=y1, workspace=ws_gemm)
        if gemm_events is not None:
            gemm_events[1].record()
        for P in Ps:
            tb.tbik_gemm_shard_partials(X, W, leaf, g, P, out=parts[P], workspace=ws_gemm)
            tb.tbik_tree_combine(parts[P], out=yP[P])
        tb.tbik_tree_combine(parts[8], out=y8f)
        tb.tbik_row_reduce(y8f, tb.TBIK_LOGSOFTMAX, out=lsm, workspace=ws_rr)

    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    gemm_events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(gemm_events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1e3 * wall / args.steps
    flop_per_step = 4 * 2.0 * M * K * N
    step_tflops = flop_per_step / (ms_per_step * 1e-3) / 1e12
    gemm_ms_in_step = sum(a.elapsed_time(b) for a, b in gemm_events) / max(1, args.steps)
    value = 2.0 * M * K * N / (gemm_ms_in_step * 1e-3) / 1e12      # the metric: the tree GEMM's own rate, measured in the timed steps

    # invariance check on what the timed steps produced
    unique = len({bytes(y.view(torch.int16).cpu().numpy().tobytes()) for y in [y1] + [yP[P] for P in Ps]})

    # ---- roofline of the dominant kernel: the tiled tree GEMM at P = 1 (one launch = 2*M*K*N flop) ----
    gemm_only = lambda: tb.tbik_gemm(X, W, leaf, g, out=y1, workspace=ws_gemm)
    for _ in range(3):
        gemm_only()
    gemm_ms = min(time_region(gemm_only, 20, torch) for _ in range(3))       # the same launch, twenty in a row, right after the steps
    # achieved: the launch's duration inside the timed steps (HIP events on the launch's stream around each of them)
    roofline = {"bound": "mfma", "kernel": "gemm_tiled_kernel (tbik_gemm, P=1, M=4096)", "achieved": round(value, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(value / PEAK_BF16_TFLOPS, 4),
                "launch_ms": round(gemm_ms_in_step, 4), "launch_ms_back_to_back": round(gemm_ms, 4), "traffic": profiled_traffic(),
                "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE x 2.00 + WRITE_SIZE x 1.00, KiB)",
                "algorithmic_bytes": 2 * M * K + 2 * K * N + 2 * M * N}

    # ---- non-invariant baseline GEMM (hipBLASLt / rocBLAS through torch.matmul) on the same operands ----
    base = lambda: torch.matmul(X, W)
    for _ in range(3):
        base()
    base_ms = min(time_region(base, 20, torch) for _ in range(3))
    # the same library splitting K by hand (what two tensor-parallel ranks would compute) does not reproduce its own bits
    whole = torch.matmul(X, W)
    halves = (torch.matmul(X[:, :K // 2], W[:K // 2]).float() + torch.matmul(X[:, K // 2:], W[K // 2:]).float()).to(torch.bfloat16)
    base_mismatch = int((whole.view(torch.int16) != halves.view(torch.int16)).sum().item())
    del whole, halves
    baseline_gemm = {"kind": "torch.matmul bf16 (hipBLASLt/rocBLAS), not shard-invariant", "ms": round(base_ms, 4),
                     "tflops": round(2.0 * M * K * N / (base_ms * 1e-3) / 1e12, 2),
                     "elements_changed_by_splitting_K_in_two": base_mismatch, "elements": M * N}

    # ---- the other kernels of the step, timed alone on the step's own (cache-resident) buffers ----
    kernels = {}
    t = best_ms(lambda: tb.tbik_rmsnorm(X, wnorm, 1e-6, out=xn), 20, torch)
    kernels["rmsnorm_4096x4096_warm"] = {"ms": round(t, 4), "GBps": round(4.0 * M * K / (t * 1e-3) / 1e9, 1),
                                         "note": "64 MiB of buffers, served by the 256 MiB memory-side cache: not an HBM figure"}
    t = best_ms(lambda: tb.tbik_row_reduce(y8f, tb.TBIK_LOGSOFTMAX, out=lsm, workspace=ws_rr), 20, torch)
    kernels["logsoftmax_4096x4096_warm"] = {"ms": round(t, 4), "GBps": round(8.0 * M * N / (t * 1e-3) / 1e9, 1),
                                            "note": "128 MiB of buffers, cache-assisted"}
    for P in Ps:
        t = min(time_region(lambda: tb.tbik_gemm_shard_partials(X, W, leaf, g, P, out=parts[P], workspace=ws_gemm), 10, torch)
                for _ in range(2))
        kernels["shard_partials_P%d" % P] = {"ms": round(t, 4), "tflops": round(2.0 * M * K * N / (t * 1e-3) / 1e12, 2)}

    # one rank's share under real tensor parallelism: the shard kernel alone at its real shape [M, K/P] x [K/P, N]
    # (fp32 partial out); the wire and the other P-1 GPUs are what this leaves out
    for P in Ps:
        Xp, Wp = X[:, :K // P], W[:K // P]
        f = lambda: tb.tbik_gemm_shard_partials(Xp, Wp, leaf, g, 1, out=parts[P][:1], workspace=ws_gemm)
        f()
        t = min(time_region(f, 20, torch) for _ in range(3))
        kernels["one_rank_share_P%d" % P] = {"ms": round(t, 4), "tflops": round(2.0 * M * (K // P) * N / (t * 1e-3) / 1e12, 2)}

    del parts, yP, y8f, lsm, xn
    kernels.update(metric_shapes(tb, syn, torch, np, to_dev, X, W))
    if args.extras:
        kernels.update(extras(tb, syn, torch, np, to_dev))
    else:                                                   # three attention lines in every run; --extras has them all
        kernels.update(attention_lines(tb, torch, ((4, 4096, torch.bfloat16),),
                                       ((64, 4096, torch.bfloat16), (1, 32768, torch.bfloat16))))

    out = {
        "metric": "TBIK GEMM TFLOP/s (% bf16 MFMA peak), bit-identical across P in {1,2,4,8}",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "8B-class o_proj: X bf16 [4096,4096] ~N(0,1), W bf16 [4096,4096] ~N(0,0.02), leaf 256, "
                               "k_first 1; step = RMSNorm + tbik_gemm(P=1) + shard_partials/tree_combine for P in {2,4,8} "
                               "+ log-softmax over the fp32 output rows; value = rate of tbik_gemm(P=1) inside the step",
                   "M": M, "K": K, "N": N, "leaf": leaf, "k_first": g, "P": [1, 2, 4, 8]},
        "pct_of_bf16_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "gemm_ms_in_step": round(gemm_ms_in_step, 4),
        "step_tflops": round(step_tflops, 2),
        "unique_outputs": unique,
        "roofline": roofline,
        "baseline_gemm": baseline_gemm,
        "kernels": kernels,
        "paper_context": "paper reports ~120 TFLOP/s = 63% of cuBLAS for its Triton kernel (BF16, K=6144, N=2048; "
                         "NVIDIA GPU, block sizes tuned on L40S) -- other hardware, context only",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(c, leaf, g, args.cpu_rows)
    print(json.dumps(out))


def cpu_baseline(c, leaf, g, rows):
    """The CPU oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    from oracle import tbik_oracle as orc
    ncores = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))
    K, N = c["K"], c["N"]
    if rows <= 0:
        t0 = time.perf_counter()
        orc.gemm(c["X"][:4], c["W"], leaf, g)                 # calibration: 4 rows
        per_row = (time.perf_counter() - t0) / 4
        rows = int(max(8, min(4096, 15.0 / max(per_row, 1e-6))))
    t0 = time.perf_counter()
    orc.gemm(c["X"][:rows], c["W"], leaf, g)
    dt = time.perf_counter() - t0
    return {"value": round(2.0 * rows * K * N / dt / 1e12, 5), "unit": "TFLOP/s", "cores": ncores, "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": "first %d of 4096 rows of the same X against the full W (whole K, all N), fp32 scalar tree order" % rows}


def metric_shapes(tb, syn, torch, np, to_dev, X, W):
    """Every shape the metric names, one line each (in every run).  MFMA-bound lines carry `frac` of the 2.5 PFLOP/s bf16
    peak and the time of torch.matmul on the same operands; HBM-bound lines carry GB/s and `frac_hbm` of 8 TB/s, cold
    (buffer sets rotated through more than the memory-side cache) and warm (one set)."""
    res = {}
    dev = X.device

    def gemm_line(name, Xd, Wd, M, leaf, g, iters):
        K, N = Wd.shape
        y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        ws = torch.empty(max(256, tb.gemm_workspace_bytes(M, N, K, leaf, g)), dtype=torch.uint8, device=dev)
        t = best_ms(lambda: tb.tbik_gemm(Xd[:M], Wd, leaf, g, out=y, workspace=ws), iters, torch)
        tbase = best_ms(lambda: torch.matmul(Xd[:M], Wd, out=y), iters, torch)
        tf = 2.0 * M * K * N / (t * 1e-3) / 1e12
        res[name] = {"ms": round(t, 4), "tflops": round(tf, 1), "frac": round(tf / PEAK_BF16_TFLOPS, 4),
                     "baseline_ms": round(tbase, 4)}

    def streaming_line(name, Xd, Wd, M, leaf, g, copies):
        """Small M: the weights are the traffic.  `copies` distinct copies of W (more than the cache in all) are walked by
        calls captured in one HIP graph, so neither the host nor the cache stands between the kernel and HBM."""
        K, N = Wd.shape
        Ws = [Wd] + [Wd.clone() for _ in range(copies - 1)]
        y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        ws = torch.empty(max(256, tb.gemm_workspace_bytes(M, N, K, leaf, g)), dtype=torch.uint8, device=dev)
        side = torch.cuda.Stream()
        per_call = {}
        for kind, call in (("tbik", lambda Wc: tb.tbik_gemm(Xd[:M], Wc, leaf, g, out=y, workspace=ws)),
                           ("baseline", lambda Wc: torch.matmul(Xd[:M], Wc, out=y))):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                call(Ws[0])
                torch.cuda.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    for Wc in Ws:
                        call(Wc)
            graph.replay()
            torch.cuda.synchronize()
            per_call[kind] = min(time_region(graph.replay, 5, torch) for _ in range(3)) / len(Ws)
        warm = best_ms(lambda: tb.tbik_gemm(Xd[:M], Wd, leaf, g, out=y, workspace=ws), 20, torch)
        t = per_call["tbik"]
        gbs = 2.0 * K * N / (t * 1e-3) / 1e9
        res[name] = {"ms_cold_in_graph": round(t, 4), "GBps_weights": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4),
                     "baseline_ms_cold_in_graph": round(per_call["baseline"], 4), "ms_warm_per_python_call": round(warm, 4)}

    gemm_line("oproj_M1024", X, W, 1024, 256, 1, 20)
    gemm_line("oproj_M4096", X, W, 4096, 256, 1, 20)
    for M in (1, 16, 64):
        streaming_line("oproj_M%d_weights_from_hbm" % M, X, W, M, 256, 1, 10)        # 10 x 32 MiB
    c = syn.gemm_downproj(4096)
    Xd, Wd = to_dev(c["X"]), to_dev(c["W"])
    gemm_line("downproj_M512", Xd, Wd, 512, 256, 3, 10)
    gemm_line("downproj_M4096", Xd, Wd, 4096, 256, 3, 10)
    for M in (1, 64):
        streaming_line("downproj_M%d_weights_from_hbm" % M, Xd, Wd, M, 256, 3, 4)    # 4 x 96 MiB
    del Xd, Wd

    # The MLP's first GEMM with the gated activation applied before anything is stored (8B class: K = 4096,
    # I = 12288), next to the same work as a GEMM into [M, 2 I] followed by the activation kernel.
    I_mlp = 12288
    rng_w = torch.Generator(device=dev)
    rng_w.manual_seed(6)
    Wgu = (torch.randn((X.shape[1], 2 * I_mlp), generator=rng_w, device=dev, dtype=torch.float32) * 0.02).to(torch.bfloat16)
    for M in (512, 4096):
        act = torch.empty((M, I_mlp), dtype=torch.bfloat16, device=dev)
        gu = torch.empty((M, 2 * I_mlp), dtype=torch.bfloat16, device=dev)
        ws = torch.empty(max(256, tb.gemm_swiglu_workspace_bytes(M, I_mlp, X.shape[1], 256, 1)), dtype=torch.uint8, device=dev)

        def two_calls():
            tb.tbik_gemm(X[:M], Wgu, 256, 1, out=gu)
            tb.tbik_silu_mul(gu[:, :I_mlp], gu[:, I_mlp:], out=act)
        # interleaved, so that both see the same clocks
        t_f, t_u = 1e9, 1e9
        for _ in range(3):
            t_f = min(t_f, best_ms(lambda: tb.tbik_gemm_swiglu(X[:M], Wgu, 256, 1, out=act, workspace=ws), 4, torch))
            t_u = min(t_u, best_ms(two_calls, 4, torch))
        tf = 2.0 * M * X.shape[1] * 2 * I_mlp / (t_f * 1e-3) / 1e12
        res["gateup_swiglu_M%d" % M] = {"ms": round(t_f, 4), "tflops": round(tf, 1), "frac": round(tf / PEAK_BF16_TFLOPS, 4),
                                        "ms_gemm_then_activation": round(t_u, 4)}
        del act, gu, ws
    del Wgu

    # 8-bit floating-point operands (E4M3), the two row-parallel shapes at M = 4096, beside torch._scaled_mm (hipBLASLt).
    for name, K8, leaf8, g8 in (("fp8_oproj_M4096", 4096, 256, 1), ("fp8_downproj_M4096", 12288, 256, 3)):
        g8r = torch.Generator(device=dev)
        g8r.manual_seed(K8)
        X8 = torch.randn((4096, K8), generator=g8r, device=dev, dtype=torch.float32).to(torch.float8_e4m3fn)
        Wt8 = torch.randn((4096, K8), generator=g8r, device=dev, dtype=torch.float32).to(torch.float8_e4m3fn)
        y8 = torch.empty((4096, 4096), dtype=torch.bfloat16, device=dev)
        ws8 = torch.empty(max(256, tb.gemm_fp8_workspace_bytes(4096, 4096, K8, leaf8, g8)), dtype=torch.uint8, device=dev)
        t = best_ms(lambda: tb.tbik_gemm_fp8(X8, Wt8, leaf8, g8, "e4m3", out=y8, workspace=ws8), 10, torch)
        one = torch.ones((), device=dev)
        try:
            tbase = best_ms(lambda: torch._scaled_mm(X8, Wt8.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16), 10, torch)
        except Exception:                      # no 8-bit matmul in this torch build: the line carries no baseline
            tbase = None
        tf = 2.0 * 4096 * K8 * 4096 / (t * 1e-3) / 1e12
        res[name] = {"ms": round(t, 4), "tflops": round(tf, 1), "frac_fp8_peak": round(tf / PEAK_FP8_TFLOPS, 4),
                     "baseline_ms": round(tbase, 4) if tbase else None}
        # small batches: the 8-bit weight is the traffic; copies of it (more than the cache in all) walked inside one HIP graph
        copies = max(2, -(-int(1.5 * CACHE_BYTES) // (4096 * K8)))
        Wts = [Wt8] + [Wt8.clone() for _ in range(copies - 1)]
        side = torch.cuda.Stream()
        for Ms in (1, 64):
            ys = torch.empty((Ms, 4096), dtype=torch.bfloat16, device=dev)
            wss = torch.empty(max(256, tb.gemm_fp8_workspace_bytes(Ms, 4096, K8, leaf8, g8)), dtype=torch.uint8, device=dev)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                tb.tbik_gemm_fp8(X8[:Ms], Wts[0], leaf8, g8, "e4m3", out=ys, workspace=wss)
                torch.cuda.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    for Wc in Wts:
                        tb.tbik_gemm_fp8(X8[:Ms], Wc, leaf8, g8, "e4m3", out=ys, workspace=wss)
            graph.replay()
            torch.cuda.synchronize()
            tc = min(time_region(graph.replay, 5, torch) for _ in range(3)) / len(Wts)
            gbs = 1.0 * K8 * 4096 / (tc * 1e-3) / 1e9
            res[name.replace("M4096", "M%d_weights_from_hbm" % Ms)] = {"ms_cold_in_graph": round(tc, 4), "GBps_weights": round(gbs, 1),
                                                                     "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
            del ys, wss, graph
        del X8, Wt8, y8, ws8, Wts

    # MXFP4 operands (random element and scale bytes: the timing does not depend on the values), same two shapes.
    for name, K4, leaf4, g4 in (("mxfp4_oproj_M4096", 4096, 512, 1), ("mxfp4_downproj_M4096", 12288, 256, 3)):
        g4r = torch.Generator(device=dev)
        g4r.manual_seed(K4 + 1)
        X4 = torch.randint(0, 256, (4096, K4 // 2), generator=g4r, device=dev, dtype=torch.uint8)
        W4 = torch.randint(0, 256, (4096, K4 // 2), generator=g4r, device=dev, dtype=torch.uint8)
        Xs4 = torch.randint(120, 134, (4096, K4 // 32), generator=g4r, device=dev, dtype=torch.uint8)
        Ws4 = torch.randint(120, 134, (4096, K4 // 32), generator=g4r, device=dev, dtype=torch.uint8)
        y4 = torch.empty((4096, 4096), dtype=torch.bfloat16, device=dev)
        ws4 = torch.empty(max(256, tb.gemm_mxfp4_workspace_bytes(4096, 4096, K4, leaf4, g4)), dtype=torch.uint8, device=dev)
        t = best_ms(lambda: tb.tbik_gemm_mxfp4(X4, Xs4, W4, Ws4, leaf4, g4, out=y4, workspace=ws4), 10, torch)
        tf = 2.0 * 4096 * K4 * 4096 / (t * 1e-3) / 1e12
        res[name] = {"ms": round(t, 4), "tflops": round(tf, 1), "frac_fp4_peak": round(tf / 10100.0, 4), "leaf": leaf4}
        del X4, W4, Xs4, Ws4, y4, ws4

    # MXFP8 operands (E4M3 elements from a normal distribution, random scale bytes), same two shapes.
    for name, Kx, leafx, gx in (("mxfp8_oproj_M4096", 4096, 256, 1), ("mxfp8_downproj_M4096", 12288, 256, 3)):
        gxr = torch.Generator(device=dev)
        gxr.manual_seed(Kx + 2)
        Xx = torch.randn((4096, Kx), generator=gxr, device=dev, dtype=torch.float32).to(torch.float8_e4m3fn)
        Wx = torch.randn((4096, Kx), generator=gxr, device=dev, dtype=torch.float32).to(torch.float8_e4m3fn)
        Xsx = torch.randint(120, 134, (4096, Kx // 32), generator=gxr, device=dev, dtype=torch.uint8)
        Wsx = torch.randint(120, 134, (4096, Kx // 32), generator=gxr, device=dev, dtype=torch.uint8)
        yx = torch.empty((4096, 4096), dtype=torch.bfloat16, device=dev)
        wsx = torch.empty(max(256, tb.gemm_mxfp8_workspace_bytes(4096, 4096, Kx, leafx, gx)), dtype=torch.uint8, device=dev)
        t = best_ms(lambda: tb.tbik_gemm_mxfp8(Xx, Xsx, Wx, Wsx, leafx, gx, "e4m3", out=yx, workspace=wsx), 10, torch)
        tf = 2.0 * 4096 * Kx * 4096 / (t * 1e-3) / 1e12
        res[name] = {"ms": round(t, 4), "tflops": round(tf, 1), "frac_fp8_peak": round(tf / PEAK_FP8_TFLOPS, 4)}
        del Xx, Wx, Xsx, Wsx, yx, wsx

    # MXFP6 operands (random element and scale bytes: the timing does not depend on the values), same two shapes.
    for name, K6, leaf6, g6 in (("mxfp6_oproj_M4096", 4096, 256, 1), ("mxfp6_downproj_M4096", 12288, 256, 3)):
        g6r = torch.Generator(device=dev)
        g6r.manual_seed(K6 + 3)
        X6 = torch.randint(0, 256, (4096, K6 * 3 // 4), generator=g6r, device=dev, dtype=torch.uint8)
        W6 = torch.randint(0, 256, (4096, K6 * 3 // 4), generator=g6r, device=dev, dtype=torch.uint8)
        Xs6 = torch.randint(120, 134, (4096, K6 // 32), generator=g6r, device=dev, dtype=torch.uint8)
        Ws6 = torch.randint(120, 134, (4096, K6 // 32), generator=g6r, device=dev, dtype=torch.uint8)
        y6 = torch.empty((4096, 4096), dtype=torch.bfloat16, device=dev)
        ws6 = torch.empty(max(256, tb.gemm_mxfp6_workspace_bytes(4096, 4096, K6, leaf6, g6)), dtype=torch.uint8, device=dev)
        t = best_ms(lambda: tb.tbik_gemm_mxfp6(X6, Xs6, W6, Ws6, leaf6, g6, "e2m3", out=y6, workspace=ws6), 10, torch)
        tf = 2.0 * 4096 * K6 * 4096 / (t * 1e-3) / 1e12
        res[name] = {"ms": round(t, 4), "tflops": round(tf, 1), "frac_fp6_peak": round(tf / 10100.0, 4)}
        del X6, W6, Xs6, Ws6, y6, ws6

    def hbm_line(name, calls, byts, iters):
        cold = best_ms(rotating(calls), iters * len(calls), torch, warm=len(calls))
        warm = best_ms(calls[0], iters, torch)
        res[name] = {"ms_cold": round(cold, 4), "GBps_cold": round(byts / (cold * 1e-3) / 1e9, 1),
                     "frac_hbm": round(byts / (cold * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                     "ms_warm": round(warm, 4), "GBps_warm": round(byts / (warm * 1e-3) / 1e9, 1), "buffer_sets": len(calls)}

    for H in (4096, 5120):
        xb, wb = syn.rmsnorm_inputs(8192, H)
        x0, w = to_dev(xb), to_dev(wb)
        n = sets_for_cold(4 * 8192 * H)
        xs = [x0] + [x0.clone() for _ in range(n - 1)]
        ys = [torch.empty_like(x0) for _ in range(n)]
        hbm_line("rmsnorm_8192x%d" % H, [(lambda i=i: tb.tbik_rmsnorm(xs[i], w, 1e-6, out=ys[i])) for i in range(n)],
                 4.0 * 8192 * H, 10)
        del xs, ys
    V = 151936
    lg = torch.from_numpy(syn.logits_f32(512, V)).to(dev)
    out = torch.empty_like(lg)
    ws_rr = torch.empty(max(256, int(tb.lib().tbik_row_reduce_workspace_bytes(512, V, tb.TBIK_LOGSOFTMAX))), dtype=torch.uint8, device=dev)
    for M in (1, 64, 512):
        # distinct row blocks of the same 512-row tensor (311 MiB in, 311 MiB out) are the buffer sets
        n = 512 // M
        calls = [(lambda i=i: tb.tbik_row_reduce(lg[i * M:(i + 1) * M], tb.TBIK_LOGSOFTMAX, out=out[i * M:(i + 1) * M], workspace=ws_rr))
                 for i in range(n)]
        hbm_line("logsoftmax_%dx151936_8V_basis" % M, calls, 8.0 * M * V, max(1, 16 // n) if n > 16 else 10)
        if M <= 64:
            # a small call is three short launches: inside one HIP graph the host's share of a call is gone
            side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                calls[0]()
                torch.cuda.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    for c in calls:
                        c()
            graph.replay()
            torch.cuda.synchronize()
            tg = min(time_region(graph.replay, 5, torch) for _ in range(3)) / len(calls)
            res["logsoftmax_%dx151936_8V_basis" % M]["ms_cold_in_graph"] = round(tg, 4)
            res["logsoftmax_%dx151936_8V_basis" % M]["GBps_cold_in_graph"] = round(8.0 * M * V / (tg * 1e-3) / 1e9, 1)
    # row sum and row maximum of the same rows: read-only, 4V bytes per row
    red_out = torch.empty(512, dtype=torch.float32, device=dev)
    for opname, op in (("rowsum", tb.TBIK_SUM), ("rowmax", tb.TBIK_MAX)):
        t = best_ms(lambda: tb.tbik_row_reduce(lg, op, out=red_out, workspace=ws_rr), 10, torch)
        res["%s_512x151936" % opname] = {"ms": round(t, 4), "GBps": round(4.0 * 512 * V / (t * 1e-3) / 1e9, 1),
                                         "frac_hbm": round(4.0 * 512 * V / (t * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                         "note": "311 MiB read once per call: more than the memory-side cache holds"}
    del lg, out
    Mc = Nc = 4096
    for P in (2, 4, 8):
        n = sets_for_cold((4 * P + 2) * Mc * Nc)
        ps = [torch.randn((P, Mc, Nc), dtype=torch.float32, device=dev) for _ in range(n)]
        ys = [torch.empty((Mc, Nc), dtype=torch.bfloat16, device=dev) for _ in range(n)]
        hbm_line("tree_combine_P%d_4096x4096" % P, [(lambda i=i: tb.tbik_tree_combine(ps[i], out=ys[i])) for i in range(n)],
                 (4.0 * P + 2) * Mc * Nc, 10)
        if P == 8:
            # Alg. 2 round by round on the same buffers (2 log2 P launches; the bytes every round moves, counted:
            # the reduce rounds read 2 and write 1 buffer per pair, the broadcast rounds read 1 and write 1)
            moved = 4.0 * Mc * Nc * sum(3 * (P >> (l + 1)) + 2 * (P >> (l + 1)) for l in range(3))
            hbm_line("tree_allreduce_rounds_P8_4096x4096", [(lambda i=i: tb.tbik_tree_allreduce(ps[i])) for i in range(n)], moved, 5)
        del ps, ys
    return res


def attention_lines(tb, torch, prefill_shapes, decode_shapes):
    """Fixed-tile attention at 8B-class heads (32 query heads over 8 key/value heads, head dimension 128): causal
    prefills of B sequences of L tokens and decode steps of B sequences over L cached keys, beside torch's SDPA."""
    res = {}
    Hq, Hkv, D = 32, 8, 128
    for B, L, dt in prefill_shapes:
        att = tb.tbik_attention if dt == torch.bfloat16 else tb.tbik_attention_f16
        tag = "" if dt == torch.bfloat16 else "fp16_"
        Q = torch.randn(B * L, Hq, D, device="cuda:0").to(dt)
        K = torch.randn(B * L, Hkv, D, device="cuda:0").to(dt)
        Vv = torch.randn(B * L, Hkv, D, device="cuda:0").to(dt)
        cu = torch.arange(0, B + 1, dtype=torch.int32, device="cuda:0") * L
        O = torch.empty_like(Q)
        ws = torch.empty(max(1, tb.attention_workspace_bytes(B, L, L, Hq, Hkv)), dtype=torch.uint8, device="cuda:0")
        f = lambda: att(Q, K, Vv, cu, cu, L, D ** -0.5, True, out=O, max_seqlen_k=L, workspace=ws)
        f(); f()
        t = min(time_region(f, 10, torch) for _ in range(3))
        q4, k4, v4 = (a.view(B, L, -1, D).transpose(1, 2) for a in (Q, K, Vv))
        b = lambda: torch.nn.functional.scaled_dot_product_attention(q4, k4, v4, is_causal=True, enable_gqa=True)
        b(); b()
        tb_ms = min(time_region(b, 10, torch) for _ in range(3))
        flops = 4.0 * B * L * L * D * Hq / 2                     # causal: half of the score matrix
        res["attention_%sprefill_%dx%d" % (tag, B, L)] = {"ms": round(t, 4), "tflops": round(flops / (t * 1e-3) / 1e12, 1),
                                                   "frac_mfma": round(flops / (t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                                                   "baseline_ms": round(tb_ms, 4)}
        del Q, K, Vv, O, q4, k4, v4
    for B, L, dt in decode_shapes:
        att = tb.tbik_attention if dt == torch.bfloat16 else tb.tbik_attention_f16
        tag = "" if dt == torch.bfloat16 else "fp16_"
        Q = torch.randn(B, Hq, D, device="cuda:0").to(dt)
        K = torch.randn(B * L, Hkv, D, device="cuda:0").to(dt)
        Vv = torch.randn(B * L, Hkv, D, device="cuda:0").to(dt)
        cuq = torch.arange(0, B + 1, dtype=torch.int32, device="cuda:0")
        cuk = cuq * L
        O = torch.empty_like(Q)
        ws = torch.empty(max(1, tb.attention_workspace_bytes(B, 1, L, Hq, Hkv)), dtype=torch.uint8, device="cuda:0")
        f = lambda: att(Q, K, Vv, cuq, cuk, 1, D ** -0.5, True, out=O, max_seqlen_k=L, workspace=ws)
        f(); f()
        t = min(time_region(f, 10, torch) for _ in range(3))
        q4 = Q.view(B, 1, Hq, D).transpose(1, 2)
        k4, v4 = (a.view(B, L, Hkv, D).transpose(1, 2) for a in (K, Vv))
        b = lambda: torch.nn.functional.scaled_dot_product_attention(q4, k4, v4, is_causal=False, enable_gqa=True)
        b(); b()
        tb_ms = min(time_region(b, 10, torch) for _ in range(3))
        byts = 2.0 * B * L * Hkv * D * 2                         # K and V read once
        res["attention_%sdecode_%dx%d" % (tag, B, L)] = {"ms": round(t, 4), "GBps_kv": round(byts / (t * 1e-3) / 1e9, 1),
                                                  "frac_hbm": round(byts / (t * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                                  "baseline_ms": round(tb_ms, 4)}
        del Q, K, Vv, O, q4, k4, v4
    return res


def extras(tb, syn, torch, np, to_dev):
    """Per-kernel timings on the other configured shapes (not part of `value`)."""
    res = {}
    c = syn.gemm_oproj(4096)
    X, W = to_dev(c["X"]), to_dev(c["W"])
    for M in (1, 16, 64, 256, 1024, 4096):
        y = torch.empty((M, 4096), dtype=torch.bfloat16, device=X.device)
        f = lambda: tb.tbik_gemm(X[:M], W, 256, 1, out=y)
        f(); f()
        t = min(time_region(f, 20, torch) for _ in range(3))
        b = lambda: torch.matmul(X[:M], W)
        b(); b()
        tb_ms = min(time_region(b, 20, torch) for _ in range(3))
        res["oproj_M%d" % M] = {"ms": round(t, 4), "tflops": round(2.0 * M * 4096 * 4096 / (t * 1e-3) / 1e12, 2),
                                "GBps_weights": round(2.0 * 4096 * 4096 / (t * 1e-3) / 1e9, 1), "baseline_ms": round(tb_ms, 4)}
    # the same small-M calls as the GPU sees them: ten calls captured in a HIP graph (no host time between launches),
    # each with its own copy of W (320 MiB in all, more than the 256 MiB memory-side cache), so the weights come from HBM
    copies = [W] + [W.clone() for _ in range(9)]
    side = torch.cuda.Stream()
    for M in (1, 16, 64):
        y = torch.empty((M, 4096), dtype=torch.bfloat16, device=X.device)
        ws = torch.empty(max(256, tb.gemm_workspace_bytes(M, 4096, 4096, 256, 1)), dtype=torch.uint8, device=X.device)
        per_call = {}
        for name, call in (("tbik", lambda Wc: tb.tbik_gemm(X[:M], Wc, 256, 1, out=y, workspace=ws)),
                           ("baseline", lambda Wc: torch.matmul(X[:M], Wc, out=y))):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                call(copies[0])
                torch.cuda.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    for Wc in copies:
                        call(Wc)
            graph.replay()
            torch.cuda.synchronize()
            per_call[name] = min(time_region(graph.replay, 5, torch) for _ in range(3)) / len(copies)
        t = per_call["tbik"]
        res["oproj_M%d_graph_weights_from_hbm" % M] = {"ms": round(t, 4), "GBps_weights": round(2.0 * 4096 * 4096 / (t * 1e-3) / 1e9, 1),
                                                       "frac_hbm": round(2.0 * 4096 * 4096 / (t * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                                       "baseline_ms": round(per_call["baseline"], 4)}
    del copies, X, W
    c = syn.gemm_downproj(4096)
    X, W = to_dev(c["X"]), to_dev(c["W"])
    for M in (1, 64, 512, 4096):
        y = torch.empty((M, 4096), dtype=torch.bfloat16, device=X.device)
        f = lambda: tb.tbik_gemm(X[:M], W, 256, 3, out=y)
        f(); f()
        t = min(time_region(f, 10, torch) for _ in range(3))
        b = lambda: torch.matmul(X[:M], W)
        b(); b()
        tb_ms = min(time_region(b, 10, torch) for _ in range(3))
        res["downproj_M%d" % M] = {"ms": round(t, 4), "tflops": round(2.0 * M * 12288 * 4096 / (t * 1e-3) / 1e12, 2),
                                   "GBps_weights": round(2.0 * 12288 * 4096 / (t * 1e-3) / 1e9, 1), "baseline_ms": round(tb_ms, 4)}
    del X, W
    # second 8B-class shape set: K = 14336 = 7 * 2^11 (leaf 256, K_first 7, 8 superleaves of 1792)
    c = syn.gemm_downproj(4096, seed=5, K=14336, N=4096, leaf=256, k_first=7)
    X, W = to_dev(c["X"]), to_dev(c["W"])
    for M in (64, 4096):
        y = torch.empty((M, 4096), dtype=torch.bfloat16, device=X.device)
        f = lambda: tb.tbik_gemm(X[:M], W, 256, 7, out=y)
        f(); f()
        t = min(time_region(f, 10, torch) for _ in range(3))
        b = lambda: torch.matmul(X[:M], W)
        b(); b()
        tb_ms = min(time_region(b, 10, torch) for _ in range(3))
        res["downproj_k14336_M%d" % M] = {"ms": round(t, 4), "tflops": round(2.0 * M * 14336 * 4096 / (t * 1e-3) / 1e12, 2),
                                          "baseline_ms": round(tb_ms, 4)}
    del X, W
    # 32B-class row-parallel shapes: hidden 5120, intermediate 25600; leaf 128 with K_first 5 / 25 gives 8 superleaves
    for name, K, N, g in (("oproj32b_k5120", 5120, 5120, 5), ("downproj32b_k25600", 25600, 5120, 25)):
        X = torch.randn((4096, K), device="cuda:0").to(torch.bfloat16)
        W = (torch.randn((K, N), device="cuda:0") * 0.02).to(torch.bfloat16)
        for M in (64, 4096):
            y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
            f = lambda: tb.tbik_gemm(X[:M], W, 128, g, out=y)
            f(); f()
            t = min(time_region(f, 10, torch) for _ in range(3))
            b = lambda: torch.matmul(X[:M], W)
            b(); b()
            tb_ms = min(time_region(b, 10, torch) for _ in range(3))
            res["%s_M%d" % (name, M)] = {"ms": round(t, 4), "tflops": round(2.0 * M * K * N / (t * 1e-3) / 1e12, 2),
                                         "baseline_ms": round(tb_ms, 4)}
        del X, W
    # fp16 operands at the o_proj shape (same kernel, the other MFMA opcode)
    c = syn.gemm_oproj(4096, fmt="fp16")
    X = torch.from_numpy(c["X"].view(np.int16)).view(torch.float16).to("cuda:0")
    W = torch.from_numpy(c["W"].view(np.int16)).view(torch.float16).to("cuda:0")
    for M in (1, 64, 4096):
        y = torch.empty((M, 4096), dtype=torch.float16, device=X.device)
        f = lambda: tb.tbik_gemm_f16(X[:M], W, 256, 1, out=y)
        f(); f()
        t = min(time_region(f, 20, torch) for _ in range(3))
        b = lambda: torch.matmul(X[:M], W)
        b(); b()
        tb_ms = min(time_region(b, 20, torch) for _ in range(3))
        res["oproj_fp16_M%d" % M] = {"ms": round(t, 4), "tflops": round(2.0 * M * 4096 * 4096 / (t * 1e-3) / 1e12, 2),
                                     "baseline_ms": round(tb_ms, 4)}
    del X, W
    # fp32 operands: the shape of the paper's kernel figure (K = 6144, N = 2048; leaf 128 = its FP32 block, K_first 3)
    # and the o_proj shape; peak of the fp32 matrix instruction: 157.3 TFLOP/s
    for name, K, N, leaf, g in (("fp32_k6144_n2048", 6144, 2048, 128, 3), ("oproj_fp32", 4096, 4096, 256, 1)):
        Xf, Wf = syn.gemm_random_f32(4, 4096, K, N)
        X, W = torch.from_numpy(Xf).to("cuda:0"), torch.from_numpy(Wf).to("cuda:0")
        for M in (64, 4096):
            y = torch.empty((M, N), dtype=torch.float32, device=X.device)
            f = lambda: tb.tbik_gemm_f32(X[:M], W, leaf, g, out=y)
            f(); f()
            t = min(time_region(f, 5, torch) for _ in range(3))
            b = lambda: torch.matmul(X[:M], W)
            b(); b()
            tb_ms = min(time_region(b, 5, torch) for _ in range(3))
            tf = 2.0 * M * K * N / (t * 1e-3) / 1e12
            res["%s_M%d" % (name, M)] = {"ms": round(t, 4), "tflops": round(tf, 2), "frac_mfma_fp32": round(tf / 157.3, 4),
                                         "baseline_ms": round(tb_ms, 4)}
        del X, W
    for H in (4096, 5120):
        xb, wb = syn.rmsnorm_inputs(8192, H)
        x, w = to_dev(xb), to_dev(wb)
        y = torch.empty_like(x)
        f = lambda: tb.tbik_rmsnorm(x, w, 1e-6, out=y)
        f(); f()
        t = min(time_region(f, 20, torch) for _ in range(3))
        res["rmsnorm_8192x%d" % H] = {"ms": round(t, 4), "GBps": round(4.0 * 8192 * H / (t * 1e-3) / 1e9, 1)}
    # fused tail of a row-parallel layer (combine + residual add + RMSNorm) against the three separate calls
    M, H = 4096, 4096
    xb, wb = syn.rmsnorm_inputs(M, H)
    resid, wn = to_dev(xb), to_dev(wb)
    for P in (2, 8):
        parts = torch.randn((P, M, H), device="cuda:0", dtype=torch.float32)
        hid, out, ybf = torch.empty_like(resid), torch.empty_like(resid), torch.empty_like(resid)
        fused = lambda: tb.tbik_combine_residual_rmsnorm(parts, resid, wn, 1e-6, hidden=hid, normed=out)

        def separate():
            tb.tbik_tree_combine(parts, out=ybf)
            torch.add(ybf, resid, out=hid)
            tb.tbik_rmsnorm(hid, wn, 1e-6, out=out)

        fused(); separate()
        t = min(time_region(fused, 20, torch) for _ in range(3))
        t3 = min(time_region(separate, 20, torch) for _ in range(3))
        byts = (4.0 * P + 2 + 2 + 2) * M * H
        res["fused_tail_P%d_4096x4096" % P] = {"ms": round(t, 4), "GBps": round(byts / (t * 1e-3) / 1e9, 1),
                                               "frac_hbm": round(byts / (t * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                               "three_calls_ms": round(t3, 4)}
        del parts
    res.update(attention_lines(tb, torch,
                               ((4, 4096, torch.bfloat16), (1, 16384, torch.bfloat16), (4, 4096, torch.float16)),
                               ((64, 4096, torch.bfloat16), (256, 2048, torch.bfloat16), (64, 4096, torch.float16),
                                (1, 32768, torch.bfloat16), (4, 32768, torch.bfloat16), (1, 131072, torch.bfloat16))))
    # a serving step: one 2048-token chunk (over 2048 keys) and 256 decode steps at 2048 keys in one call
    Hq, Hkv, D = 32, 8, 128
    lq, lk = [1] * 256 + [2048], [2048] * 257
    Q = torch.randn(sum(lq), Hq, D, device="cuda:0").to(torch.bfloat16)
    K = torch.randn(sum(lk), Hkv, D, device="cuda:0").to(torch.bfloat16)
    Vv = torch.randn(sum(lk), Hkv, D, device="cuda:0").to(torch.bfloat16)
    cuq = torch.tensor(np.concatenate([[0], np.cumsum(lq)]), dtype=torch.int32, device="cuda:0")
    cuk = torch.tensor(np.concatenate([[0], np.cumsum(lk)]), dtype=torch.int32, device="cuda:0")
    O = torch.empty_like(Q)
    f = lambda: tb.tbik_attention(Q, K, Vv, cuq, cuk, 2048, D ** -0.5, True, out=O, max_seqlen_k=2048)
    f(); f()
    t = min(time_region(f, 10, torch) for _ in range(3))
    res["attention_chunk_2048_plus_256_decodes_at_2048"] = {"ms": round(t, 4), "GBps_kv": round(4.0 * sum(lk) * Hkv * D / (t * 1e-3) / 1e9, 1)}
    del Q, K, Vv, O
    V = 151936
    for M in (1, 64, 512):
        x = torch.from_numpy(syn.logits_f32(M, V)).to("cuda:0")
        o = torch.empty_like(x)
        f = lambda: tb.tbik_row_reduce(x, tb.TBIK_LOGSOFTMAX, out=o)
        f(); f()
        t = min(time_region(f, 10, torch) for _ in range(3))
        res["logsoftmax_%dx151936" % M] = {"ms": round(t, 4), "GBps_8V_basis": round(8.0 * M * V / (t * 1e-3) / 1e9, 1)}
    return res


if __name__ == "__main__":
    main()
