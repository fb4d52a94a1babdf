#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu] [--no-sgemm]

A step is one gradient of the 400-480-3203 network (the paper's network, section 6.1) over a batch of 4096
synthetic patterns, through ulsnn_mlp_grad: every stage of the path (two forward products with their fused
epilogues, softmax / cross-entropy / output delta, three backward products, loss).  Inputs are resident in HBM
before the timed region.  Before the W warm-up steps the same step runs untimed for --settle-seconds (0.15 s,
reported as "settle_steps"): for its first ~40 ms under load a fresh process runs 2-10 % slower.  Flops are counted with the paper's convention (section 6.2): batch * (4 n_i n_h +
6 n_h n_o); elementwise and reduction work counts as zero.  The same run also times the standalone SGEMM at the
square sizes of the second workload (reported under "sgemm").

"roofline" describes the dominant kernel of the step: the matrix-core GEMM launch that takes the most time,
timed live with HIP events recorded on the launch stream (ulsnn_mlp_grad_timed), against the MI355X fp32 matrix
peak of 157.3 TFLOP/s (nominal 2.4 GHz) and, as "frac_at_measured_clock", against the same 256 flop per clock and
compute unit at the shader clock a probe wavefront measured while the step was running ("device").
"unsettled" is the same K steps timed straight after the W warm-up steps of a fresh process, before any settling.
"cpu_baseline" is the CPU oracle (float arithmetic) timed on the host cores on the same workload;
"cpu_baselines" holds it for the other workloads (small network, SGEMM, bf16-rounded inputs), on stated samples.
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

PEAK_FP32_MFMA_TFLOPS = 157.3      # 256 CUs x 256 flop/clk/CU x 2.4 GHz
FLOP_PER_CLK_PER_CU = 256          # fp32 matrix instructions
# HBM bytes per launch of each stage's kernels (calibrated rocprofv3 counters) are read from this summary at run time:
# its lines "bench_traffic: stage=<name> bytes_per_launch=<n>".
TRAFFIC_PROFILE = os.path.join("profiles", "mlp_grad_b4096_hbm_traffic_pmc.md")
TRAFFIC_PROFILE_BF16 = os.path.join("profiles", "mlp_grad_bf16_b65536_hbm_traffic_pmc.md")
PEAK_HBM_GBS = 8000.0


def pmc_traffic(profile=TRAFFIC_PROFILE):
    out = {}
    try:
        for line in open(os.path.join(ROOT, profile)):
            if line.startswith("bench_traffic:"):
                f = dict(kv.split("=") for kv in line.split()[1:])
                out[f["stage"]] = float(f["bytes_per_launch"])
    except OSError:
        pass
    return out
METRIC = "fp32 GFLOP/s (% of MFMA FP32 peak); MLP gradient patterns/sec"
BATCH = 4096
SEED = 2


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-seconds", type=float, default=0.15,
                    help="before the warm-up steps, run the step untimed for this long: the first ~40 ms of load "
                         "after a process starts run 2-10 %% slower (clocks ramping up)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-sgemm", action="store_true", help="skip the standalone SGEMM sweep")
    ap.add_argument("--sgemm-sizes", type=int, nargs="*", default=[256, 1024, 4096, 8192])
    ap.add_argument("--no-bf16", action="store_true", help="skip the bf16-operand workload (batch 65536)")
    ap.add_argument("--no-large-batch", action="store_true", help="skip the fp32 batch-262144 chunk measurement")
    ap.add_argument("--no-small-net", action="store_true", help="skip the 64-32-10 latency measurement")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the squared-error, error-only and optimiser-step measurements (batch 4096)")
    ap.add_argument("--no-epoch", action="store_true",
                    help="skip the whole 9,000,000-pattern epoch (14.4 GB of patterns generated on the GPU)")
    ap.add_argument("--epoch", action="store_true", help="accepted for compatibility: the epoch runs by default")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (reference for HBM byte counters)")
    return ap.parse_args()


def settle(torch, f, seconds):
    """Run f() untimed for `seconds`: a GPU that has idled (host-side work between two measurements) or a fresh
    process runs its first tens of milliseconds under load several per cent slower."""
    t = time.perf_counter()
    while time.perf_counter() - t < seconds:
        f()
        torch.cuda.synchronize()


def bench_sgemm(ulsnn, si, torch, sizes):
    """alpha = 1, beta = 0.5, entries uniform[-1,1], seed 1; NN, NT, TN.  `ms` = one call's share of a run of
    back-to-back calls bracketed by two events (throughput; what `gflops` is computed from); `ms_single` = median
    of calls timed one at a time with an event on each side and a synchronisation in between (latency: adds the
    event overhead and an idle gap, which dominates below 1024)."""
    out = {}
    for size in sizes:
        m = n = k = size
        A, B, C0 = si.gemm_operands(1, m, k, k, n, m, n, device="cuda:0")
        for ta, tb in (("N", "N"), ("N", "T"), ("T", "N")):
            Cm = C0.clone()
            reps = 30 if size <= 1024 else (10 if size <= 4096 else 5)
            settle(torch, lambda: ulsnn.sgemm(ta, tb, m, n, k, 1.0, A, k, B, n, 0.5, Cm, n), 0.03)
            times = []
            for _ in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                ulsnn.sgemm(ta, tb, m, n, k, 1.0, A, k, B, n, 0.5, Cm, n)
                e1.record()
                e1.synchronize()
                times.append(e0.elapsed_time(e1))
            times.sort()
            single = times[len(times) // 2]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                ulsnn.sgemm(ta, tb, m, n, k, 1.0, A, k, B, n, 0.5, Cm, n)
            e1.record()
            e1.synchronize()
            per_call = e0.elapsed_time(e1) / reps
            gf = ulsnn.sgemm_flops(m, n, k) / (per_call * 1e-3) / 1e9
            out[f"{ta}{tb}_{size}"] = {"ms": round(per_call, 4), "ms_single": round(single, 4), "gflops": round(gf, 1),
                                      "frac_of_peak": round(gf / (PEAK_FP32_MFMA_TFLOPS * 1e3), 4)}
        del A, B, C0
    return out


def bench_sgemm_strided_and_cold(ulsnn, si, torch, sizes):
    """The paper times its SGEMM with a stride that differs from the row length and with the caches flushed
    (section 3.4).  "ld_plus_8" / "ld_odd": all three operands stored with leading dimension N + 8 / N + 1 (rows
    then start 32 / 4 bytes off the 16-byte grid), throughput timing as in bench_sgemm.  "cold": sizes up to 1024,
    one call at a time, a 512 MB buffer rewritten between calls so that no operand is left in L2 or the Infinity
    Cache; median of the calls."""
    out = {}
    big = max((s_ for s_ in sizes if s_ >= 2048), default=None)
    if big is not None:
        m = n = k = big
        for tag, pad in (("ld_plus_8", 8), ("ld_odd", 1)):
            ld = big + pad
            A, B, C0 = si.gemm_operands(1, m, k, k, n, m, n, ld, ld, ld, device="cuda:0")
            for ta, tb in (("N", "N"), ("N", "T"), ("T", "N")):
                Cm = C0.clone()
                settle(torch, lambda: ulsnn.sgemm(ta, tb, m, n, k, 1.0, A, ld, B, ld, 0.5, Cm, ld), 0.03)
                reps = 10
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    ulsnn.sgemm(ta, tb, m, n, k, 1.0, A, ld, B, ld, 0.5, Cm, ld)
                e1.record()
                e1.synchronize()
                per_call = e0.elapsed_time(e1) / reps
                gf = ulsnn.sgemm_flops(m, n, k) / (per_call * 1e-3) / 1e9
                out[f"{ta}{tb}_{big}_{tag}"] = {"ld": ld, "ms": round(per_call, 4), "gflops": round(gf, 1),
                                               "frac_of_peak": round(gf / (PEAK_FP32_MFMA_TFLOPS * 1e3), 4)}
            del A, B, C0
    scrub = torch.empty(128 << 20, dtype=torch.float32, device="cuda:0")      # 512 MB > 256 MB Infinity Cache
    for size in (s_ for s_ in sizes if s_ <= 1024):
        m = n = k = size
        A, B, C0 = si.gemm_operands(1, m, k, k, n, m, n, device="cuda:0")
        for ta, tb in (("N", "N"), ("N", "T"), ("T", "N")):
            Cm = C0.clone()
            times = []
            for _ in range(9):
                scrub.fill_(1.0)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                ulsnn.sgemm(ta, tb, m, n, k, 1.0, A, k, B, n, 0.5, Cm, n)
                e1.record()
                e1.synchronize()
                times.append(e0.elapsed_time(e1))
            times.sort()
            ms = times[len(times) // 2]
            gf = ulsnn.sgemm_flops(m, n, k) / (ms * 1e-3) / 1e9
            out[f"{ta}{tb}_{size}_cold"] = {"ms_single": round(ms, 4), "gflops": round(gf, 1),
                                            "frac_of_peak": round(gf / (PEAK_FP32_MFMA_TFLOPS * 1e3), 4)}
        del A, B, C0
    del scrub
    # with a workspace (ulsnn_sgemm_ws) the planner may cut k into slices where a product cannot fill the chip
    for tag, (ta, tb, m, n, k) in (("NN_512", ("N", "N", 512, 512, 512)), ("TN_256x256x65536", ("T", "N", 256, 256, 65536))):
        A, B, C0 = si.gemm_operands(1, *((m, k) if ta == "N" else (k, m)), *((k, n) if tb == "N" else (n, k)), m, n,
                                    device="cuda:0")
        lda, ldb = A.shape[1], B.shape[1]
        ws = torch.empty(64 * m * n * 4, dtype=torch.uint8, device="cuda:0")
        row = {"plan": ulsnn.sgemm_ws_describe_plan(ta, tb, m, n, k, ws.numel()).strip()}
        for name, f in (("ms", lambda: ulsnn.sgemm(ta, tb, m, n, k, 1.0, A, lda, B, ldb, 0.5, C0, n)),
                        ("ms_with_workspace", lambda: ulsnn.sgemm_ws(ta, tb, m, n, k, 1.0, A, lda, B, ldb, 0.5, C0, n, ws))):
            settle(torch, f, 0.03)
            reps = 50
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                f()
            e1.record()
            e1.synchronize()
            row[name] = round(e0.elapsed_time(e1) / reps, 4)
        row["gflops_with_workspace"] = round(ulsnn.sgemm_flops(m, n, k) / (row["ms_with_workspace"] * 1e-3) / 1e9, 1)
        out[f"{tag}_split_k"] = row
        del A, B, C0, ws
    return out


def cpu_baseline(si, shape, W1, W2, X, y):
    import numpy as np

    import oracle
    t0 = time.perf_counter()
    g = oracle.mlp_grad(W1.numpy(), W2.numpy(), X.numpy(), y.numpy(), dtype=np.float32)
    dt = time.perf_counter() - t0
    flops = oracle.grad_flops(X.shape[0], shape.n_in, shape.n_hid, shape.n_out)
    return {"value": round(flops / dt / 1e9, 3), "unit": "GFLOP/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"the whole workload once: {X.shape[0]} patterns, float-arithmetic oracle, {dt:.2f} s",
            "patterns_per_s": round(X.shape[0] / dt, 1), "loss": g.loss}


def cpu_baselines_other(si, torch, shape, W1, W2):
    """The oracle timed on the other workloads, each on a bounded, stated sample (a few seconds of host time)."""
    import numpy as np

    import oracle
    out = {}
    # small network, batch 256, with biases: the whole workload, repeated
    sm = si.MLP_SMALL
    sW1, sW2, sb1, sb2 = (t.numpy() for t in si.mlp_weights(sm, 0))
    sX, sy = (t.numpy() for t in si.mlp_patterns(sm, 0, 0, 256))
    reps = 20
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.mlp_grad(sW1, sW2, sX, sy, sb1, sb2, dtype=np.float32)
    dt = (time.perf_counter() - t0) / reps
    out["small_net"] = {"value": round(oracle.grad_flops(256, sm.n_in, sm.n_hid, sm.n_out) / dt / 1e9, 3),
                        "unit": "GFLOP/s", "us_per_call": round(dt * 1e6, 1), "cores": oracle.threads(), "kind": "oracle",
                        "sample": f"64-32-10, batch 256, with biases: the whole workload, mean of {reps} calls"}
    # SGEMM, the naive three-loop product (float accumulator): whole products up to 1024, a row slice at 4096
    for size, rows in ((256, 256), (1024, 1024), (4096, 128)):
        A, B, C0 = si.gemm_operands(1, size, size, size, size, size, size)
        A, B, C0 = A.numpy(), B.numpy(), C0.numpy()
        for ta, tb in (("N", "N"), ("N", "T"), ("T", "N")) if size <= 1024 else (("N", "N"),):
            t0 = time.perf_counter()
            oracle.sgemm(ta, tb, rows, size, size, 1.0, A, size, B, size, 0.5, C0, size)
            dt = time.perf_counter() - t0
            what = "whole product" if rows == size else f"first {rows} rows of C (1/{size // rows} of the product)"
            out[f"sgemm_{ta}{tb}_{size}"] = {"value": round(oracle.sgemm_flops(rows, size, size) / dt / 1e9, 3),
                                            "unit": "GFLOP/s", "seconds": round(dt, 4), "cores": oracle.threads(),
                                            "kind": "oracle", "sample": f"M=N=K={size}, alpha 1, beta 0.5: {what}"}
    # bf16 workload: the float oracle on the inputs rounded to bf16, first 4096 of the 65536 patterns
    rb = lambda t: t.to(torch.bfloat16).float().numpy()
    Xs, ys = si.mlp_patterns(shape, SEED, 0, 4096)
    t0 = time.perf_counter()
    oracle.mlp_grad(rb(W1), rb(W2), rb(Xs), ys.numpy(), dtype=np.float32)
    dt = time.perf_counter() - t0
    out["bf16_inputs"] = {"value": round(oracle.grad_flops(4096, shape.n_in, shape.n_hid, shape.n_out) / dt / 1e9, 3),
                          "unit": "GFLOP/s", "seconds": round(dt, 3), "cores": oracle.threads(), "kind": "oracle",
                          "sample": "400-480-3203 on inputs rounded to bf16: the first 4096 of the 65536 patterns "
                                    "(1/16 of the workload), float arithmetic"}
    return out


def bench_variants(ulsnn, si, torch, shape, W1, W2, X, y, ws):
    """The other entry points on the same network and batch: squared-error gradient (section 4.2), error-only
    evaluation, one conjugate-gradient iteration (gradient + Polak-Ribiere direction + line search), and the
    vector primitives over the 1,729,440 weights."""
    dev, b = X.device, X.shape[0]
    n_i, n_h, n_o = shape.n_in, shape.n_hid, shape.n_out
    out = ulsnn.MlpGradResult(torch.empty_like(W1), torch.empty_like(W2), torch.empty(1, device=dev))

    def per_call(f, reps):
        settle(torch, f, 0.05)
        t0 = time.perf_counter()
        for _ in range(reps):
            f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    res = {}
    T = si.mlp_targets(shape, SEED, 0, b, device=dev)
    sec = per_call(lambda: ulsnn.mlp_grad_mse(W1, W2, X, T, out=out, workspace=ws), 30)
    fl = ulsnn.mlp_grad_flops(n_i, n_h, n_o, b)
    res["mse_grad"] = {"ms": round(sec * 1e3, 4), "gflops": round(fl / sec / 1e9, 1),
                       "frac_of_fp32_mfma_peak": round(fl / sec / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4)}
    del T
    loss = torch.empty(1, device=dev)
    sec = per_call(lambda: ulsnn.mlp_loss(W1, W2, X, y, loss=loss, workspace=ws), 30)
    fl = ulsnn.mlp_loss_flops(n_i, n_h, n_o, b)
    res["loss_only"] = {"ms": round(sec * 1e3, 4), "gflops": round(fl / sec / 1e9, 1),
                        "frac_of_fp32_mfma_peak": round(fl / sec / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4)}

    # one conjugate-gradient iteration from the initial weights, repeated from the same start
    n1 = W1.numel()
    grad = torch.empty(n1 + W2.numel(), device=dev)
    d = torch.empty_like(grad)
    gout = ulsnn.MlpGradResult(grad[:n1].view_as(W1), grad[n1:].view_as(W2), torch.empty(1, device=dev))
    lws = torch.empty(ulsnn.mlp_line_search_workspace_bytes(n_i, n_h, n_o, b), dtype=torch.uint8, device=dev)
    bracket, last = 512, None
    times = []
    for rep in range(4):
        V1, V2 = W1.clone(), W2.clone()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ulsnn.mlp_grad(V1, V2, X, y, out=gout, workspace=ws)
        ulsnn.cg_direction(grad, None, d)
        last = ulsnn.mlp_line_search(V1, V2, d[:n1].view_as(W1), d[n1:].view_as(W2), X, y, bracket, 1e-5, 30,
                                     workspace=lws)
        torch.cuda.synchronize()
        if rep:
            times.append(time.perf_counter() - t0)
    sec = min(times)
    fl = (ulsnn.mlp_grad_flops(n_i, n_h, n_o, b) + last.error_evaluations * ulsnn.mlp_loss_flops(n_i, n_h, n_o, b)
          + last.gradient_evaluations * ulsnn.mlp_grad_flops(n_i, n_h, n_o, bracket))
    res["cg_iteration"] = {"ms": round(sec * 1e3, 3), "gflops": round(fl / sec / 1e9, 1),
                           "error_evaluations": last.error_evaluations,
                           "gradient_evaluations_on_subset": last.gradient_evaluations, "bracket_batch": bracket,
                           "alpha": last.alpha, "loss_before": last.loss0, "loss_after": last.loss,
                           "note": "gradient + direction + line search; the host synchronises once per 8 bracketing "
                                   "steps and once at the end"}
    # vector primitives: HBM/L2-resident 6.9 MB vectors, launch-latency bound
    dot_out = torch.empty(1, device=dev)
    vws = torch.empty(ulsnn.VEC_WORKSPACE_BYTES, dtype=torch.uint8, device=dev)
    sec = per_call(lambda: ulsnn.dot(grad, d, out=dot_out, workspace=vws), 200)
    res["dot"] = {"us": round(sec * 1e6, 2), "GB_per_s": round(2 * grad.numel() * 4 / sec / 1e9, 1)}
    sec = per_call(lambda: ulsnn.axpy(1e-9, grad, d), 200)
    res["axpy"] = {"us": round(sec * 1e6, 2), "GB_per_s": round(3 * grad.numel() * 4 / sec / 1e9, 1)}
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU; --gpus {args.gpus} is not supported "
              f"(the gradient is additive over patterns, so more GPUs would each take a share of the "
              f"patterns and all-reduce 1,729,441 floats; that path is not built)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_1911_05181_amd as ulsnn
    import synth_inputs as si

    ulsnn.load()                       # fails loudly if the HIP library has not been built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    shape = si.MLP_JOCR
    W1c, W2c, _, _ = si.mlp_weights(shape, SEED)
    Xc, yc = si.mlp_patterns(shape, SEED, 0, BATCH)
    W1, W2, X, y = W1c.to(dev), W2c.to(dev), Xc.to(dev), yc.to(dev)
    need = ulsnn.mlp_grad_workspace_bytes(shape.n_in, shape.n_hid, shape.n_out, BATCH)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    out = ulsnn.MlpGradResult(torch.empty_like(W1), torch.empty_like(W2), torch.empty(1, device=dev))
    flops = ulsnn.mlp_grad_flops(shape.n_in, shape.n_hid, shape.n_out, BATCH)

    # what a fresh process gives straight after the W warm-up steps: its first tens of milliseconds under load run
    # at a lower clock
    for _ in range(args.warmup):
        ulsnn.mlp_grad(W1, W2, X, y, out=out, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ulsnn.mlp_grad(W1, W2, X, y, out=out, workspace=ws)
    torch.cuda.synchronize()
    dt_cold = time.perf_counter() - t0

    # untimed: bring clocks and queues to their steady state, then the W warm-up steps
    settle_steps = 0
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle_seconds:
        for _ in range(10):
            ulsnn.mlp_grad(W1, W2, X, y, out=out, workspace=ws)
        torch.cuda.synchronize()
        settle_steps += 10
    for _ in range(args.warmup):
        ulsnn.mlp_grad(W1, W2, X, y, out=out, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ulsnn.mlp_grad(W1, W2, X, y, out=out, workspace=ws)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    gflops = flops * args.steps / dt / 1e9
    loss = out.loss.item()

    # the same call timed one by one with events on the launch stream (each call waits for the one before)
    n_single = max(20, min(args.steps, 50))
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_single)]
    for e0, e1 in evs:
        e0.record()
        ulsnn.mlp_grad(W1, W2, X, y, out=out, workspace=ws)
        e1.record()
    torch.cuda.synchronize()
    singles = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    per_call = {"n": n_single, "median_ms": round(singles[n_single // 2], 4), "min_ms": round(singles[0], 4),
                "max_ms": round(singles[-1], 4)}

    # shader clock while the step runs: a probe wavefront on a second stream reads the cycle counter and the wall
    # clock for 20 ms in the middle of a run of the same steps
    info = ulsnn.device_info()
    probe_out = torch.zeros(2, dtype=torch.int64, device=dev)
    side = torch.cuda.Stream()
    n_probe = max(60, int(0.045 / (ms_per_step * 1e-3)))
    for i in range(n_probe):
        if i == 10:
            ulsnn.clock_probe(20.0, probe_out, stream=side)
        ulsnn.mlp_grad(W1, W2, X, y, out=out, workspace=ws)
    torch.cuda.synchronize()
    cycles, ticks = (int(v) for v in probe_out.tolist())
    sclk_mhz = cycles / ticks * info["wall_clock_khz"] / 1e3 if ticks > 0 else None
    peak_at_clock = info["compute_units"] * FLOP_PER_CLK_PER_CU * sclk_mhz * 1e6 / 1e12 if sclk_mhz else None
    device = {"compute_units": info["compute_units"], "max_shader_clock_mhz": info["max_shader_clock_khz"] / 1e3,
              "shader_clock_mhz_under_load": round(sclk_mhz, 1) if sclk_mhz else None,
              "probe_window_ms": round(ticks / info["wall_clock_khz"], 3) if ticks > 0 else None,
              "fp32_mfma_peak_at_measured_clock_tflops": round(peak_at_clock, 2) if peak_at_clock else None}

    # per-stage durations from HIP events on the launch stream (same kernels, same workspace)
    reps = max(5, min(args.steps, 20))
    acc = {k: 0.0 for k in ulsnn.MLP_STAGES}
    for _ in range(reps):
        _, ms = ulsnn.mlp_grad_timed(W1, W2, X, y, out=out, workspace=ws)
        for k, v in ms.items():
            acc[k] += v / reps
    n_i, n_h, n_o = shape.n_in, shape.n_hid, shape.n_out
    stage_flops = {"hidden_layer": 2.0 * BATCH * n_i * n_h, "output_layer": 2.0 * BATCH * n_h * n_o,
                   "backward_products": 4.0 * BATCH * n_h * n_o, "dW1_product": 2.0 * BATCH * n_i * n_h}
    stages = {k: {"ms": round(v, 4), "tflops": round(stage_flops[k] / (v * 1e-3) / 1e12, 2) if k in stage_flops
                  and v > 0 else None} for k, v in acc.items()}
    dom = max(stage_flops, key=lambda k: acc[k])
    achieved = stage_flops[dom] / (acc[dom] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": f"fp32 MFMA GEMM launch of stage '{dom}'", "achieved": round(achieved, 2),
                "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_MFMA_TFLOPS, 4),
                "frac_at_measured_clock": round(achieved / peak_at_clock, 4) if peak_at_clock else None,
                "traffic": pmc_traffic().get(dom), "traffic_unit": "bytes of HBM per launch (calibrated PMC)",
                "traffic_source": TRAFFIC_PROFILE,
                "flops_per_launch": stage_flops[dom], "avg_launch_ms": round(acc[dom], 4)}

    result = {
        "metric": METRIC, "value": round(gflops, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "settle_steps": settle_steps, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "mlp_grad 400-480-3203 (1,729,440 parameters, no biases), batch 4096, seed 2 "
                               "(BASELINE configs[2]); sgemm sweep = configs[1]",
                   "batch": BATCH, "flops_per_step": flops},
        "patterns_per_s": round(BATCH * args.steps / dt, 1),
        "frac_of_fp32_mfma_peak": round(gflops / (PEAK_FP32_MFMA_TFLOPS * 1e3), 4),
        "frac_at_measured_clock": round(gflops / 1e3 / peak_at_clock, 4) if peak_at_clock else None,
        "unsettled": {"ms_per_step": round(dt_cold / args.steps * 1e3, 4),
                      "gflops": round(flops * args.steps / dt_cold / 1e9, 1),
                      "frac_of_fp32_mfma_peak": round(flops * args.steps / dt_cold / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4),
                      "note": "the same K steps timed straight after the W warm-up steps of the fresh process"},
        "per_call_events": per_call,
        "device": device,
        "loss": loss, "stages": stages, "roofline": roofline,
    }
    def time_batch(W1_, W2_, X_, y_, reps):
        b = X_.shape[0]
        odt = 1 if W1_.dtype == torch.bfloat16 else 0
        ws_ = torch.empty(ulsnn.mlp_grad_workspace_bytes(shape.n_in, shape.n_hid, shape.n_out, b, odt),
                          dtype=torch.uint8, device=dev)
        out_ = ulsnn.MlpGradResult(torch.empty(W1_.shape, device=dev), torch.empty(W2_.shape, device=dev),
                                   torch.empty(1, device=dev))
        settle(torch, lambda: ulsnn.mlp_grad(W1_, W2_, X_, y_, out=out_, workspace=ws_), 0.1)
        t1 = time.perf_counter()
        for _ in range(reps):
            ulsnn.mlp_grad(W1_, W2_, X_, y_, out=out_, workspace=ws_)
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t1) / reps
        fl = ulsnn.mlp_grad_flops(shape.n_in, shape.n_hid, shape.n_out, b)
        return {"batch": b, "ms": round(sec * 1e3, 4), "gflops": round(fl / sec / 1e9, 1),
                "patterns_per_s": round(b / sec, 1)}

    if not args.no_large_batch:
        # one chunk of the epoch workload (BASELINE configs[3]): 262144 patterns resident in HBM, fp32
        Xl, yl = si.mlp_patterns(shape, SEED, 0, 262144, device=dev)
        r = time_batch(W1, W2, Xl, yl, 3)
        r["frac_of_fp32_mfma_peak"] = round(r["gflops"] / (PEAK_FP32_MFMA_TFLOPS * 1e3), 4)
        r["workload"] = "same net, fp32, one 262144-pattern chunk of the 9,000,000-pattern epoch"
        result["large_batch"] = r
        del Xl, yl
    if not args.no_small_net:
        # the small case (BASELINE configs[0]): 64-32-10 with biases, batch 256 -- launch-latency bound
        sm = si.MLP_SMALL
        sW1, sW2, sb1, sb2 = (t.to(dev) for t in si.mlp_weights(sm, 0))
        sX, sy = si.mlp_patterns(sm, 0, 0, 256, device=dev)
        sws = torch.empty(ulsnn.mlp_grad_workspace_bytes(sm.n_in, sm.n_hid, sm.n_out, 256), dtype=torch.uint8, device=dev)
        sout = ulsnn.MlpGradResult(torch.empty_like(sW1), torch.empty_like(sW2), torch.empty(1, device=dev),
                                   torch.empty_like(sb1), torch.empty_like(sb2))
        settle(torch, lambda: ulsnn.mlp_grad(sW1, sW2, sX, sy, sb1, sb2, out=sout, workspace=sws), 0.05)
        t1 = time.perf_counter()
        for _ in range(200):
            ulsnn.mlp_grad(sW1, sW2, sX, sy, sb1, sb2, out=sout, workspace=sws)
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t1) / 200
        result["small_net"] = {"workload": "64-32-10 with biases, batch 256 (small-network path: two launches; latency bound)",
                               "us_per_call": round(sec * 1e6, 2), "patterns_per_s": round(256 / sec, 1),
                               "gflops": round(ulsnn.mlp_grad_flops(sm.n_in, sm.n_hid, sm.n_out, 256) / sec / 1e9, 2)}
    if not args.no_variants:
        result["variants"] = bench_variants(ulsnn, si, torch, shape, W1, W2, X, y, ws)
    if not args.no_epoch:
        # the epoch workload (BASELINE configs[3]): 9,000,000 patterns resident in HBM, chunks of 262144 summed
        n_ep, chunk = 9_000_000, 262144
        Xe = torch.empty(n_ep, shape.n_in, device=dev)
        ye = torch.empty(n_ep, dtype=torch.int32, device=dev)
        for p0 in range(0, n_ep, chunk):
            rows = min(chunk, n_ep - p0)
            Xe[p0:p0 + rows], ye[p0:p0 + rows] = si.mlp_patterns(shape, SEED, p0, rows, device=dev)
        wse = torch.empty(ulsnn.mlp_grad_workspace_bytes(shape.n_in, shape.n_hid, shape.n_out, chunk),
                          dtype=torch.uint8, device=dev)
        ulsnn.mlp_grad_epoch(W1, W2, Xe[:2 * chunk], ye[:2 * chunk], chunk, out=out, workspace=wse)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ulsnn.mlp_grad_epoch(W1, W2, Xe, ye, chunk, out=out, workspace=wse)
        torch.cuda.synchronize()
        sec = time.perf_counter() - t1
        fl = ulsnn.mlp_grad_flops(shape.n_in, shape.n_hid, shape.n_out, n_ep)
        result["epoch"] = {"workload": "same net, fp32, 9,000,000 patterns resident in HBM (14.4 GB), 34 chunks of "
                                       "262144 + one of 87104, gradients and loss summed",
                           "patterns": n_ep, "seconds": round(sec, 4), "gflops": round(fl / sec / 1e9, 1),
                           "patterns_per_s": round(n_ep / sec, 1),
                           "frac_of_fp32_mfma_peak": round(fl / sec / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4),
                           "loss_per_pattern": round(out.loss.item() / n_ep, 6)}
        del Xe, ye, wse
    if not args.no_bf16:
        # bf16-operand workload (BASELINE configs[4]): X, W stored bf16, batch 65536, fp32 accumulation
        Xb, yb = si.mlp_patterns(shape, SEED, 0, 65536, device=dev)
        r = time_batch(W1.to(torch.bfloat16), W2.to(torch.bfloat16), Xb.to(torch.bfloat16), yb, 5)
        r["x_of_fp32_mfma_peak"] = round(r["gflops"] / (PEAK_FP32_MFMA_TFLOPS * 1e3), 3)
        r["frac_of_bf16_mfma_peak"] = round(r["gflops"] / 2.5e6, 4)
        r["workload"] = "same net, X/W/H/dO/dA1 in bf16, fp32 accumulate, batch 65536"
        # HBM side of this workload: every tensor the step cannot avoid moving, once each way as listed
        n_i, n_h, n_o = shape.n_in, shape.n_hid, shape.n_out
        alg = 65536 * (n_i + 4 * n_h + 3 * n_o) * 2 + 3 * 2 * (n_i * n_h + n_h * n_o) + 4 * (n_i * n_h + n_h * n_o)
        gbs = alg / (r["ms"] * 1e-3) / 1e9
        r["roofline_hbm"] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": round(gbs / PEAK_HBM_GBS, 4), "algorithmic_bytes": alg,
                             "algorithmic_bytes_note": "X read; H and dA1 written once and read once, logits written once and "
                                                       "read twice (bf16; the delta is never stored); bf16 weights read by "
                                                       "three products; fp32 gradients written",
                             "traffic": pmc_traffic(TRAFFIC_PROFILE_BF16).get("bf16_gradient"),
                             "traffic_unit": "bytes of HBM per gradient (calibrated PMC, all kernels)",
                             "traffic_source": TRAFFIC_PROFILE_BF16}
        result["bf16"] = r
        # the squared-error form on the same operands (dense fp32 targets, 840 MB)
        Wb1, Wb2, Xbb = W1.to(torch.bfloat16), W2.to(torch.bfloat16), Xb.to(torch.bfloat16)
        Tb = si.mlp_targets(shape, SEED, 0, 65536, device=dev)
        wsb = torch.empty(ulsnn.mlp_grad_workspace_bytes(shape.n_in, shape.n_hid, shape.n_out, 65536, 1),
                          dtype=torch.uint8, device=dev)
        settle(torch, lambda: ulsnn.mlp_grad_mse(Wb1, Wb2, Xbb, Tb, out=out, workspace=wsb), 0.1)
        t1 = time.perf_counter()
        for _ in range(5):
            ulsnn.mlp_grad_mse(Wb1, Wb2, Xbb, Tb, out=out, workspace=wsb)
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t1) / 5
        result["bf16"]["mse_grad"] = {"ms": round(sec * 1e3, 4),
                                      "gflops": round(ulsnn.mlp_grad_flops(shape.n_in, shape.n_hid, shape.n_out, 65536) / sec / 1e9, 1)}
        del Xb, yb, Tb, wsb, Xbb
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                 # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    if not args.no_sgemm:
        result["sgemm"] = bench_sgemm(ulsnn, si, torch, args.sgemm_sizes)
        result["sgemm"].update(bench_sgemm_strided_and_cold(ulsnn, si, torch, args.sgemm_sizes))
    if not args.no_cpu:
        cb = cpu_baseline(si, shape, W1c, W2c, Xc, yc)
        cb["gpu_speedup"] = round(gflops / cb["value"], 1)
        result["cpu_baseline"] = cb
        others = cpu_baselines_other(si, torch, shape, W1c, W2c)
        # the epoch workload: the 4096-pattern slice above, scaled by the pattern count
        others["epoch"] = {"value": cb["value"], "unit": "GFLOP/s", "cores": cb["cores"], "kind": "oracle",
                           "seconds_scaled": round(9_000_000 / cb["patterns_per_s"], 1),
                           "sample": "the 4096-pattern slice of cpu_baseline, time scaled by 9,000,000 / 4096"}
        if "epoch" in result:
            others["epoch"]["gpu_speedup"] = round(others["epoch"]["seconds_scaled"] / result["epoch"]["seconds"], 1)
        if "small_net" in result:
            others["small_net"]["gpu_speedup"] = round(others["small_net"]["us_per_call"] / result["small_net"]["us_per_call"], 1)
        if "bf16" in result:
            others["bf16_inputs"]["gpu_speedup"] = round(result["bf16"]["gflops"] / others["bf16_inputs"]["value"], 1)
        for key, v in others.items():
            if key.startswith("sgemm_") and "sgemm" in result:
                g = result["sgemm"].get(key[len("sgemm_"):])
                if g:
                    v["gpu_speedup"] = round(g["gflops"] / v["value"], 1)
        result["cpu_baselines"] = others
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
