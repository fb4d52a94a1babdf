"""The counting formulas against the figures the paper prints (tests/golden/paper_counts.txt)."""
import os

import oracle


def _golden(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "paper_counts.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split()
                vals[k] = float(v)
    return vals


def test_parameter_counts(golden_dir):
    g = _golden(golden_dir)
    assert oracle.param_count(100, 50, 50) == g["params_100_50_50"]
    assert oracle.param_count(100, 50, 50) * 4 == g["bytes_100_50_50"]
    assert oracle.param_count(400, 480, 3203) == g["params_400_480_3203"]
    # "6.6 MBytes": 1,729,440 floats = 6.597 MiB
    assert round(oracle.param_count(400, 480, 3203) * 4 / 2**20, 1) == g["mbytes_400_480_3203"]


def test_flop_counts(golden_dir):
    g = _golden(golden_dir)
    n_p = int(g["patterns_epoch"])
    e = oracle.error_flops(n_p, 400, 480, 3203)
    gr = oracle.grad_flops(n_p, 400, 480, 3203)
    assert round(e / 1e12) == g["error_tflops_epoch"]
    # the paper prints 92; the formula gives 92.57e12, so the paper truncated rather than rounded
    assert int(gr / 1e12) == g["grad_tflops_epoch"]
    assert round(0.8 * e / 1e12) == g["error_tflops_80pct"]
    assert round(0.8 * gr / 1e12) == g["grad_tflops_80pct"]
    procs = g["slave_processors"]
    # the per-processor figures are the rounded 26 and 74 TFlops divided by 193
    assert round(g["error_tflops_80pct"] * 1e3 / procs) == g["error_gflops_per_proc_80pct"]
    assert round(g["grad_tflops_80pct"] * 1e3 / procs) == g["grad_gflops_per_proc_80pct"]
    # and the unrounded formula agrees to within that rounding
    assert abs(0.8 * gr / procs / 1e9 - g["grad_gflops_per_proc_80pct"]) < 2.0
    assert abs(0.8 * e / procs / 1e9 - g["error_gflops_per_proc_80pct"]) < 2.5


def test_per_pattern_flops_and_sgemm():
    assert oracle.grad_flops(1, 400, 480, 3203) == 9_992_640
    assert oracle.sgemm_flops(320, 320, 320) == 2 * 320**3
    # a gradient is the five GEMMs of section 4.2: two of size n_i*n_h... (2 each) and three with n_h*n_o
    n_i, n_h, n_o, b = 400, 480, 3203, 7
    five = (oracle.sgemm_flops(b, n_h, n_i) + oracle.sgemm_flops(b, n_o, n_h) + oracle.sgemm_flops(n_h, n_o, b)
            + oracle.sgemm_flops(b, n_h, n_o) + oracle.sgemm_flops(n_i, n_h, b))
    assert five == oracle.grad_flops(b, n_i, n_h, n_o)

