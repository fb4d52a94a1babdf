"""Parity of ulsnn_sgemm (HIP, through the C ABI) against the CPU oracle.

Bars (the fp32 GEMM bound of the benchmark spec):
  * integer-valued inputs whose partial sums stay below 2^24: BIT-EXACT against the oracle;
  * uniform[-1,1] inputs: |C_gpu - C_ref| <= 1e-4 * |alpha| * S_ij + 1e-6 * |beta * C0_ij|, where C_ref is the
    double-accumulator oracle and S_ij = sum_p |a_ip||b_pj|.  The observed max of |err| / S is printed; fp32
    accumulation gives about 1e-7..1e-6, so the bound has two orders of margin and a regression shows early.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_1911_05181_amd as ulsnn
import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _stored_dims(ta, tb, m, n, k):
    return ((m, k) if ta == "N" else (k, m)), ((k, n) if tb == "N" else (n, k))


def _padded(M, ld, fill=np.nan):
    S = np.full((M.shape[0], ld), fill, dtype=np.float32)
    S[:, :M.shape[1]] = M
    return S


def _run(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C0, ldc):
    dA, dB, dC = (torch.from_numpy(x).to(DEV) for x in (A, B, C0))
    ulsnn.sgemm(ta, tb, m, n, k, alpha, dA, lda, dB, ldb, beta, dC, ldc)
    torch.cuda.synchronize()
    return dC.cpu().numpy()


INT_SHAPES = [(1, 1, 1), (3, 5, 7), (33, 31, 9), (130, 70, 33), (257, 129, 100), (64, 48, 130), (128, 128, 16),
              (200, 300, 17),
              # edges narrower than one 16-byte load, in a later tile (67 = 64 + 3) and in the only tile (3, 2)
              (100, 67, 48), (67, 100, 48), (40, 3, 40), (2, 50, 64), (131, 134, 96)]


@pytest.mark.parametrize("ta,tb", list(itertools.product("NT", "NT")))
@pytest.mark.parametrize("m,n,k", INT_SHAPES)
def test_small_integers_bit_exact(ta, tb, m, n, k):
    (ra, ca), (rb, cb) = _stored_dims(ta, tb, m, n, k)
    pad = 3                                                    # odd leading dimensions: 4-byte aligned rows only
    A = _padded(si.small_integers(31, si.T_A, ra, ca).numpy(), ca + pad)
    B = _padded(si.small_integers(31, si.T_B, rb, cb).numpy(), cb + pad)
    for alpha, beta in [(1.0, 0.0), (-1.0, 1.0), (2.0, 0.5), (0.5, -2.0)]:
        A2 = A * 2 if alpha == 0.5 else A
        C0 = _padded(si.small_integers(31, si.T_C, m, n, even=True).numpy(), n + pad)
        want = oracle.sgemm(ta, tb, m, n, k, alpha, A2, ca + pad, B, cb + pad, beta, C0, n + pad)
        got = _run(ta, tb, m, n, k, alpha, A2, ca + pad, B, cb + pad, beta, C0, n + pad)
        assert np.array_equal(got[:, :n], want[:, :n]), (ta, tb, m, n, k, alpha, beta)
        assert np.isnan(got[:, n:]).all()                      # padding columns of C are not written


def _check_bound(got, ref, S, alpha, beta, C0):
    err = np.abs(got.astype(np.float64) - ref)
    bound = 1e-4 * abs(alpha) * S + 1e-6 * np.abs(beta * C0.astype(np.float64))
    ratio = float((err / np.maximum(S, 1e-30)).max())
    assert (err <= bound).all(), f"max err/S = {ratio:.3e}"
    return ratio


@pytest.mark.parametrize("ta,tb", [("N", "N"), ("N", "T"), ("T", "N"), ("T", "T")])
@pytest.mark.parametrize("size,extra_ld", [(256, 0), (1024, 0), (300, 8), (515, 1)])
def test_uniform_full_parity(ta, tb, size, extra_ld):
    m = n = k = size
    (ra, ca), (rb, cb) = _stored_dims(ta, tb, m, n, k)
    A, B, C0 = si.gemm_operands(1, ra, ca, rb, cb, m, n, lda=ca + extra_ld, ldb=cb + extra_ld, ldc=n + extra_ld)
    A, B, C0 = A.numpy(), B.numpy(), C0.numpy()
    alpha, beta = 1.0, 0.5
    got = _run(ta, tb, m, n, k, alpha, A, ca + extra_ld, B, cb + extra_ld, beta, C0, n + extra_ld)
    ref, S = oracle.sgemm_exact(ta, tb, m, n, k, alpha, A, ca + extra_ld, B, cb + extra_ld, beta, C0, n + extra_ld)
    ratio = _check_bound(got[:, :n], ref, S, alpha, beta, C0[:, :n])
    assert np.array_equal(got[:, n:], C0[:, n:])
    print(f"sgemm {ta}{tb} {size} ld+{extra_ld}: max |err|/S = {ratio:.3e}")
    assert ratio < 5e-6                                         # what fp32 accumulation should achieve


@pytest.mark.parametrize("ta,tb", [("N", "N"), ("N", "T"), ("T", "N")])
@pytest.mark.parametrize("size,samples", [(4096, 24), (8192, 12)])
def test_uniform_large_sampled(ta, tb, size, samples):
    """Full benchmark sizes: whole rows and whole columns of C, chosen at random, against the oracle."""
    m = n = k = size
    (ra, ca), (rb, cb) = _stored_dims(ta, tb, m, n, k)
    A, B, C0 = si.gemm_operands(1, ra, ca, rb, cb, m, n, device=DEV)
    alpha, beta = 1.0, 0.5
    dC = C0.clone()
    ulsnn.sgemm(ta, tb, m, n, k, alpha, A, ca, B, cb, beta, dC, n)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    A, B, C0 = A.cpu().numpy(), B.cpu().numpy(), C0.cpu().numpy()
    rng = np.random.default_rng(size)
    worst = 0.0
    for i in rng.choice(m, samples, replace=False):            # row i of C needs row i of op(A)
        Ai = np.ascontiguousarray(A[i:i + 1, :] if ta == "N" else A[:, i:i + 1])
        lda_i = ca if ta == "N" else 1
        ref, S = oracle.sgemm_exact(ta, tb, 1, n, k, alpha, Ai, lda_i, B, cb, beta, C0[i:i + 1], n)
        worst = max(worst, _check_bound(got[i:i + 1], ref, S, alpha, beta, C0[i:i + 1]))
    for j in rng.choice(n, samples, replace=False):            # column j of C needs column j of op(B)
        Bj = np.ascontiguousarray(B[:, j:j + 1] if tb == "N" else B[j:j + 1, :])
        ldb_j = 1 if tb == "N" else cb
        Cj = np.ascontiguousarray(C0[:, j:j + 1])
        ref, S = oracle.sgemm_exact(ta, tb, m, 1, k, alpha, A, ca, Bj, ldb_j, beta, Cj, 1)
        worst = max(worst, _check_bound(got[:, j:j + 1], ref, S, alpha, beta, Cj))
    print(f"sgemm {ta}{tb} {size}: sampled max |err|/S = {worst:.3e}")
    assert worst < 2e-5


def test_blas_rules_on_device():
    m, n, k = 70, 90, 50
    A, B, C0 = si.gemm_operands(9, m, k, k, n, m, n)
    A, B, C0 = A.numpy(), B.numpy(), C0.numpy()
    nan = np.full((m, n), np.nan, np.float32)
    got = _run("N", "N", m, n, k, 1.0, A, k, B, n, 0.0, nan, n)                 # beta = 0: C is not read
    assert np.isfinite(got).all()
    assert np.array_equal(_run("N", "N", m, n, 0, 1.0, A, k, B, n, 0.5, C0, n), np.float32(0.5) * C0)
    assert np.array_equal(_run("N", "N", m, n, k, 0.0, A, k, B, n, -2.0, C0, n), np.float32(-2.0) * C0)
    assert np.array_equal(_run("N", "N", m, n, k, 0.0, A, k, B, n, 0.0, nan, n), np.zeros_like(C0))
    assert np.array_equal(_run("N", "N", m, n, k, 0.0, A, k, B, n, 1.0, C0, n), C0)
    assert np.array_equal(_run("N", "N", 0, n, k, 1.0, A, k, B, n, 0.5, C0, n), C0)   # m = 0: untouched
    with pytest.raises(ulsnn.UlsnnError):
        _run("N", "N", m, n, k, 1.0, A, k - 1, B, n, 0.0, C0, n)


def test_runs_are_bit_reproducible():
    m, n, k = 777, 513, 1029
    A, B, C0 = si.gemm_operands(5, k, m, n, k, m, n)            # T, T
    A, B, C0 = A.numpy(), B.numpy(), C0.numpy()
    a = _run("T", "T", m, n, k, 1.0, A, m, B, k, 0.5, C0, n)
    b = _run("T", "T", m, n, k, 1.0, A, m, B, k, 0.5, C0, n)
    assert np.array_equal(a, b)


def test_runs_on_a_side_stream():
    m = n = k = 256
    A, B, C0 = si.gemm_operands(6, m, k, k, n, m, n, device=DEV)
    want = C0.clone()
    ulsnn.sgemm("N", "N", m, n, k, 1.0, A, k, B, n, 0.5, want, n)
    s = torch.cuda.Stream()
    got = C0.clone()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        ulsnn.sgemm("N", "N", m, n, k, 1.0, A, k, B, n, 0.5, got, n)
    s.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(got, want)


# every tile shape x every layout on shapes whose edges are not multiples of 4 (and of the tile), with and
# without k splits: integer matrices, so any blocking must reproduce the oracle bit for bit
EDGE_SHAPES = [(131, 135, 96), (259, 67, 64), (70, 259, 48), (300, 3, 80), (2, 133, 64), (257, 130, 40)]


@pytest.mark.parametrize("tile", range(len(ulsnn.TILE_SHAPES)), ids=ulsnn.TILE_SHAPES)
@pytest.mark.parametrize("ta,tb", list(itertools.product("NT", "NT")))
def test_every_tile_shape_on_ragged_edges(tile, ta, tb):
    for (m, n, k) in EDGE_SHAPES:
        (ra, ca), (rb, cb) = _stored_dims(ta, tb, m, n, k)
        pad = 1
        A = _padded(si.small_integers(41, si.T_A, ra, ca).numpy(), ca + pad)
        B = _padded(si.small_integers(41, si.T_B, rb, cb).numpy(), cb + pad)
        C0 = _padded(si.small_integers(41, si.T_C, m, n, even=True).numpy(), n + pad)
        want = oracle.sgemm(ta, tb, m, n, k, 1.0, A, ca + pad, B, cb + pad, 0.5, C0, n + pad)
        for splits in (1, 3):
            dA, dB, dC = (torch.from_numpy(x).to(DEV) for x in (A, B, C0))
            ulsnn.sgemm_planned(tile, splits, ta, tb, m, n, k, 1.0, dA, ca + pad, dB, cb + pad, 0.5, dC, n + pad)
            torch.cuda.synchronize()
            got = dC.cpu().numpy()
            assert np.array_equal(got[:, :n], want[:, :n]), (ulsnn.TILE_SHAPES[tile], ta, tb, m, n, k, splits)
            assert np.isnan(got[:, n:]).all()


@pytest.mark.parametrize("ta,tb,m,n,k", [("N", "N", 256, 256, 4096), ("T", "N", 400, 480, 3000), ("N", "T", 130, 70, 5001),
                                          ("T", "T", 64, 48, 2048), ("N", "N", 1024, 1024, 1024)])
def test_sgemm_with_workspace_splits_k_deterministically(ta, tb, m, n, k):
    """ulsnn_sgemm_ws: the planner may cut k into slices when the workspace allows it (few tiles of C, long k).
    Integer inputs (partial sums below 2^24): bit-exact against the oracle whatever the split; uniform inputs
    inside the bound; the same call twice gives the same bits; without room for two slices it is ulsnn_sgemm."""
    (ra, ca), (rb, cb) = _stored_dims(ta, tb, m, n, k)
    ws = torch.empty(16 * m * n * 4, dtype=torch.uint8, device=DEV)
    plan = ulsnn.sgemm_ws_describe_plan(ta, tb, m, n, k, ws.numel())
    splits = int(plan.split("splits=")[1].split()[0])
    assert (splits > 1) == (k > 1024), plan      # the long-k cases really take the split path, 1024^3 does not
    A = si.small_integers(7, si.T_A, ra, ca, bound=4).numpy()
    B = si.small_integers(7, si.T_B, rb, cb, bound=4).numpy()
    C0 = si.small_integers(7, si.T_C, m, n, even=True).numpy()
    want = oracle.sgemm(ta, tb, m, n, k, 1.0, A, ca, B, cb, 0.5, C0, n)
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    dC = torch.from_numpy(C0).to(DEV)
    ulsnn.sgemm_ws(ta, tb, m, n, k, 1.0, dA, ca, dB, cb, 0.5, dC, n, ws)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), want)
    Au, Bu, Cu = si.gemm_operands(1, ra, ca, rb, cb, m, n)
    ref, S = oracle.sgemm_exact(ta, tb, m, n, k, 1.0, Au.numpy(), ca, Bu.numpy(), cb, 0.5, Cu.numpy(), n)
    runs = []
    for workspace in (ws, ws, None):
        dC = Cu.to(DEV)
        ulsnn.sgemm_ws(ta, tb, m, n, k, 1.0, Au.to(DEV), ca, Bu.to(DEV), cb, 0.5, dC, n, workspace)
        torch.cuda.synchronize()
        runs.append(dC.cpu().numpy())
        ratio = _check_bound(runs[-1], ref, S, 1.0, 0.5, Cu.numpy())
        assert ratio < 5e-6
    assert np.array_equal(runs[0], runs[1])
    plain = Cu.to(DEV)
    ulsnn.sgemm(ta, tb, m, n, k, 1.0, Au.to(DEV), ca, Bu.to(DEV), cb, 0.5, plain, n)
    torch.cuda.synchronize()
    assert np.array_equal(runs[2], plain.cpu().numpy())
