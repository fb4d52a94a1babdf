"""Pins for the CPU SGEMM oracle: things the mathematics fixes, none of them the oracle's own formula.

  * exact integer products against numpy's int64 matmul (every trans combination, ld > cols, alpha, beta)
  * closed forms: identity, all-ones, diagonal scaling, (AB)^T = B^T A^T
  * BLAS rules: beta == 0 never reads C; k == 0 and alpha == 0 give beta*C; padding is never touched
  * the double-accumulator form against numpy's float64 matmul; the float form inside the rounding bound
"""
import itertools

import numpy as np
import pytest

import oracle
import synth_inputs as si


def _stored(rows, cols, ld, seed, tid, bound=8, even=False):
    """rows x ld integer-valued storage whose padding columns are NaN (must never be read)."""
    M = si.small_integers(seed, tid, rows, cols, bound, even).numpy()
    S = np.full((rows, ld), np.nan, dtype=np.float32)
    S[:, :cols] = M
    return S, M.astype(np.int64)


SHAPES = [(1, 1, 1), (1, 9, 1), (3, 5, 7), (7, 3, 5), (17, 33, 65), (64, 48, 130)]


@pytest.mark.parametrize("ta,tb", list(itertools.product("NT", "NT")))
@pytest.mark.parametrize("m,n,k", SHAPES)
def test_small_integers_exact(ta, tb, m, n, k):
    pad = 3
    ra, ca = (m, k) if ta == "N" else (k, m)
    rb, cb = (k, n) if tb == "N" else (n, k)
    A, Ai = _stored(ra, ca, ca + pad, 11, si.T_A)
    B, Bi = _stored(rb, cb, cb + pad, 11, si.T_B)
    opA = Ai if ta == "N" else Ai.T
    opB = Bi if tb == "N" else Bi.T
    prod = opA @ opB                                  # exact in int64
    for alpha, beta in [(1.0, 0.0), (-1.0, 1.0), (2.0, 0.5), (0.5, -2.0)]:
        # even C entries keep beta*C integral; A, B even when alpha = 0.5 keeps alpha*sum integral
        if alpha == 0.5:
            A2, B2, prod2 = A * 2, B, prod * 2
        else:
            A2, B2, prod2 = A, B, prod
        Cst, Ci = _stored(m, n, n + pad, 11, si.T_C, even=True)
        want = alpha * prod2 + (0 if beta == 0 else beta * Ci)
        got = oracle.sgemm(ta, tb, m, n, k, alpha, A2, ca + pad, B2, cb + pad, beta, Cst, n + pad)
        assert np.array_equal(got[:, :n].astype(np.float64), want.astype(np.float64))
        assert np.isnan(got[:, n:]).all()                 # padding of C untouched
        ref, S = oracle.sgemm_exact(ta, tb, m, n, k, alpha, A2, ca + pad, B2, cb + pad, beta, Cst, n + pad)
        assert np.array_equal(ref, want.astype(np.float64))
        assert np.array_equal(S, (np.abs(opA) @ np.abs(opB) * (2 if alpha == 0.5 else 1)).astype(np.float64))


def test_identity_ones_diagonal():
    n = 23
    _, B, C0 = si.gemm_operands(5, n, n, n, 31, n, 31)
    B, C0 = B.numpy(), C0.numpy()
    I = np.eye(n, dtype=np.float32)
    # A = I:  C = alpha*B + beta*C, and each product has a single non-zero term, so it is exact up to one rounding
    got = oracle.sgemm("N", "N", n, 31, n, 1.0, I, n, B, 31, 0.0, C0, 31)
    assert np.array_equal(got, B)
    got = oracle.sgemm("T", "N", n, 31, n, 2.0, I, n, B, 31, 1.0, C0, 31)
    assert np.array_equal(got, 2.0 * B + C0)
    # B = ones: every column of C is the row sum of A
    A = si.small_integers(6, si.T_A, 9, 40).numpy()
    ones = np.ones((40, 4), dtype=np.float32)
    got = oracle.sgemm("N", "N", 9, 4, 40, 1.0, A, 40, ones, 4, 0.0, np.zeros((9, 4), np.float32), 4)
    assert np.array_equal(got, np.repeat(A.sum(axis=1, keepdims=True), 4, axis=1))
    # A = diag(d): rows of B scaled
    d = np.arange(1, n + 1, dtype=np.float32)
    got = oracle.sgemm("N", "N", n, 31, n, 1.0, np.diag(d), n, B, 31, 0.0, C0, 31)
    assert np.array_equal(got, d[:, None] * B)


def test_transpose_identity():
    """(op(A) op(B))^T = op(B)^T op(A)^T ties the four index paths to each other; in double every
    product is exact and both sides add the same terms in the same order, so equality is bitwise."""
    m, n, k = 13, 29, 37
    A, B, _ = si.gemm_operands(7, m, k, k, n, m, n)
    A, B = A.numpy(), B.numpy()
    Z = np.zeros((m, n), np.float32)
    ZT = np.zeros((n, m), np.float32)
    nn, _ = oracle.sgemm_exact("N", "N", m, n, k, 1.0, A, k, B, n, 0.0, Z, n)
    At, Bt = np.ascontiguousarray(A.T), np.ascontiguousarray(B.T)
    tt, _ = oracle.sgemm_exact("T", "T", m, n, k, 1.0, At, m, Bt, k, 0.0, Z, n)
    nt, _ = oracle.sgemm_exact("N", "T", m, n, k, 1.0, A, k, Bt, k, 0.0, Z, n)
    tn, _ = oracle.sgemm_exact("T", "N", m, n, k, 1.0, At, m, B, n, 0.0, Z, n)
    sw, _ = oracle.sgemm_exact("T", "T", n, m, k, 1.0, B, n, A, k, 0.0, ZT, m)     # = B^T A^T = (AB)^T
    assert np.array_equal(nn, tt) and np.array_equal(nn, nt) and np.array_equal(nn, tn)
    assert np.array_equal(nn, sw.T)


def test_blas_rules():
    m, n, k = 6, 10, 12
    A, B, C0 = si.gemm_operands(9, m, k, k, n, m, n)
    A, B, C0 = A.numpy(), B.numpy(), C0.numpy()
    nan = np.full((m, n), np.nan, np.float32)
    got = oracle.sgemm("N", "N", m, n, k, 1.0, A, k, B, n, 0.0, nan, n)          # beta = 0: C not read
    assert np.isfinite(got).all()
    ref, _ = oracle.sgemm_exact("N", "N", m, n, k, 1.0, A, k, B, n, 0.0, nan, n)
    assert np.isfinite(ref).all()
    got = oracle.sgemm("N", "N", m, n, 0, 1.0, A, k, B, n, 0.5, C0, n)           # k = 0: C = beta*C
    assert np.array_equal(got, np.float32(0.5) * C0)
    got = oracle.sgemm("N", "N", m, n, k, 0.0, A, k, B, n, -2.0, C0, n)          # alpha = 0: C = beta*C
    assert np.array_equal(got, np.float32(-2.0) * C0)
    got = oracle.sgemm("N", "N", 0, n, k, 1.0, A, k, B, n, 0.5, C0, n)           # m = 0: nothing touched
    assert np.array_equal(got, C0)
    for bad in [dict(ta="X"), dict(m=-1), dict(lda=k - 1), dict(ldb=n - 1), dict(ldc=n - 1)]:
        a = dict(ta="N", tb="N", m=m, n=n, k=k, lda=k, ldb=n, ldc=n)
        a.update(bad)
        with pytest.raises(ValueError):
            oracle.sgemm(a["ta"], a["tb"], a["m"], a["n"], a["k"], 1.0, A, a["lda"], B, a["ldb"], 0.0, C0, a["ldc"])


@pytest.mark.parametrize("ta,tb", list(itertools.product("NT", "NT")))
def test_against_float64_matmul_and_rounding_bound(ta, tb):
    m, n, k = 70, 45, 300
    ra, ca = (m, k) if ta == "N" else (k, m)
    rb, cb = (k, n) if tb == "N" else (n, k)
    A, B, C0 = si.gemm_operands(3, ra, ca, rb, cb, m, n, lda=ca + 5, ldb=cb + 1, ldc=n + 2)
    A, B, C0 = A.numpy(), B.numpy(), C0.numpy()
    opA = (A[:, :ca] if ta == "N" else A[:, :ca].T).astype(np.float64)
    opB = (B[:, :cb] if tb == "N" else B[:, :cb].T).astype(np.float64)
    alpha, beta = 1.0, 0.5
    want = alpha * (opA @ opB) + beta * C0[:, :n].astype(np.float64)
    ref, S = oracle.sgemm_exact(ta, tb, m, n, k, alpha, A, ca + 5, B, cb + 1, beta, C0, n + 2)
    assert np.abs(ref - want).max() <= 1e-13 * S.max()            # two double summations of exact products
    assert np.allclose(S, np.abs(opA) @ np.abs(opB), rtol=1e-13)
    got = oracle.sgemm(ta, tb, m, n, k, alpha, A, ca + 5, B, cb + 1, beta, C0, n + 2)[:, :n]
    eps = 2.0**-24
    # standard bound for a float dot product summed in order: (k+2) eps sum|a||b| (+ the beta*C rounding)
    assert (np.abs(got - ref) <= (k + 2) * eps * S + 2 * eps * np.abs(want)).all()
    # and it is not vacuous: float and double accumulation really differ
    assert np.abs(got - ref).max() > 0
