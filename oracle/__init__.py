"""Python face of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may import this package.
The product (`paper_1911_05181_amd`) never does, and this package never imports the product.

The arithmetic lives in plain C next to this file (ref_sgemm.c, ref_mlp.c + ref_mlp_body.inc); the functions
here only marshal numpy arrays.  The counting formulas at the bottom restate the paper's flop and parameter
counts (sections 3.1, 5.1 and 6.2).
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build())
        fp, dp, ip = C.POINTER(C.c_float), C.POINTER(C.c_double), C.POINTER(C.c_int)
        L.ref_sgemm.argtypes = [C.c_char, C.c_char, C.c_int, C.c_int, C.c_int, C.c_float, fp, C.c_int, fp,
                                C.c_int, C.c_float, fp, C.c_int]
        L.ref_sgemm_exact.argtypes = [C.c_char, C.c_char, C.c_int, C.c_int, C.c_int, C.c_float, fp, C.c_int, fp,
                                      C.c_int, C.c_float, fp, C.c_int, dp, dp]
        for name, rp in (("f64", dp), ("f32", fp)):
            g = getattr(L, "ref_mlp_grad_" + name)
            g.argtypes = [C.c_int] * 4 + [rp] * 5 + [ip] + [rp] * 4 + [dp] + [rp] * 4
            g.restype = C.c_int
            f = getattr(L, "ref_mlp_loss_" + name)
            f.argtypes = [C.c_int] * 4 + [rp] * 5 + [ip, dp]
            f.restype = C.c_int
            g = getattr(L, "ref_mlp_grad_mse_" + name)
            g.argtypes = [C.c_int] * 4 + [rp] * 6 + [rp] * 4 + [dp] + [rp] * 2
            g.restype = C.c_int
            f = getattr(L, "ref_mlp_mse_" + name)
            f.argtypes = [C.c_int] * 4 + [rp] * 6 + [dp]
            f.restype = C.c_int
        L.ref_sgemm.restype = L.ref_sgemm_exact.restype = L.ref_threads.restype = C.c_int
        _lib = L
    return _lib


def threads() -> int:
    """Host threads the oracle's row-parallel loops use."""
    return int(lib().ref_threads())


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    a = np.asarray(a)
    assert a.dtype == np.float32 and a.flags.c_contiguous, "oracle sgemm takes C-contiguous float32"
    return a


def sgemm(transa: str, transb: str, m: int, n: int, k: int, alpha: float, A, lda: int, B, ldb: int, beta: float,
          Cmat, ldc: int) -> np.ndarray:
    """Float-accumulator triple loop; returns a new array shaped like Cmat (rows x ldc storage)."""
    A, B = _f32(A), _f32(B)
    out = np.array(_f32(Cmat), copy=True)
    rc = lib().ref_sgemm(transa.encode(), transb.encode(), m, n, k, alpha, _p(A, C.c_float), lda,
                         _p(B, C.c_float), ldb, beta, _p(out, C.c_float), ldc)
    if rc:
        raise ValueError(f"ref_sgemm: bad argument {rc}")
    return out


def sgemm_exact(transa: str, transb: str, m: int, n: int, k: int, alpha: float, A, lda: int, B, ldb: int,
                beta: float, C0, ldc: int):
    """Double-accumulator reference: returns (Cref[m x n] float64, S[m x n] float64 = sum_p |a||b|)."""
    A, B, C0 = _f32(A), _f32(B), _f32(C0)
    Cref = np.empty((m, n), dtype=np.float64)
    S = np.empty((m, n), dtype=np.float64)
    rc = lib().ref_sgemm_exact(transa.encode(), transb.encode(), m, n, k, alpha, _p(A, C.c_float), lda,
                               _p(B, C.c_float), ldb, beta, _p(C0, C.c_float), ldc, _p(Cref, C.c_double),
                               _p(S, C.c_double))
    if rc:
        raise ValueError(f"ref_sgemm_exact: bad argument {rc}")
    return Cref, S


class MlpGrad:
    """Result of one oracle gradient evaluation (all arrays in the oracle's arithmetic type)."""
    __slots__ = ("dW1", "dW2", "db1", "db2", "loss", "H", "P", "dO", "dA1")


def mlp_grad(W1, W2, X, labels, b1=None, b2=None, dtype=np.float64, intermediates: bool = False) -> MlpGrad:
    """Loss and gradient of the MLP, summed over the patterns, every operation in `dtype`.

    Inputs of another float type are converted first (float32 -> float64 is exact).
    """
    dtype = np.dtype(dtype)
    ct, sfx = (C.c_double, "f64") if dtype == np.float64 else (C.c_float, "f32")
    cv = lambda a: None if a is None else np.ascontiguousarray(np.asarray(a), dtype=dtype)
    W1, W2, X, b1, b2 = cv(W1), cv(W2), cv(X), cv(b1), cv(b2)
    labels = np.ascontiguousarray(np.asarray(labels), dtype=np.int32)
    n_in, n_hid = W1.shape
    n_out = W2.shape[1]
    batch = X.shape[0]
    assert W2.shape[0] == n_hid and X.shape == (batch, n_in) and labels.shape == (batch,)
    assert (b1 is None) == (b2 is None)
    r = MlpGrad()
    r.dW1 = np.empty((n_in, n_hid), dtype)
    r.dW2 = np.empty((n_hid, n_out), dtype)
    r.db1 = None if b1 is None else np.empty(n_hid, dtype)
    r.db2 = None if b2 is None else np.empty(n_out, dtype)
    r.H = np.empty((batch, n_hid), dtype) if intermediates else None
    r.P = np.empty((batch, n_out), dtype) if intermediates else None
    r.dO = np.empty((batch, n_out), dtype) if intermediates else None
    r.dA1 = np.empty((batch, n_hid), dtype) if intermediates else None
    loss = C.c_double(0.0)
    rc = getattr(lib(), "ref_mlp_grad_" + sfx)(
        n_in, n_hid, n_out, batch, _p(W1, ct), _p(W2, ct), _p(b1, ct), _p(b2, ct), _p(X, ct),
        _p(labels, C.c_int), _p(r.dW1, ct), _p(r.dW2, ct), _p(r.db1, ct), _p(r.db2, ct), C.byref(loss),
        _p(r.H, ct), _p(r.P, ct), _p(r.dO, ct), _p(r.dA1, ct))
    if rc:
        raise ValueError(f"ref_mlp_grad: error {rc}")
    r.loss = loss.value
    return r


def mlp_loss(W1, W2, X, labels, b1=None, b2=None, dtype=np.float64) -> float:
    """Loss alone (forward only), summed over the patterns."""
    dtype = np.dtype(dtype)
    ct, sfx = (C.c_double, "f64") if dtype == np.float64 else (C.c_float, "f32")
    cv = lambda a: None if a is None else np.ascontiguousarray(np.asarray(a), dtype=dtype)
    W1, W2, X, b1, b2 = cv(W1), cv(W2), cv(X), cv(b1), cv(b2)
    labels = np.ascontiguousarray(np.asarray(labels), dtype=np.int32)
    n_in, n_hid = W1.shape
    loss = C.c_double(0.0)
    rc = getattr(lib(), "ref_mlp_loss_" + sfx)(n_in, n_hid, W2.shape[1], X.shape[0], _p(W1, ct), _p(W2, ct),
                                               _p(b1, ct), _p(b2, ct), _p(X, ct), _p(labels, C.c_int),
                                               C.byref(loss))
    if rc:
        raise ValueError(f"ref_mlp_loss: error {rc}")
    return loss.value


class MlpMseGrad:
    """Result of one oracle evaluation of the paper's tanh-output / squared-error form."""
    __slots__ = ("dW1", "dW2", "db1", "db2", "loss", "H", "Y")


def mlp_grad_mse(W1, W2, X, T, b1=None, b2=None, dtype=np.float64, intermediates: bool = False) -> MlpMseGrad:
    """E = sum (tanh(tanh(X W1 + b1) W2 + b2) - T)^2 and its true gradient, every operation in `dtype`."""
    dtype = np.dtype(dtype)
    ct, sfx = (C.c_double, "f64") if dtype == np.float64 else (C.c_float, "f32")
    cv = lambda a: None if a is None else np.ascontiguousarray(np.asarray(a), dtype=dtype)
    W1, W2, X, T, b1, b2 = cv(W1), cv(W2), cv(X), cv(T), cv(b1), cv(b2)
    n_in, n_hid = W1.shape
    n_out = W2.shape[1]
    batch = X.shape[0]
    assert W2.shape[0] == n_hid and X.shape == (batch, n_in) and T.shape == (batch, n_out)
    assert (b1 is None) == (b2 is None)
    r = MlpMseGrad()
    r.dW1 = np.empty((n_in, n_hid), dtype)
    r.dW2 = np.empty((n_hid, n_out), dtype)
    r.db1 = None if b1 is None else np.empty(n_hid, dtype)
    r.db2 = None if b2 is None else np.empty(n_out, dtype)
    r.H = np.empty((batch, n_hid), dtype) if intermediates else None
    r.Y = np.empty((batch, n_out), dtype) if intermediates else None
    loss = C.c_double(0.0)
    rc = getattr(lib(), "ref_mlp_grad_mse_" + sfx)(
        n_in, n_hid, n_out, batch, _p(W1, ct), _p(W2, ct), _p(b1, ct), _p(b2, ct), _p(X, ct), _p(T, ct),
        _p(r.dW1, ct), _p(r.dW2, ct), _p(r.db1, ct), _p(r.db2, ct), C.byref(loss), _p(r.H, ct), _p(r.Y, ct))
    if rc:
        raise ValueError(f"ref_mlp_grad_mse: error {rc}")
    r.loss = loss.value
    return r


def mlp_mse(W1, W2, X, T, b1=None, b2=None, dtype=np.float64) -> float:
    """E alone (forward only)."""
    dtype = np.dtype(dtype)
    ct, sfx = (C.c_double, "f64") if dtype == np.float64 else (C.c_float, "f32")
    cv = lambda a: None if a is None else np.ascontiguousarray(np.asarray(a), dtype=dtype)
    W1, W2, X, T, b1, b2 = cv(W1), cv(W2), cv(X), cv(T), cv(b1), cv(b2)
    loss = C.c_double(0.0)
    rc = getattr(lib(), "ref_mlp_mse_" + sfx)(W1.shape[0], W1.shape[1], W2.shape[1], X.shape[0], _p(W1, ct),
                                              _p(W2, ct), _p(b1, ct), _p(b2, ct), _p(X, ct), _p(T, ct),
                                              C.byref(loss))
    if rc:
        raise ValueError(f"ref_mlp_mse: error {rc}")
    return loss.value


# ---------------------------------------------------------------------------------------------------------
# counting formulas (the paper's conventions: elementwise and reduction work is not counted)
# ---------------------------------------------------------------------------------------------------------

def sgemm_flops(m: int, n: int, k: int) -> int:
    """2MNK (section 3.1)."""
    return 2 * m * n * k


def param_count(n_in: int, n_hid: int, n_out: int) -> int:
    """Weights of a one-hidden-layer net without biases (section 5.1: 100-50-50 -> 7500; 400-480-3203 -> 1,729,440)."""
    return n_in * n_hid + n_hid * n_out


def error_flops(n_p: int, n_in: int, n_hid: int, n_out: int) -> int:
    """2 n_p (n_i + n_o) n_h for one evaluation of the error (section 6.2)."""
    return 2 * n_p * (n_in + n_out) * n_hid


def grad_flops(n_p: int, n_in: int, n_hid: int, n_out: int) -> int:
    """n_p (4 n_i n_h + 6 n_h n_o) for one gradient (section 6.2)."""
    return n_p * (4 * n_in * n_hid + 6 * n_hid * n_out)
