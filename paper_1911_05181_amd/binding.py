"""ctypes binding of libulsnn.so: same names as the C entry points, argument marshalling only.

There is no fallback: if the library has not been built, or a call returns an error status, an exception is
raised.  Tensors must live on the GPU (their data_ptr() is handed to the library as a device pointer).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libulsnn.so"
_lib = None


class UlsnnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class _MlpDesc(C.Structure):
    _fields_ = [("n_in", C.c_int), ("n_hid", C.c_int), ("n_out", C.c_int),
                ("b1", C.c_void_p), ("b2", C.c_void_p), ("db1", C.c_void_p), ("db2", C.c_void_p),
                ("accumulate", C.c_int), ("operand_dtype", C.c_int),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("hip_stream", C.c_void_p)]


class LineSearchResult(C.Structure):
    """ulsnn_line_search_result (host memory)."""
    _fields_ = [("alpha", C.c_float), ("loss", C.c_float), ("loss0", C.c_float), ("bracket_lo", C.c_float),
                ("bracket_hi", C.c_float), ("error_evaluations", C.c_int), ("gradient_evaluations", C.c_int)]


VEC_WORKSPACE_BYTES = 16640   # ULSNN_VEC_WORKSPACE_BYTES


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load():
    """Load the shared library (built in-tree by paper_1911_05181_amd/build.py).  Fails loudly if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_1911_05181_amd.build` "
                          f"(or __graft_entry__.build()); there is no fallback path")
    L = C.CDLL(path)
    vp, i, f = C.c_void_p, C.c_int, C.c_float
    L.ulsnn_sgemm.argtypes = [C.c_char, C.c_char, i, i, i, f, vp, i, vp, i, f, vp, i, vp]
    L.ulsnn_sgemm.restype = i
    L.ulsnn_sgemm_ws.argtypes = [C.c_char, C.c_char, i, i, i, f, vp, i, vp, i, f, vp, i, vp, C.c_size_t, vp]
    L.ulsnn_sgemm_ws.restype = i
    L.ulsnn_mlp_grad_workspace_bytes.argtypes = [C.POINTER(_MlpDesc), i]
    L.ulsnn_mlp_grad_workspace_bytes.restype = C.c_size_t
    L.ulsnn_mlp_grad.argtypes = [C.POINTER(_MlpDesc), vp, vp, vp, vp, i, vp, vp, vp]
    L.ulsnn_mlp_grad.restype = i
    L.ulsnn_mlp_grad_static.argtypes = [C.POINTER(_MlpDesc), vp, vp, vp, vp, i, vp, vp, vp]
    L.ulsnn_mlp_grad_static.restype = i
    L.ulsnn_static_scratch_bytes.argtypes = []
    L.ulsnn_static_scratch_bytes.restype = C.c_size_t
    L.ulsnn_static_scratch_init.argtypes = []
    L.ulsnn_static_scratch_init.restype = i
    L.ulsnn_check_labels.argtypes = [vp, C.c_int64, i, vp, vp]
    L.ulsnn_check_labels.restype = i
    L.ulsnn_mlp_grad_epoch.argtypes = [C.POINTER(_MlpDesc), vp, vp, vp, vp, C.c_int64, i, vp, vp, vp]
    L.ulsnn_mlp_grad_epoch.restype = i
    L.ulsnn_mlp_grad_timed.argtypes = [C.POINTER(_MlpDesc), vp, vp, vp, vp, i, vp, vp, vp, C.POINTER(C.c_float)]
    L.ulsnn_mlp_grad_timed.restype = i
    L.ulsnn_mlp_loss.argtypes = [C.POINTER(_MlpDesc), vp, vp, vp, vp, i, vp]
    L.ulsnn_mlp_loss.restype = i
    L.ulsnn_mlp_grad_mse.argtypes = [C.POINTER(_MlpDesc), vp, vp, vp, vp, i, vp, vp, vp]
    L.ulsnn_mlp_grad_mse.restype = i
    L.ulsnn_mlp_mse.argtypes = [C.POINTER(_MlpDesc), vp, vp, vp, vp, i, vp]
    L.ulsnn_mlp_mse.restype = i
    L.ulsnn_mlp_loss_flops.argtypes = [i, i, i, C.c_int64]
    L.ulsnn_mlp_loss_flops.restype = C.c_double
    L.ulsnn_dot.argtypes = [C.c_int64, vp, vp, vp, vp, C.c_size_t, vp]
    L.ulsnn_dot.restype = i
    L.ulsnn_axpy.argtypes = [C.c_int64, f, vp, vp, vp]
    L.ulsnn_axpy.restype = i
    L.ulsnn_cg_direction.argtypes = [C.c_int64, vp, vp, vp, vp, vp, C.c_size_t, vp]
    L.ulsnn_cg_direction.restype = i
    L.ulsnn_mlp_line_search_workspace_bytes.argtypes = [C.POINTER(_MlpDesc), i]
    L.ulsnn_mlp_line_search_workspace_bytes.restype = C.c_size_t
    L.ulsnn_mlp_line_search.argtypes = [C.POINTER(_MlpDesc), vp, vp, vp, vp, vp, vp, i, i, f, i,
                                        C.POINTER(LineSearchResult)]
    L.ulsnn_mlp_line_search.restype = i
    L.ulsnn_sgemm_planned.argtypes = [i, i, C.c_char, C.c_char, i, i, i, C.c_float, vp, i, vp, i, C.c_float, vp, i, vp,
                                      C.c_size_t, vp]
    L.ulsnn_sgemm_planned.restype = i
    L.ulsnn_sgemm_describe_plan.argtypes = [C.c_char, C.c_char, i, i, i, C.c_char_p, C.c_size_t]
    L.ulsnn_sgemm_describe_plan.restype = i
    L.ulsnn_sgemm_ws_describe_plan.argtypes = [C.c_char, C.c_char, i, i, i, C.c_size_t, C.c_char_p, C.c_size_t]
    L.ulsnn_sgemm_ws_describe_plan.restype = i
    L.ulsnn_mlp_grad_describe_plan.argtypes = [C.POINTER(_MlpDesc), i, C.c_char_p, C.c_size_t]
    L.ulsnn_mlp_grad_describe_plan.restype = i
    L.ulsnn_device_info.argtypes = [C.POINTER(i), C.POINTER(i), C.POINTER(i)]
    L.ulsnn_device_info.restype = i
    L.ulsnn_clock_probe.argtypes = [C.c_double, vp, vp]
    L.ulsnn_clock_probe.restype = i
    L.ulsnn_sgemm_flops.argtypes = [i, i, i]
    L.ulsnn_sgemm_flops.restype = C.c_double
    L.ulsnn_mlp_grad_flops.argtypes = [i, i, i, C.c_int64]
    L.ulsnn_mlp_grad_flops.restype = C.c_double
    L.ulsnn_status_string.argtypes = [i]
    L.ulsnn_status_string.restype = C.c_char_p
    L.ulsnn_version.argtypes = []
    L.ulsnn_version.restype = i
    _lib = L
    return L


def status_string(status: int) -> str:
    return load().ulsnn_status_string(int(status)).decode()


def version() -> int:
    return int(load().ulsnn_version())


def device_info() -> dict:
    """Compute units, maximum shader clock and wall-clock rate (kHz) of the current device (ulsnn_device_info)."""
    cu, sclk, wall = C.c_int(0), C.c_int(0), C.c_int(0)
    rc = load().ulsnn_device_info(C.byref(cu), C.byref(sclk), C.byref(wall))
    if rc:
        raise UlsnnError(rc, "ulsnn_device_info")
    return {"compute_units": cu.value, "max_shader_clock_khz": sclk.value, "wall_clock_khz": wall.value}


def clock_probe(window_ms: float, out: torch.Tensor, stream=None) -> None:
    """Queue the clock probe (ulsnn_clock_probe); `out` is a two-element int64 GPU tensor: shader cycles, wall ticks."""
    if not (_on_gpu(out) and out.dtype == torch.int64 and out.numel() == 2 and out.is_contiguous()):
        raise TypeError("out must be a contiguous two-element int64 tensor on the GPU")
    rc = load().ulsnn_clock_probe(float(window_ms), _ptr(out), _stream(stream))
    if rc:
        raise UlsnnError(rc, "ulsnn_clock_probe")


def sgemm_flops(m: int, n: int, k: int) -> float:
    return float(load().ulsnn_sgemm_flops(m, n, k))


def mlp_grad_flops(n_in: int, n_hid: int, n_out: int, batch: int) -> float:
    return float(load().ulsnn_mlp_grad_flops(n_in, n_hid, n_out, batch))


def mlp_loss_flops(n_in: int, n_hid: int, n_out: int, batch: int) -> float:
    return float(load().ulsnn_mlp_loss_flops(n_in, n_hid, n_out, batch))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _on_gpu(t) -> bool:
    return isinstance(t, torch.Tensor) and t.is_cuda


def _dev_f32(t: torch.Tensor, name: str):
    if not (_on_gpu(t) and t.dtype == torch.float32):
        raise TypeError(f"{name} must be a float32 tensor on the GPU")


def _dense_f32(t: torch.Tensor, name: str, numel: int = None, shape=None):
    """A contiguous float32 GPU tensor, optionally of a given element count or shape."""
    _dev_f32(t, name)
    if not t.is_contiguous():
        raise ValueError(f"{name} must be dense (contiguous)")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{name} must hold {numel} elements, not {t.numel()}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, not {tuple(t.shape)}")


def _workspace(workspace, need: int, device, stream):
    """The caller's workspace (checked), or a fresh one.  A fresh one is handed to torch's caching allocator
    again when this function's caller returns, while the kernels that use it may still be queued: that is safe on
    the current stream (same-stream reuse is ordered) and, with record_stream, on any other stream."""
    if workspace is not None:
        if not (_on_gpu(workspace) and workspace.is_contiguous()):
            raise TypeError("workspace must be a contiguous GPU tensor")
        return workspace
    workspace = torch.empty(max(int(need), 256), dtype=torch.uint8, device=device)
    if stream is not None:
        workspace.record_stream(stream)
    return workspace


def _check_gemm_operand(t, name, rows, cols, ld):
    """The stored matrix (rows x cols, row stride ld) must lie inside the tensor."""
    if rows <= 0 or cols <= 0:
        return
    if t is None:
        raise ValueError(f"{name} is missing")
    if ld < cols:
        return                      # the library reports the leading-dimension error
    if (rows - 1) * ld + cols > t.numel():
        raise ValueError(f"{name}: {rows} x {cols} with leading dimension {ld} needs "
                         f"{(rows - 1) * ld + cols} elements, the tensor holds {t.numel()}")


def _check_sgemm_tensors(transa, transb, m, n, k, alpha, A, lda, B, ldb, Cmat, ldc):
    """Types, and that every element the product touches lies inside its tensor (the library cannot know the
    size of the memory behind a pointer).  Flags and sizes themselves are checked by the library."""
    for t, nm in ((A, "A"), (B, "B"), (Cmat, "C")):
        if t is not None:
            _dense_f32(t, nm)
    if min(m, n, k) < 0 or str(transa)[:1] not in "NnTtCc" or str(transb)[:1] not in "NnTtCc":
        return
    _check_gemm_operand(Cmat, "C", m, n, ldc)
    if m > 0 and n > 0 and k > 0 and alpha != 0.0:
        a_rows, a_cols = (m, k) if str(transa)[:1] in "Nn" else (k, m)
        b_rows, b_cols = (k, n) if str(transb)[:1] in "Nn" else (n, k)
        _check_gemm_operand(A, "A", a_rows, a_cols, lda)
        _check_gemm_operand(B, "B", b_rows, b_cols, ldb)


def sgemm(transa: str, transb: str, m: int, n: int, k: int, alpha: float, A: torch.Tensor, lda: int,
          B: torch.Tensor, ldb: int, beta: float, Cmat: torch.Tensor, ldc: int, stream=None) -> None:
    """C = alpha*op(A)*op(B) + beta*C in place on the GPU (row-major, BLAS SGEMM argument order)."""
    _check_sgemm_tensors(transa, transb, m, n, k, alpha, A, lda, B, ldb, Cmat, ldc)
    rc = load().ulsnn_sgemm(transa.encode()[:1], transb.encode()[:1], m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb,
                            beta, _ptr(Cmat), ldc, _stream(stream))
    if rc:
        raise UlsnnError(rc, "ulsnn_sgemm")


def sgemm_ws(transa: str, transb: str, m: int, n: int, k: int, alpha: float, A: torch.Tensor, lda: int,
             B: torch.Tensor, ldb: int, beta: float, Cmat: torch.Tensor, ldc: int, workspace: torch.Tensor,
             stream=None) -> None:
    """ulsnn_sgemm_ws: SGEMM that may split k into as many slices as `workspace` holds partial products for."""
    _check_sgemm_tensors(transa, transb, m, n, k, alpha, A, lda, B, ldb, Cmat, ldc)
    if workspace is not None and not (_on_gpu(workspace) and workspace.is_contiguous()):
        raise TypeError("workspace must be a contiguous GPU tensor")
    rc = load().ulsnn_sgemm_ws(transa.encode()[:1], transb.encode()[:1], m, n, k, alpha, _ptr(A), lda, _ptr(B), ldb,
                               beta, _ptr(Cmat), ldc, _ptr(workspace),
                               0 if workspace is None else workspace.numel() * workspace.element_size(),
                               _stream(stream))
    if rc:
        raise UlsnnError(rc, "ulsnn_sgemm_ws")


def _vec_ws(workspace, device, stream=None):
    return _workspace(workspace, VEC_WORKSPACE_BYTES, device, stream)


def dot(x: torch.Tensor, y: torch.Tensor, *, out: Optional[torch.Tensor] = None, workspace=None, stream=None):
    """sum x*y over all elements (ulsnn_dot); returns a one-element device tensor."""
    _dev_f32(x, "x"), _dev_f32(y, "y")
    if x.numel() != y.numel() or not (x.is_contiguous() and y.is_contiguous()):
        raise ValueError("dot: contiguous tensors of equal size")
    if out is None:
        out = torch.empty(1, device=x.device)
    workspace = _vec_ws(workspace, x.device, stream)
    rc = load().ulsnn_dot(x.numel(), _ptr(x), _ptr(y), _ptr(out), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise UlsnnError(rc, "ulsnn_dot")
    return out


def axpy(alpha: float, x: torch.Tensor, y: torch.Tensor, stream=None) -> torch.Tensor:
    """y += alpha*x in place (ulsnn_axpy)."""
    _dev_f32(x, "x"), _dev_f32(y, "y")
    if x.numel() != y.numel() or not (x.is_contiguous() and y.is_contiguous()):
        raise ValueError("axpy: contiguous tensors of equal size")
    rc = load().ulsnn_axpy(x.numel(), alpha, _ptr(x), _ptr(y), _stream(stream))
    if rc:
        raise UlsnnError(rc, "ulsnn_axpy")
    return y


def cg_direction(g_new: torch.Tensor, g_old: Optional[torch.Tensor], d: torch.Tensor, *, beta=None, workspace=None,
                 stream=None):
    """Polak-Ribiere update of the direction d in place (ulsnn_cg_direction); returns (d, beta device tensor)."""
    _dev_f32(g_new, "g_new"), _dev_f32(d, "d")
    if g_old is not None:
        _dev_f32(g_old, "g_old")
    for t in (g_new, d) + ((g_old,) if g_old is not None else ()):
        if t.numel() != g_new.numel() or not t.is_contiguous():
            raise ValueError("cg_direction: contiguous tensors of equal size")
    if beta is None:
        beta = torch.empty(1, device=d.device)
    workspace = _vec_ws(workspace, d.device, stream)
    rc = load().ulsnn_cg_direction(g_new.numel(), _ptr(g_new), _ptr(g_old), _ptr(d), _ptr(beta), _ptr(workspace),
                                   workspace.numel(), _stream(stream))
    if rc:
        raise UlsnnError(rc, "ulsnn_cg_direction")
    return d, beta


def mlp_line_search_workspace_bytes(n_in: int, n_hid: int, n_out: int, batch: int) -> int:
    d = _desc(n_in, n_hid, n_out, None, None, None, None, False, None, None)
    return int(load().ulsnn_mlp_line_search_workspace_bytes(C.byref(d), batch))


def mlp_line_search(W1, W2, d1, d2, X, labels, bracket_batch: int, alpha0: float, max_doublings: int, *,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> LineSearchResult:
    """Line search along (d1, d2); updates W1, W2 in place (ulsnn_mlp_line_search).  Synchronises the stream."""
    n_in, n_hid, n_out, _, odt = _mlp_common(W1, W2, X, labels, None, None, MlpGradResult(None, None, None), False)
    for t, ref, nm in ((d1, W1, "d1"), (d2, W2, "d2")):
        _dev_f32(t, nm)
        if t.shape != ref.shape or not t.is_contiguous():
            raise ValueError(f"{nm} must be contiguous and shaped like its weight matrix")
    batch = X.shape[0]
    workspace = _workspace(workspace, mlp_line_search_workspace_bytes(n_in, n_hid, n_out, batch), W1.device, stream)
    d = _desc(n_in, n_hid, n_out, None, None, None, None, False, workspace, stream, odt)
    res = LineSearchResult()
    rc = load().ulsnn_mlp_line_search(C.byref(d), _ptr(W1), _ptr(W2), _ptr(d1), _ptr(d2), _ptr(X), _ptr(labels), batch,
                                      bracket_batch, alpha0, max_doublings, C.byref(res))
    if rc:
        raise UlsnnError(rc, "ulsnn_mlp_line_search")
    return res


TILE_SHAPES = ("256x128", "128x128w8", "128x128", "128x64", "64x128", "64x64", "64x64k64", "160x128", "64x64k32")   # index = ULSNN_TILE_*


def sgemm_planned(tile_shape: int, k_splits: int, transa: str, transb: str, m: int, n: int, k: int, alpha: float,
                  A: torch.Tensor, lda: int, B: torch.Tensor, ldb: int, beta: float, Cmat: torch.Tensor, ldc: int,
                  workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """ulsnn_sgemm_planned: SGEMM with the tile shape and k split chosen by the caller."""
    _check_sgemm_tensors(transa, transb, m, n, k, alpha, A, lda, B, ldb, Cmat, ldc)
    if k_splits > 1 and m > 0 and n > 0 and Cmat is not None:
        workspace = _workspace(workspace, k_splits * m * n * 4, Cmat.device, stream)
    rc = load().ulsnn_sgemm_planned(tile_shape, k_splits, transa.encode()[:1], transb.encode()[:1], m, n, k, alpha,
                                    _ptr(A), lda, _ptr(B), ldb, beta, _ptr(Cmat), ldc, _ptr(workspace),
                                    0 if workspace is None else workspace.numel() * workspace.element_size(),
                                    _stream(stream))
    if rc:
        raise UlsnnError(rc, "ulsnn_sgemm_planned")


def _desc(n_in, n_hid, n_out, b1, b2, db1, db2, accumulate, workspace, stream, operand_dtype=0) -> _MlpDesc:
    d = _MlpDesc()
    d.n_in, d.n_hid, d.n_out = n_in, n_hid, n_out
    d.b1, d.b2, d.db1, d.db2 = _ptr(b1), _ptr(b2), _ptr(db1), _ptr(db2)
    d.accumulate = int(accumulate)
    d.operand_dtype = operand_dtype
    d.workspace = _ptr(workspace)
    d.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    d.hip_stream = _stream(stream) if torch.cuda.is_available() else None
    return d


def mlp_grad_workspace_bytes(n_in: int, n_hid: int, n_out: int, batch: int, operand_dtype: int = 0) -> int:
    """Workspace bytes for fp32 (operand_dtype 0) or bf16-stored (1) operands."""
    d = _MlpDesc()
    d.n_in, d.n_hid, d.n_out = n_in, n_hid, n_out
    d.operand_dtype = operand_dtype
    return int(load().ulsnn_mlp_grad_workspace_bytes(C.byref(d), batch))


def sgemm_describe_plan(transa: str, transb: str, m: int, n: int, k: int) -> str:
    """Tile shape and grid ulsnn_sgemm would use (host only)."""
    buf = C.create_string_buffer(256)
    rc = load().ulsnn_sgemm_describe_plan(transa.encode(), transb.encode(), m, n, k, buf, len(buf))
    if rc:
        raise UlsnnError(rc, "ulsnn_sgemm_describe_plan")
    return buf.value.decode()


def sgemm_ws_describe_plan(transa: str, transb: str, m: int, n: int, k: int, workspace_bytes: int) -> str:
    """Tile shape, grid and k split ulsnn_sgemm_ws would use with a workspace of that size (host only)."""
    buf = C.create_string_buffer(256)
    rc = load().ulsnn_sgemm_ws_describe_plan(transa.encode(), transb.encode(), m, n, k, workspace_bytes, buf, len(buf))
    if rc:
        raise UlsnnError(rc, "ulsnn_sgemm_ws_describe_plan")
    return buf.value.decode()


def mlp_grad_describe_plan(n_in: int, n_hid: int, n_out: int, batch: int) -> str:
    """Tile shapes, k splits and modelled times the library would use (host-only; launches nothing)."""
    d = _MlpDesc()
    d.n_in, d.n_hid, d.n_out = n_in, n_hid, n_out
    buf = C.create_string_buffer(2048)
    rc = load().ulsnn_mlp_grad_describe_plan(C.byref(d), batch, buf, len(buf))
    if rc:
        raise UlsnnError(rc, "ulsnn_mlp_grad_describe_plan")
    return buf.value.decode()


@dataclass
class MlpGradResult:
    dW1: torch.Tensor
    dW2: torch.Tensor
    loss: torch.Tensor            # one float on the device
    db1: Optional[torch.Tensor] = None
    db2: Optional[torch.Tensor] = None


def _mlp_common(W1, W2, X, labels, b1, b2, out, accumulate, dense_targets=False):
    """Checks shapes and types; returns (n_in, n_hid, n_out, out, operand_dtype).  W1, W2 and X are all float32
    (operand_dtype 0) or all bfloat16 (operand_dtype 1); gradients and loss are always float32.  `labels` is the
    int32 label vector, or with dense_targets the float32 target matrix [batch x n_out]."""
    if W1.dtype == torch.bfloat16:
        for t, nm in ((W1, "W1"), (W2, "W2"), (X, "X")):
            if not (_on_gpu(t) and t.dtype == torch.bfloat16):
                raise TypeError(f"{nm} must be a bfloat16 tensor on the GPU (W1 is bfloat16)")
        operand_dtype = 1
    else:
        _dev_f32(W1, "W1"), _dev_f32(W2, "W2"), _dev_f32(X, "X")
        operand_dtype = 0
    if dense_targets:
        _dev_f32(labels, "T")
        if labels.dim() != 2 or labels.shape[1] != W2.shape[1]:
            raise ValueError("T must be [batch x n_out]")
    elif not (_on_gpu(labels) and labels.dtype == torch.int32):
        raise TypeError("labels must be an int32 tensor on the GPU")
    for t in (W1, W2, X, labels):
        if not t.is_contiguous():
            raise ValueError("W1, W2, X and labels must be dense (contiguous)")
    n_in, n_hid = W1.shape
    n_out = W2.shape[1]
    if W2.shape[0] != n_hid or X.shape[1] != n_in or labels.shape[0] != X.shape[0]:
        raise ValueError("shape mismatch between W1, W2, X and labels")
    if (b1 is None) != (b2 is None):
        raise ValueError("give both biases or neither")
    if b1 is not None:
        _dense_f32(b1, "b1", numel=n_hid)
        _dense_f32(b2, "b2", numel=n_out)
    if out is not None:
        if out.dW1 is not None or out.dW2 is not None:
            _dense_f32(out.dW1, "out.dW1", shape=W1.shape)
            _dense_f32(out.dW2, "out.dW2", shape=W2.shape)
        if out.loss is not None:
            _dense_f32(out.loss, "out.loss", numel=1)
        if b1 is not None and out.dW1 is not None:
            if out.db1 is None or out.db2 is None:
                raise ValueError("out.db1 and out.db2 are needed when biases are given")
            _dense_f32(out.db1, "out.db1", numel=n_hid)
            _dense_f32(out.db2, "out.db2", numel=n_out)
    if out is None:
        if accumulate:
            raise ValueError("accumulate=True needs the tensors to add to (out=...)")
        dev = W1.device
        out = MlpGradResult(torch.empty(W1.shape, dtype=torch.float32, device=dev),
                            torch.empty(W2.shape, dtype=torch.float32, device=dev), torch.empty(1, device=dev),
                            None if b1 is None else torch.empty_like(b1),
                            None if b2 is None else torch.empty_like(b2))
    return n_in, n_hid, n_out, out, operand_dtype


def mlp_grad(W1, W2, X, labels, b1=None, b2=None, *, out: Optional[MlpGradResult] = None, accumulate=False,
             workspace: Optional[torch.Tensor] = None, stream=None) -> MlpGradResult:
    """Loss and gradient of the MLP summed over the rows of X (ulsnn_mlp_grad).  Asynchronous on the stream."""
    n_in, n_hid, n_out, out, odt = _mlp_common(W1, W2, X, labels, b1, b2, out, accumulate)
    batch = X.shape[0]
    workspace = _workspace(workspace, mlp_grad_workspace_bytes(n_in, n_hid, n_out, batch, odt), W1.device, stream)
    d = _desc(n_in, n_hid, n_out, b1, b2, out.db1, out.db2, accumulate, workspace, stream, odt)
    rc = load().ulsnn_mlp_grad(C.byref(d), _ptr(W1), _ptr(W2), _ptr(X), _ptr(labels), batch, _ptr(out.dW1),
                               _ptr(out.dW2), _ptr(out.loss))
    if rc:
        raise UlsnnError(rc, "ulsnn_mlp_grad")
    return out


def mlp_grad_static(W1, W2, X, labels, b1=None, b2=None, *, out: Optional[MlpGradResult] = None, accumulate=False,
                    stream=None) -> MlpGradResult:
    """ulsnn_mlp_grad_static: the gradient with the library's built-in scratch array instead of a workspace."""
    n_in, n_hid, n_out, out, odt = _mlp_common(W1, W2, X, labels, b1, b2, out, accumulate)
    d = _desc(n_in, n_hid, n_out, b1, b2, out.db1, out.db2, accumulate, None, stream, odt)
    rc = load().ulsnn_mlp_grad_static(C.byref(d), _ptr(W1), _ptr(W2), _ptr(X), _ptr(labels), X.shape[0],
                                      _ptr(out.dW1), _ptr(out.dW2), _ptr(out.loss))
    if rc:
        raise UlsnnError(rc, "ulsnn_mlp_grad_static")
    return out


def static_scratch_bytes() -> int:
    return int(load().ulsnn_static_scratch_bytes())


def static_scratch_init() -> None:
    rc = load().ulsnn_static_scratch_init()
    if rc:
        raise UlsnnError(rc, "ulsnn_static_scratch_init")


def check_labels(labels: torch.Tensor, n_out: int, *, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Number of labels outside [0, n_out) as a one-element int64 device tensor (ulsnn_check_labels)."""
    if not (_on_gpu(labels) and labels.dtype == torch.int32 and labels.is_contiguous()):
        raise TypeError("labels must be a contiguous int32 tensor on the GPU")
    if out is None:
        out = torch.empty(1, dtype=torch.int64, device=labels.device)
    elif not (_on_gpu(out) and out.dtype == torch.int64 and out.numel() == 1):
        raise TypeError("out must be a one-element int64 tensor on the GPU")
    rc = load().ulsnn_check_labels(_ptr(labels), labels.numel(), n_out, _ptr(out), _stream(stream))
    if rc:
        raise UlsnnError(rc, "ulsnn_check_labels")
    return out


def _loss_only(entry, W1, W2, X, targets, b1, b2, loss, accumulate, workspace, stream, dense):
    n_in, n_hid, n_out, _, odt = _mlp_common(W1, W2, X, targets, b1, b2, MlpGradResult(None, None, None), accumulate,
                                              dense_targets=dense)
    batch = X.shape[0]
    if loss is None:
        if accumulate:
            raise ValueError("accumulate=True needs the tensor to add to (loss=...)")
        loss = torch.empty(1, device=W1.device)
    else:
        _dense_f32(loss, "loss", numel=1)
    workspace = _workspace(workspace, mlp_grad_workspace_bytes(n_in, n_hid, n_out, batch, odt), W1.device, stream)
    d = _desc(n_in, n_hid, n_out, b1, b2, None, None, accumulate, workspace, stream, odt)
    rc = getattr(load(), entry)(C.byref(d), _ptr(W1), _ptr(W2), _ptr(X), _ptr(targets), batch, _ptr(loss))
    if rc:
        raise UlsnnError(rc, entry)
    return loss


def mlp_loss(W1, W2, X, labels, b1=None, b2=None, *, loss=None, accumulate=False, workspace=None, stream=None):
    """Loss alone, summed over the rows of X (ulsnn_mlp_loss).  Returns the one-element device tensor."""
    return _loss_only("ulsnn_mlp_loss", W1, W2, X, labels, b1, b2, loss, accumulate, workspace, stream, False)


def mlp_mse(W1, W2, X, T, b1=None, b2=None, *, loss=None, accumulate=False, workspace=None, stream=None):
    """Summed squared error of the tanh-output network against dense targets T (ulsnn_mlp_mse)."""
    return _loss_only("ulsnn_mlp_mse", W1, W2, X, T, b1, b2, loss, accumulate, workspace, stream, True)


def mlp_grad_mse(W1, W2, X, T, b1=None, b2=None, *, out: Optional[MlpGradResult] = None, accumulate=False,
                 workspace: Optional[torch.Tensor] = None, stream=None) -> MlpGradResult:
    """Squared error of the tanh-output network and its gradient (ulsnn_mlp_grad_mse), the paper's own form."""
    n_in, n_hid, n_out, out, odt = _mlp_common(W1, W2, X, T, b1, b2, out, accumulate, dense_targets=True)
    batch = X.shape[0]
    workspace = _workspace(workspace, mlp_grad_workspace_bytes(n_in, n_hid, n_out, batch, odt), W1.device, stream)
    d = _desc(n_in, n_hid, n_out, b1, b2, out.db1, out.db2, accumulate, workspace, stream, odt)
    rc = load().ulsnn_mlp_grad_mse(C.byref(d), _ptr(W1), _ptr(W2), _ptr(X), _ptr(T), batch, _ptr(out.dW1),
                                   _ptr(out.dW2), _ptr(out.loss))
    if rc:
        raise UlsnnError(rc, "ulsnn_mlp_grad_mse")
    return out


MLP_STAGES = ("hidden_layer", "output_layer", "softmax_ce", "backward_products", "backward_reductions",
              "dW1_product", "dW1_reduction", "bias_grads")


def mlp_grad_timed(W1, W2, X, labels, b1=None, b2=None, *, out: Optional[MlpGradResult] = None, accumulate=False,
                   workspace: Optional[torch.Tensor] = None, stream=None):
    """ulsnn_mlp_grad_timed: the same work with HIP events at the stage boundaries.  Synchronises the stream.
    Returns (result, {stage name: milliseconds})."""
    n_in, n_hid, n_out, out, odt = _mlp_common(W1, W2, X, labels, b1, b2, out, accumulate)
    batch = X.shape[0]
    workspace = _workspace(workspace, mlp_grad_workspace_bytes(n_in, n_hid, n_out, batch, odt), W1.device, stream)
    d = _desc(n_in, n_hid, n_out, b1, b2, out.db1, out.db2, accumulate, workspace, stream, odt)
    ms = (C.c_float * len(MLP_STAGES))()
    rc = load().ulsnn_mlp_grad_timed(C.byref(d), _ptr(W1), _ptr(W2), _ptr(X), _ptr(labels), batch, _ptr(out.dW1),
                                     _ptr(out.dW2), _ptr(out.loss), ms)
    if rc:
        raise UlsnnError(rc, "ulsnn_mlp_grad_timed")
    return out, dict(zip(MLP_STAGES, (float(v) for v in ms)))


def mlp_grad_epoch(W1, W2, X, labels, chunk: int, b1=None, b2=None, *, out: Optional[MlpGradResult] = None,
                   accumulate=False, workspace: Optional[torch.Tensor] = None, stream=None) -> MlpGradResult:
    """Gradient over all rows of X taken `chunk` patterns at a time and summed (ulsnn_mlp_grad_epoch)."""
    n_in, n_hid, n_out, out, odt = _mlp_common(W1, W2, X, labels, b1, b2, out, accumulate)
    n = X.shape[0]
    workspace = _workspace(workspace, mlp_grad_workspace_bytes(n_in, n_hid, n_out, min(max(chunk, 1), max(n, 1)), odt),
                           W1.device, stream)
    d = _desc(n_in, n_hid, n_out, b1, b2, out.db1, out.db2, accumulate, workspace, stream, odt)
    rc = load().ulsnn_mlp_grad_epoch(C.byref(d), _ptr(W1), _ptr(W2), _ptr(X), _ptr(labels), n, chunk,
                                     _ptr(out.dW1), _ptr(out.dW2), _ptr(out.loss))
    if rc:
        raise UlsnnError(rc, "ulsnn_mlp_grad_epoch")
    return out
