"""Host-side checks of the C ABI that need no GPU: every declared symbol is exported, and argument
validation (which runs before any HIP call) returns the documented status codes."""
import ctypes as C
import os
import re

import pytest

import paper_1911_05181_amd as ulsnn
from paper_1911_05181_amd.binding import _MlpDesc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, E_NULL, E_TRANS, E_DIM, E_LD, E_WS, E_UNSUP, E_HIP = range(8)


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ulsnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ulsnn_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ulsnn.load()
    names = _declared_functions()
    assert {"ulsnn_sgemm", "ulsnn_mlp_grad", "ulsnn_mlp_grad_epoch", "ulsnn_mlp_grad_workspace_bytes",
            "ulsnn_status_string", "ulsnn_version", "ulsnn_sgemm_flops", "ulsnn_mlp_grad_flops"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings_and_version():
    assert ulsnn.version() >= 100
    seen = {ulsnn.status_string(s) for s in range(8)}
    assert len(seen) == 8 and ulsnn.status_string(99) == "unknown status"


def test_counting_conventions_match_the_paper():
    # section 3.1: 2MNK; section 6.2: n_p (4 n_i n_h + 6 n_h n_o); section 5.1 network
    assert ulsnn.sgemm_flops(320, 320, 320) == 2 * 320**3
    assert ulsnn.mlp_grad_flops(400, 480, 3203, 1) == 9_992_640
    assert int(ulsnn.mlp_grad_flops(400, 480, 3203, 9_264_000) / 1e12) == 92
    assert round(ulsnn.mlp_loss_flops(400, 480, 3203, 9_264_000) / 1e12) == 32      # "32 Tera" for one error evaluation


def _sgemm(ta, tb, m, n, k, lda, ldb, ldc, A=1, B=1, Cm=1, alpha=1.0):
    # pointers are never dereferenced on these paths: every call below must be rejected (or be a no-op)
    L = ulsnn.load()
    p = lambda v: C.c_void_p(0x1000 if v else 0)
    return L.ulsnn_sgemm(ta.encode(), tb.encode(), m, n, k, alpha, p(A), lda, p(B), ldb, 0.0, p(Cm), ldc, None)


def test_sgemm_argument_errors():
    assert _sgemm("X", "N", 4, 4, 4, 4, 4, 4) == E_TRANS
    assert _sgemm("N", "Q", 4, 4, 4, 4, 4, 4) == E_TRANS
    assert _sgemm("N", "N", -1, 4, 4, 4, 4, 4) == E_DIM
    assert _sgemm("N", "N", 4, -1, 4, 4, 4, 4) == E_DIM
    assert _sgemm("N", "N", 4, 4, -1, 4, 4, 4) == E_DIM
    assert _sgemm("N", "N", 4, 5, 6, 5, 5, 5) == E_LD      # lda < k
    assert _sgemm("T", "N", 4, 5, 6, 3, 5, 5) == E_LD      # A stored k x m: lda < m
    assert _sgemm("N", "N", 4, 5, 6, 6, 4, 5) == E_LD      # ldb < n
    assert _sgemm("N", "T", 4, 5, 6, 6, 5, 5) == E_LD      # B stored n x k: ldb < k
    assert _sgemm("N", "N", 4, 5, 6, 6, 5, 4) == E_LD      # ldc < n
    assert _sgemm("N", "N", 0, 5, 6, 6, 5, 5) == OK        # m == 0: nothing to do, no launch
    assert _sgemm("N", "N", 4, 0, 6, 6, 1, 1) == OK
    assert _sgemm("N", "N", 4, 5, 6, 6, 5, 5, Cm=0) == E_NULL
    assert _sgemm("N", "N", 4, 5, 6, 6, 5, 5, A=0) == E_NULL
    assert _sgemm("N", "N", 4, 5, 6, 6, 5, 5, B=0) == E_NULL
    for t in "NnTtCc":
        assert _sgemm(t, t, 0, 0, 0, 1, 1, 1) == OK


def _desc(**kw):
    d = _MlpDesc()
    d.n_in, d.n_hid, d.n_out = 400, 480, 3203
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def _grad(d, W1=1, W2=1, X=1, y=1, batch=8, dW1=1, dW2=1, loss=1):
    L = ulsnn.load()
    p = lambda v: C.c_void_p(0x1000 if v else 0)
    return L.ulsnn_mlp_grad(C.byref(d) if d is not None else None, p(W1), p(W2), p(X), p(y), batch, p(dW1),
                            p(dW2), p(loss))


def test_mlp_grad_argument_errors():
    assert _grad(None) == E_NULL
    assert _grad(_desc(n_hid=0)) == E_DIM
    assert _grad(_desc(), batch=-1) == E_DIM
    for missing in ("W1", "W2", "X", "y", "dW1", "dW2", "loss"):
        assert _grad(_desc(), **{missing: 0}) == E_NULL
    assert _grad(_desc(b1=0x1000)) == E_NULL                     # biases: all four or none
    assert _grad(_desc(b1=0x1000, b2=0x1000, db1=0x1000)) == E_NULL
    assert _grad(_desc(operand_dtype=2)) == E_UNSUP              # only fp32 (0) and bf16 storage (1) exist
    assert _grad(_desc(operand_dtype=1)) == E_WS                 # bf16 storage: accepted, then needs a workspace
    assert _grad(_desc(accumulate=2)) == E_UNSUP
    assert _grad(_desc()) == E_WS                                # no workspace
    need = ulsnn.mlp_grad_workspace_bytes(400, 480, 3203, 8)
    assert _grad(_desc(workspace=0x1000, workspace_bytes=need - 1)) == E_WS
    assert _grad(_desc(workspace=0x1010, workspace_bytes=need)) == E_WS      # not 256-byte aligned
    L = ulsnn.load()
    p = C.c_void_p(0x1000)
    d = _desc(workspace=0x1000, workspace_bytes=1 << 40)
    assert L.ulsnn_mlp_grad_epoch(C.byref(d), p, p, p, p, 100, 0, p, p, p) == E_DIM
    assert L.ulsnn_mlp_grad_epoch(C.byref(_desc()), p, p, p, p, 100, 10, p, p, p) == E_WS


def test_sgemm_planned_argument_errors_and_plan_description():
    L = ulsnn.load()
    p = C.c_void_p(0x1000)
    f = lambda tile, sp, ta, tb, m, n, k, ws=None, wsb=0: L.ulsnn_sgemm_planned(
        tile, sp, ta, tb, m, n, k, 1.0, p, max(k, m, 1), p, max(n, k, 1), 0.0, p, max(n, 1), ws, wsb, None)
    assert f(len(ulsnn.TILE_SHAPES), 1, b"N", b"N", 8, 8, 8) == E_DIM           # no such tile shape
    assert f(-1, 1, b"N", b"N", 8, 8, 8) == E_DIM
    assert f(0, 0, b"N", b"N", 8, 8, 8) == E_DIM           # k_splits < 1
    assert f(0, 1, b"X", b"N", 8, 8, 8) == E_TRANS
    assert f(0, 1, b"N", b"N", 0, 8, 8) == OK              # empty product: nothing to do
    assert f(2, 4, b"N", b"N", 64, 64, 256) == E_WS        # split without workspace
    assert f(2, 4, b"N", b"N", 64, 64, 256, C.c_void_p(0x1000), 100) == E_WS   # too small
    assert f(2, 4, b"N", b"N", 64, 64, 256, C.c_void_p(0x1010), 1 << 20) == E_WS   # misaligned
    assert L.ulsnn_sgemm_planned(0, 1, b"N", b"N", 8, 8, 8, 1.0, p, 4, p, 8, 0.0, p, 8, None, 0, None) == E_LD
    line = ulsnn.sgemm_describe_plan("N", "T", 8192, 8192, 8192)
    assert line.startswith("tile=256x128 ") and "splits=1" in line
    assert ulsnn.sgemm_describe_plan("N", "N", 64, 64, 64).startswith("tile=64x64")
    assert ulsnn.sgemm_describe_plan("N", "N", 1024, 1024, 1024).startswith("tile=64x64k64 ")   # under-filled launch
    buf = C.create_string_buffer(8)
    assert L.ulsnn_sgemm_describe_plan(b"N", b"N", 0, 8, 8, buf, 8) == E_DIM
    assert L.ulsnn_sgemm_describe_plan(b"N", b"N", 8, 8, 8, None, 8) == E_NULL


def test_optimiser_step_argument_errors():
    L = ulsnn.load()
    p, ws = C.c_void_p(0x1000), C.c_void_p(0x2000)
    n = ulsnn.VEC_WORKSPACE_BYTES
    assert L.ulsnn_dot(-1, p, p, p, ws, n, None) == E_DIM
    assert L.ulsnn_dot(8, None, p, p, ws, n, None) == E_NULL
    assert L.ulsnn_dot(8, p, p, None, ws, n, None) == E_NULL
    assert L.ulsnn_dot(8, p, p, p, None, n, None) == E_WS
    assert L.ulsnn_dot(8, p, p, p, ws, n - 1, None) == E_WS
    assert L.ulsnn_dot(8, p, p, p, C.c_void_p(0x2010), n, None) == E_WS
    assert L.ulsnn_axpy(-1, 1.0, p, p, None) == E_DIM
    assert L.ulsnn_axpy(0, 1.0, None, None, None) == OK
    assert L.ulsnn_axpy(8, 1.0, None, p, None) == E_NULL
    assert L.ulsnn_cg_direction(8, None, p, p, p, ws, n, None) == E_NULL
    assert L.ulsnn_cg_direction(8, p, p, None, p, ws, n, None) == E_NULL
    assert L.ulsnn_cg_direction(8, p, p, p, p, ws, 100, None) == E_WS
    assert L.ulsnn_cg_direction(-2, p, p, p, p, ws, n, None) == E_DIM
    # line search
    res = ulsnn.LineSearchResult()
    f = lambda d, batch=8, bracket=4, alpha0=0.1, k=5, r=res: L.ulsnn_mlp_line_search(
        C.byref(d), p, p, p, p, p, p, batch, bracket, alpha0, k, C.byref(r) if r is not None else None)
    assert f(_desc(), r=None) == E_NULL
    assert f(_desc(), batch=0) == E_DIM
    assert f(_desc(), bracket=0) == E_DIM
    assert f(_desc(), alpha0=0.0) == E_DIM
    assert f(_desc(), alpha0=float("inf")) == E_DIM
    assert f(_desc(), k=-1) == E_DIM
    assert f(_desc(), k=61) == E_DIM
    assert f(_desc(operand_dtype=1)) == E_UNSUP
    assert f(_desc(b1=0x1000, b2=0x1000, db1=0x1000, db2=0x1000)) == E_UNSUP
    assert f(_desc()) == E_WS
    need = ulsnn.mlp_line_search_workspace_bytes(400, 480, 3203, 8)
    assert need > ulsnn.mlp_grad_workspace_bytes(400, 480, 3203, 8) + 2 * 4 * (400 * 480 + 480 * 3203)
    assert f(_desc(workspace=0x1000, workspace_bytes=need - 1)) == E_WS
    assert L.ulsnn_mlp_line_search(C.byref(_desc(workspace=0x1000, workspace_bytes=need)), p, p, None, p, p, p, 8, 4,
                                   0.1, 5, C.byref(res)) == E_NULL


def test_loss_only_and_mse_argument_errors():
    L = ulsnn.load()
    p, z = C.c_void_p(0x1000), C.c_void_p(0)
    d = _desc()
    assert L.ulsnn_mlp_loss(None, p, p, p, p, 8, p) == E_NULL
    assert L.ulsnn_mlp_loss(C.byref(d), p, p, p, p, 8, z) == E_NULL
    assert L.ulsnn_mlp_loss(C.byref(d), p, p, p, z, 8, p) == E_NULL          # labels missing
    assert L.ulsnn_mlp_loss(C.byref(d), p, p, p, p, -1, p) == E_DIM
    assert L.ulsnn_mlp_loss(C.byref(d), p, p, p, p, 8, p) == E_WS            # needs the workspace
    assert L.ulsnn_mlp_grad_mse(C.byref(d), p, p, p, z, 8, p, p, p) == E_NULL   # targets missing
    assert L.ulsnn_mlp_grad_mse(C.byref(_desc(operand_dtype=1)), p, p, p, p, 8, p, p, p) == E_WS    # bf16: accepted
    assert L.ulsnn_mlp_mse(C.byref(_desc(operand_dtype=2)), p, p, p, p, 8, p) == E_UNSUP
    assert L.ulsnn_mlp_grad_mse(C.byref(d), p, p, p, p, 8, p, p, p) == E_WS


def test_workspace_query():
    w = ulsnn.mlp_grad_workspace_bytes
    assert w(400, 480, 3203, 0) == 0 and w(0, 480, 3203, 16) == 0
    sizes = [w(400, 480, 3203, b) for b in (1, 100, 4096, 32768, 65536, 65537, 262144, 9_000_000)]
    assert all(a <= b for a, b in zip(sizes, sizes[1:]))         # non-decreasing in batch
    assert sizes[-1] == sizes[-2] == sizes[-3] == sizes[-4]      # constant above the internal pass size
    assert sizes[2] >= 4096 * (3203 + 2 * 480) * 4               # holds Z, H and dA1 of the batch
    assert sizes[-1] < 2 << 30                                   # and stays modest for any batch


def test_bf16_workspace_is_separate_query():
    w32 = ulsnn.mlp_grad_workspace_bytes(400, 480, 3203, 4096, 0)
    w16 = ulsnn.mlp_grad_workspace_bytes(400, 480, 3203, 4096, 1)
    assert w16 > 0 and w16 != w32
    # bf16 path: H, dA1 and the logits / output delta are 2 bytes wide, the softmax statistics of the output
    # layer's epilogue (8 bytes per row and 32 columns) stand in for fp32 logits, plus aligned weight copies
    assert w16 >= 4096 * (3232 * 2 + 101 * 8 + 2 * 480 * 2) + 480 * 3208 * 2
    assert w16 < w32


def test_plan_description():
    text = ulsnn.mlp_grad_describe_plan(400, 480, 3203, 4096)
    lines = text.strip().splitlines()
    assert lines[0].startswith("rows_per_pass=4096")
    names = [l.split(":")[0] for l in lines[1:]]
    assert names == ["hidden_layer", "output_layer", "dW2", "hidden_delta", "dW1"]      # the five products
    for l in lines[1:]:
        f = dict(kv.split("=") for kv in l.split(": ")[1].split())
        tm, tn = (int(v) for v in f["tiles"].split("x"))
        assert tm >= 1 and tn >= 1 and int(f["splits"]) >= 1 and float(f["model_us"]) > 0
        assert int(f["splits"]) * int(f["kchunk"]) >= {"hidden_layer": 400, "output_layer": 480, "dW2": 4096,
                                                        "hidden_delta": 3203, "dW1": 4096}[l.split(":")[0]]
    # the weight-gradient products have few output tiles and a long k: they must be k-split to fill 256 CUs
    split = {l.split(":")[0]: int(dict(kv.split("=") for kv in l.split(": ")[1].split())["splits"]) for l in lines[1:]}
    assert split["dW2"] > 1 and split["dW1"] > 1 and split["hidden_layer"] == 1 and split["output_layer"] == 1
    L = ulsnn.load()
    import ctypes as C2
    buf = C2.create_string_buffer(16)
    d = _desc()
    assert L.ulsnn_mlp_grad_describe_plan(C2.byref(d), 4096, buf, 16) == OK and len(buf.value) <= 15   # truncated
    assert L.ulsnn_mlp_grad_describe_plan(None, 4096, buf, 16) == E_NULL
    assert L.ulsnn_mlp_grad_describe_plan(C2.byref(d), 0, buf, 16) == E_DIM


def test_binding_refuses_cpu_tensors():
    import torch
    a = torch.zeros(4, 4)
    with pytest.raises(TypeError):
        ulsnn.sgemm("N", "N", 4, 4, 4, 1.0, a, 4, a, 4, 0.0, a, 4)


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only: any other --gpus value ends with a message and a non-zero status before any
    GPU or library work."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and r.stdout.strip() == ""
    assert "ONE GPU" in r.stderr and "--gpus 2" in r.stderr


def test_sgemm_ws_argument_errors():
    L = ulsnn.load()
    p = C.c_void_p(0x1000)
    f = lambda ta, tb, m, n, k, lda, ldb, ldc, ws, wsb: L.ulsnn_sgemm_ws(ta, tb, m, n, k, 1.0, p, lda, p, ldb, 0.0, p, ldc,
                                                                         ws, wsb, None)
    assert f(b"X", b"N", 4, 4, 4, 4, 4, 4, None, 0) == E_TRANS
    assert f(b"N", b"N", -1, 4, 4, 4, 4, 4, None, 0) == E_DIM
    assert f(b"N", b"N", 4, 5, 6, 5, 5, 5, None, 0) == E_LD
    assert f(b"N", b"N", 4, 5, 6, 6, 5, 5, None, 1024) == E_WS                   # bytes without a pointer
    assert f(b"N", b"N", 4, 5, 6, 6, 5, 5, C.c_void_p(0x1010), 1024) == E_WS     # misaligned
    assert f(b"N", b"N", 0, 5, 6, 6, 5, 5, None, 0) == OK                        # nothing to do
    assert L.ulsnn_sgemm_ws(b"N", b"N", 4, 5, 6, 1.0, None, 6, p, 5, 0.0, p, 5, None, 0, None) == E_NULL


def test_leading_dimension_and_network_size_limits():
    """Kernels keep 32-bit element offsets inside a tile of up to 256 rows, so lda / ldb (and the network
    dimensions, which become leading dimensions) above ULSNN_MAX_LD are refused before anything is launched."""
    L = ulsnn.load()
    max_ld = 1 << 24
    assert 255 * max_ld + 64 < 1 << 32      # what the limit protects: row 255 of a tile, plus a k step
    assert _sgemm("N", "N", 4, 5, 6, max_ld + 1, 5, 5) == E_UNSUP
    assert _sgemm("N", "N", 4, 5, 6, 6, max_ld + 1, 5) == E_UNSUP
    p = C.c_void_p(0x1000)
    assert L.ulsnn_sgemm_planned(0, 1, b"N", b"N", 8, 8, 8, 1.0, p, max_ld + 1, p, 8, 0.0, p, 8, None, 0, None) == E_UNSUP
    assert _grad(_desc(n_out=max_ld + 1)) == E_UNSUP
    assert _grad(_desc(n_in=max_ld + 8)) == E_UNSUP


def test_check_labels_and_static_scratch_argument_errors():
    L = ulsnn.load()
    p = C.c_void_p(0x1000)
    assert L.ulsnn_check_labels(p, -1, 10, p, None) == E_DIM
    assert L.ulsnn_check_labels(p, 5, 0, p, None) == E_DIM
    assert L.ulsnn_check_labels(None, 5, 10, p, None) == E_NULL
    assert L.ulsnn_check_labels(p, 5, 10, None, None) == E_NULL
    assert ulsnn.static_scratch_bytes() == 64 << 20
    # validation comes first, then the size check against the built-in array: neither touches the GPU
    assert L.ulsnn_mlp_grad_static(None, p, p, p, p, 8, p, p, p) == E_NULL
    assert L.ulsnn_mlp_grad_static(C.byref(_desc()), p, p, None, p, 8, p, p, p) == E_NULL
    assert ulsnn.mlp_grad_workspace_bytes(400, 480, 3203, 4096) > ulsnn.static_scratch_bytes()
    assert L.ulsnn_mlp_grad_static(C.byref(_desc()), p, p, p, p, 4096, p, p, p) == E_WS


def test_plan_description_lists_the_shorter_last_pass():
    text = ulsnn.mlp_grad_describe_plan(400, 480, 3203, 87104)        # 65536 + 21568
    lines = text.strip().splitlines()
    assert lines[0].startswith("rows_per_pass=65536") and len(lines) == 12
    assert lines[6].startswith("tail_rows=21568")
    assert [l.split(":")[0] for l in lines[7:]] == ["hidden_layer", "output_layer", "dW2", "hidden_delta", "dW1"]
    # a whole number of passes has no tail section, and its first pass is planned like any 65536-row pass
    whole = ulsnn.mlp_grad_describe_plan(400, 480, 3203, 262144).strip().splitlines()
    assert len(whole) == 6 and whole[1:] == lines[1:6]


class _NoLaunch:
    """Stands in for the loaded library: any call through it fails the test."""

    def __getattr__(self, name):
        raise AssertionError(f"the binding called {name} although an argument was invalid")


def test_binding_checks_every_tensor_before_calling_the_library(monkeypatch):
    """Wrong dtype, shape, size or layout of ANY tensor argument (biases and caller-supplied outputs included)
    raises in Python; the library, which would hand the pointers to kernels, is never reached.  The device
    predicate is replaced so that the checks can run on CPU tensors here."""
    import torch
    from paper_1911_05181_amd import binding as b

    real_lib = b.load()
    monkeypatch.setattr(b, "_on_gpu", lambda t: isinstance(t, torch.Tensor))
    monkeypatch.setattr(b, "load", lambda: _NoLaunch())
    monkeypatch.setattr(b, "mlp_grad_workspace_bytes", lambda *a: 1024)
    n_in, n_hid, n_out, batch = 6, 5, 4, 3
    W1, W2 = torch.zeros(n_in, n_hid), torch.zeros(n_hid, n_out)
    X, y = torch.zeros(batch, n_in), torch.zeros(batch, dtype=torch.int32)
    b1, b2 = torch.zeros(n_hid), torch.zeros(n_out)

    def out(**kw):
        o = b.MlpGradResult(torch.zeros(n_in, n_hid), torch.zeros(n_hid, n_out), torch.zeros(1), torch.zeros(n_hid),
                            torch.zeros(n_out))
        for k, v in kw.items():
            setattr(o, k, v)
        return o

    bad = [
        dict(b1=b1.double(), b2=b2), dict(b1=b1, b2=b2[:3]), dict(b1=torch.zeros(n_hid + 1), b2=b2),
        dict(b1=b1, b2=torch.zeros(2 * n_out)[::2]),
        dict(out=out(dW2=torch.zeros(n_hid, n_out + 1))), dict(out=out(dW1=torch.zeros(n_hid, n_in))),
        dict(out=out(dW1=torch.zeros(n_in, n_hid, dtype=torch.float64))), dict(out=out(loss=torch.zeros(2))),
        dict(out=out(dW2=torch.zeros(n_out, n_hid).t())),
        dict(b1=b1, b2=b2, out=out(db1=torch.zeros(n_hid - 1))), dict(b1=b1, b2=b2, out=out(db2=None)),
        dict(workspace=[1, 2, 3]),
    ]
    for kw in bad:
        with pytest.raises((TypeError, ValueError)):
            b.mlp_grad(W1, W2, X, y, **kw)
    with pytest.raises((TypeError, ValueError)):
        b.mlp_loss(W1, W2, X, y, loss=torch.zeros(3))
    with pytest.raises((TypeError, ValueError)):
        b.mlp_grad_static(W1, W2, X, y, b1, b2, out=out(db1=torch.zeros(1)))
    # SGEMM: the stored operands must lie inside their tensors
    A, B, Cm = torch.zeros(4 * 6), torch.zeros(6 * 5), torch.zeros(4 * 5)
    for args in [("N", "N", 4, 5, 6, 1.0, A, 7, B, 5, 0.0, Cm, 5),      # lda 7: A would need 27 elements
                 ("N", "N", 4, 5, 6, 1.0, A, 6, B, 6, 0.0, Cm, 5),      # ldb 6: B would need 35
                 ("N", "N", 4, 5, 6, 1.0, A, 6, B, 5, 0.0, Cm, 6),      # ldc 6: C would need 23
                 ("T", "N", 5, 5, 6, 1.0, A, 5, B, 5, 0.0, torch.zeros(25), 5),   # A stored 6 x 5 with lda 5: 30 > 24
                 ("N", "T", 4, 6, 6, 1.0, A, 6, B, 6, 0.0, torch.zeros(24), 6)]:  # B stored 6 x 6: 36 > 30
        with pytest.raises(ValueError):
            b.sgemm(*args)
        with pytest.raises(ValueError):
            b.sgemm_planned(5, 1, *args)
    del real_lib


def test_bench_reads_its_traffic_figures_from_the_committed_profiles():
    """bench.py's roofline.traffic comes from lines of the profile summaries, not from constants in the script."""
    import importlib.util
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    fp32 = bench.pmc_traffic()
    for stage in ("backward_products", "output_layer", "hidden_layer", "dW1_product"):
        assert fp32[stage] > 1e6
    # the paired backward launch moves at least its algorithmic bytes (read dO twice, H, W2; write the partials)
    assert fp32["backward_products"] >= 2 * 4096 * 3203 * 4 + 4096 * 480 * 4 + 480 * 3203 * 4
    bf16 = bench.pmc_traffic(bench.TRAFFIC_PROFILE_BF16)
    assert bf16["bf16_gradient"] >= 65536 * (400 + 4 * 480 + 3 * 3203) * 2


def test_sgemm_ws_plan_splits_only_where_it_pays():
    """Host only: with a workspace the planner cuts k where the product cannot fill the chip otherwise (512^3, a small
    output with a long k) and leaves the close calls unsplit (256^3, 1024^3); without room for two slices never."""
    def splits(*a):
        return int(ulsnn.sgemm_ws_describe_plan(*a).split("splits=")[1].split()[0])
    room = lambda m, n: 64 * m * n * 4
    assert splits("N", "N", 512, 512, 512, room(512, 512)) > 1
    assert splits("T", "N", 256, 256, 65536, room(256, 256)) > 8
    assert splits("N", "N", 256, 256, 256, room(256, 256)) == 1
    assert splits("N", "T", 1024, 1024, 1024, room(1024, 1024)) == 1
    assert splits("N", "N", 512, 512, 512, 512 * 512 * 4) == 1
    assert splits("N", "N", 512, 512, 512, 0) == 1
    L = ulsnn.load()
    import ctypes
    buf = ctypes.create_string_buffer(64)
    assert L.ulsnn_sgemm_ws_describe_plan(b"N", b"N", 8, 8, 8, 0, None, 8) == 1      # null buffer
    assert L.ulsnn_sgemm_ws_describe_plan(b"X", b"N", 8, 8, 8, 0, buf, 64) == 2      # bad trans
    assert L.ulsnn_sgemm_ws_describe_plan(b"N", b"N", 0, 8, 8, 0, buf, 64) == 3      # bad dimension
