"""Parity of ulsnn_mlp_grad / ulsnn_mlp_grad_epoch (HIP, through the C ABI) against the CPU oracle.

Bar (task statement): relative L2 error <= 1e-4 per gradient tensor against the double-precision oracle fed the
same fp32 inputs; loss within 1e-5 relative.  fp32 products summed over up to 4096..40000 patterns carry a
relative error of a few 1e-7..1e-6, so observed values (printed) should sit near 1e-6.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_1911_05181_amd as ulsnn
import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_GRAD, TOL_LOSS = 1e-4, 1e-5


def _rel(a, b):
    a = a.astype(np.float64)
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a)


def _problem(shape, seed, batch, random_biases=False, first=0):
    W1, W2, b1, b2 = si.mlp_weights(shape, seed)
    if shape.biases and random_biases:
        b1, b2 = si.random_biases(shape, seed, 0.2)
    X, y = si.mlp_patterns(shape, seed, first, batch)
    return W1, W2, b1, b2, X, y


def _np(t):
    return None if t is None else t.numpy()


def _dev(t):
    return None if t is None else t.to(DEV)


def _compare(res, ref, tag):
    torch.cuda.synchronize()
    worst = 0.0
    for name in ("dW1", "dW2", "db1", "db2"):
        g, r = getattr(res, name), getattr(ref, name)
        if r is None:
            continue
        e = _rel(g.cpu().numpy(), r)
        worst = max(worst, e)
        assert e <= TOL_GRAD, (tag, name, e)
    le = abs(res.loss.item() - ref.loss) / max(abs(ref.loss), 1e-30)
    assert le <= TOL_LOSS, (tag, "loss", le)
    print(f"{tag}: worst gradient rel-L2 {worst:.2e}, loss rel {le:.2e}")


def _gpu_grad(W1, W2, b1, b2, X, y, **kw):
    return ulsnn.mlp_grad(_dev(W1), _dev(W2), _dev(X), _dev(y), _dev(b1), _dev(b2), **kw)


def _oracle_grad(W1, W2, b1, b2, X, y):
    return oracle.mlp_grad(_np(W1), _np(W2), _np(X), _np(y), _np(b1), _np(b2))


def test_small_net_with_biases():
    """64-32-10, batch 256, seed 0: the small configuration (zero biases as specified, then random ones)."""
    for rb in (False, True):
        p = _problem(si.MLP_SMALL, 0, 256, random_biases=rb)
        _compare(_gpu_grad(*p), _oracle_grad(*p), f"64-32-10 B=256 random_biases={rb}")


@pytest.mark.parametrize("n_in,n_hid,n_out,batch,biases", [
    (100, 130, 259, 300, True),      # every dimension ragged against the 128/64/32 tiles
    (17, 33, 5, 1, True),            # a single pattern
    (400, 480, 3203, 257, False),    # the paper's network, a batch with a ragged tail
    (64, 32, 4500, 37, True),        # rows too long for the register softmax
    (33, 7, 2, 1000, False),
    (1, 1, 1, 3, True),              # degenerate: one class, so every delta and the loss are zero
    (3, 1, 2, 5, False),             # a single hidden unit
    (2, 5, 1, 4, True),
])
def test_ragged_shapes(n_in, n_hid, n_out, batch, biases):
    p = _problem(si.MlpShape(n_in, n_hid, n_out, biases), 5, batch, random_biases=True)
    _compare(_gpu_grad(*p), _oracle_grad(*p), f"{n_in}-{n_hid}-{n_out} B={batch}")


def test_jocr_network_full_batch():
    """400-480-3203 (the paper's network, section 6.1), batch 4096, seed 2: the benchmark workload, every
    element of both gradients against the oracle."""
    p = _problem(si.MLP_JOCR, 2, 4096)
    ref = _oracle_grad(*p)
    res = _gpu_grad(*p)
    _compare(res, ref, "400-480-3203 B=4096")
    # how far a plain fp32 evaluation (the float oracle, sums in index order) is from the double one: the GPU's
    # distance above is of this size, so the 1e-4 bound is a bound on real errors, not on rounding noise
    f32 = oracle.mlp_grad(*(_np(t) for t in (p[0], p[1], p[4], p[5])), dtype=np.float32)
    print(f"float oracle vs double oracle: dW1 {_rel(f32.dW1, ref.dW1):.2e} dW2 {_rel(f32.dW2, ref.dW2):.2e}")
    assert _rel(f32.dW1, ref.dW1) < 1e-5 and _rel(f32.dW2, ref.dW2) < 1e-5
    again = _gpu_grad(*p)
    torch.cuda.synchronize()
    assert torch.equal(res.dW1, again.dW1) and torch.equal(res.dW2, again.dW2) and torch.equal(res.loss, again.loss)


def test_empty_batch_and_accumulate():
    shape = si.MlpShape(20, 12, 9, True)
    W1, W2, b1, b2, X, y = _problem(shape, 7, 64, random_biases=True)
    res = _gpu_grad(W1, W2, b1, b2, X[:0], y[:0])
    torch.cuda.synchronize()
    for t in (res.dW1, res.dW2, res.db1, res.db2, res.loss):
        assert not t.any()
    # accumulate: two halves added into the same tensors equal the whole (additivity, section 4.3)
    out = _gpu_grad(W1, W2, b1, b2, X[:40], y[:40])
    _gpu_grad(W1, W2, b1, b2, X[40:], y[40:], out=out, accumulate=True)
    _gpu_grad(W1, W2, b1, b2, X[:0], y[:0], out=out, accumulate=True)        # adds nothing
    _compare(out, _oracle_grad(W1, W2, b1, b2, X, y), "accumulate 40+24+0")


def test_out_of_range_labels_are_ignored():
    shape = si.MlpShape(30, 20, 11, True)
    W1, W2, b1, b2, X, y = _problem(shape, 8, 50, random_biases=True)
    y = y.clone()
    y[3], y[17], y[49] = -1, 11, 1 << 20
    _compare(_gpu_grad(W1, W2, b1, b2, X, y), _oracle_grad(W1, W2, b1, b2, X, y), "ignored labels")


def test_closed_form_zero_output_weights():
    shape = si.MLP_JOCR
    W1, W2, _, _, X, y = _problem(shape, 2, 512)
    res = _gpu_grad(W1, torch.zeros_like(W2), None, None, X, y)
    torch.cuda.synchronize()
    assert abs(res.loss.item() - 512 * math.log(3203)) <= 1e-5 * 512 * math.log(3203)   # B ln n_out
    assert not res.dW1.any()                                                            # dH = dO * 0


def test_chunked_epoch_matches_oracle_and_single_call():
    """Epoch gradient over 3 chunks of 1024 + a tail of 300 patterns (the streaming path at reduced size)."""
    n = 3 * 1024 + 300
    p = _problem(si.MLP_JOCR, 2, n)
    W1, W2, _, _, X, y = p
    res = ulsnn.mlp_grad_epoch(_dev(W1), _dev(W2), _dev(X), _dev(y), 1024)
    _compare(res, _oracle_grad(*p), "epoch 3x1024+300")
    # a chunk larger than the data is a single call
    one = ulsnn.mlp_grad_epoch(_dev(W1), _dev(W2), _dev(X), _dev(y), 1 << 20)
    whole = _gpu_grad(*p)
    torch.cuda.synchronize()
    assert torch.equal(one.dW1, whole.dW1) and torch.equal(one.dW2, whole.dW2)


def test_batch_larger_than_internal_slab():
    """A batch that the library splits into several internal passes (small net so the oracle stays quick)."""
    p = _problem(si.MLP_SMALL, 0, 70_000, random_biases=True)
    _compare(_gpu_grad(*p), _oracle_grad(*p), "64-32-10 B=70000")


def test_timed_variant_matches_and_reports_stages():
    p = _problem(si.MLP_JOCR, 2, 1024)
    W1, W2, _, _, X, y = p
    want = _gpu_grad(*p)
    got, ms = ulsnn.mlp_grad_timed(_dev(W1), _dev(W2), _dev(X), _dev(y))
    torch.cuda.synchronize()
    assert torch.equal(got.dW1, want.dW1) and torch.equal(got.dW2, want.dW2) and torch.equal(got.loss, want.loss)
    assert list(ms) == list(ulsnn.MLP_STAGES) and all(v >= 0 for v in ms.values())
    assert ms["output_layer"] > 0 and ms["backward_products"] > 0
    with pytest.raises(ulsnn.UlsnnError) as e:                       # more than one internal pass: refused
        big = _problem(si.MLP_SMALL, 0, 70_000)
        ulsnn.mlp_grad_timed(_dev(big[0]), _dev(big[1]), _dev(big[4]), _dev(big[5]))
    assert e.value.status == 6


def test_additivity_on_device():
    p = _problem(si.MLP_JOCR, 2, 1500)
    W1, W2, _, _, X, y = p
    whole = _gpu_grad(*p)
    a = _gpu_grad(W1, W2, None, None, X[:700], y[:700])
    b = _gpu_grad(W1, W2, None, None, X[700:], y[700:])
    torch.cuda.synchronize()
    for name in ("dW1", "dW2"):
        s = (getattr(a, name) + getattr(b, name)).cpu().numpy()
        assert _rel(s, getattr(whole, name).cpu().numpy().astype(np.float64)) < 1e-5
    assert abs(a.loss.item() + b.loss.item() - whole.loss.item()) < 1e-5 * whole.loss.item()


def test_workspace_too_small_is_refused():
    p = _problem(si.MLP_SMALL, 0, 256)
    ws = torch.empty(1024, dtype=torch.uint8, device=DEV)
    with pytest.raises(ulsnn.UlsnnError) as e:
        _gpu_grad(*p, workspace=ws)
    assert e.value.status == 5


def test_full_size_epoch_9_million_patterns():
    """The epoch workload at its full size: 9,000,000 patterns resident on the GPU, chunks of 262144.
    The oracle cannot run 90 TFLOP, so parity is pinned by (i) additivity: the epoch gradient equals the float64
    sum of the 35 per-chunk gradients computed by separate calls, and (ii) the oracle on one 4096-pattern prefix
    of a chunk chosen in the middle of the epoch, regenerated from the counter-based generator."""
    shape, n, chunk = si.MLP_JOCR, 9_000_000, 262144
    W1, W2, _, _ = si.mlp_weights(shape, 2, device=DEV)
    X = torch.empty(n, shape.n_in, device=DEV)
    y = torch.empty(n, dtype=torch.int32, device=DEV)
    for p0 in range(0, n, chunk):
        rows = min(chunk, n - p0)
        X[p0:p0 + rows], y[p0:p0 + rows] = si.mlp_patterns(shape, 2, p0, rows, device=DEV)
    ws = torch.empty(ulsnn.mlp_grad_workspace_bytes(shape.n_in, shape.n_hid, shape.n_out, chunk), dtype=torch.uint8,
                     device=DEV)
    res = ulsnn.mlp_grad_epoch(W1, W2, X, y, chunk, workspace=ws)
    torch.cuda.synchronize()
    s1 = torch.zeros(W1.shape, dtype=torch.float64, device=DEV)
    s2 = torch.zeros(W2.shape, dtype=torch.float64, device=DEV)
    sl = 0.0
    part = ulsnn.MlpGradResult(torch.empty_like(W1), torch.empty_like(W2), torch.empty(1, device=DEV))
    for p0 in range(0, n, chunk):
        rows = min(chunk, n - p0)
        ulsnn.mlp_grad(W1, W2, X[p0:p0 + rows], y[p0:p0 + rows], out=part, workspace=ws)
        s1 += part.dW1.double()
        s2 += part.dW2.double()
        sl += part.loss.item()
    e1 = ((res.dW1.double() - s1).norm() / s1.norm()).item()
    e2 = ((res.dW2.double() - s2).norm() / s2.norm()).item()
    print(f"epoch 9e6 vs float64 sum of 35 chunk gradients: dW1 {e1:.2e} dW2 {e2:.2e} loss {abs(res.loss.item() - sl) / sl:.2e}")
    assert e1 < 1e-5 and e2 < 1e-5 and abs(res.loss.item() - sl) <= 1e-5 * sl
    # one chunk from the middle of the epoch against the oracle (first 4096 patterns of chunk 17)
    p0 = 17 * chunk
    Xc, yc = si.mlp_patterns(shape, 2, p0, 4096)                       # regenerated on the CPU
    assert torch.equal(Xc, X[p0:p0 + 4096].cpu()) and torch.equal(yc, y[p0:p0 + 4096].cpu())
    got = ulsnn.mlp_grad(W1, W2, X[p0:p0 + 4096], y[p0:p0 + 4096])
    torch.cuda.synchronize()
    _compare(got, _oracle_grad(W1.cpu(), W2.cpu(), None, None, Xc, yc), "chunk 17 prefix of the epoch")


@pytest.mark.parametrize("n_in,n_hid,n_out,batch,biases", [(64, 32, 10, 256, True), (128, 64, 40, 1000, False),
                                                          (5, 4, 3, 7, True), (17, 33, 5, 1, True),
                                                          (100, 64, 64, 4096, False), (64, 32, 10, 4097, True)])
def test_small_network_path_against_oracle_and_general_path(n_in, n_hid, n_out, batch, biases):
    """Small nets at small batches run as two launches (one workgroup per 16 patterns, then a sum of the shares).
    The event-timed entry point always takes the general path: both must agree with the oracle and each other.
    (The last case is one pattern over the small path's batch limit: general path on both sides.)"""
    p = _problem(si.MlpShape(n_in, n_hid, n_out, biases), 3, batch, random_biases=True)
    W1, W2, b1, b2, X, y = p
    ref = _oracle_grad(*p)
    small = _gpu_grad(*p)
    _compare(small, ref, f"small path {n_in}-{n_hid}-{n_out} B={batch}")
    general, _ = ulsnn.mlp_grad_timed(_dev(W1), _dev(W2), _dev(X), _dev(y), _dev(b1), _dev(b2))
    _compare(general, ref, f"general path {n_in}-{n_hid}-{n_out} B={batch}")
    for name in ("dW1", "dW2"):
        assert _rel(getattr(small, name).cpu().numpy(), getattr(general, name).cpu().numpy().astype(np.float64)) < 1e-5
    # error-only evaluation, accumulation and ignored labels on the same path
    only = ulsnn.mlp_loss(_dev(W1), _dev(W2), _dev(X), _dev(y), _dev(b1), _dev(b2))
    torch.cuda.synchronize()
    assert abs(only.item() - ref.loss) <= TOL_LOSS * ref.loss
    twice = _gpu_grad(*p)
    ulsnn.mlp_grad(_dev(W1), _dev(W2), _dev(X), _dev(y), _dev(b1), _dev(b2), out=twice, accumulate=True)
    torch.cuda.synchronize()
    assert _rel(twice.dW2.cpu().numpy(), 2 * ref.dW2) <= TOL_GRAD and abs(twice.loss.item() - 2 * ref.loss) <= 2e-5 * ref.loss
    y2 = y.clone()
    y2[::3] = -1
    _compare(_gpu_grad(W1, W2, b1, b2, X, y2), _oracle_grad(W1, W2, b1, b2, X, y2), "small path, ignored labels")


@pytest.mark.parametrize("n_in,n_hid,n_out,batch", [(64, 32, 10, 256), (100, 130, 259, 300), (400, 480, 3203, 1024)])
def test_gradient_call_can_be_captured_in_a_hip_graph(n_in, n_hid, n_out, batch):
    """The entry point only enqueues kernels on the caller's stream (no allocation, no memset, no synchronisation),
    so a caller may capture it in a HIP graph.  Every replay, with eager calls and synchronisations in between,
    must reproduce the eager result bit for bit, and that result must match the oracle."""
    p = _problem(si.MlpShape(n_in, n_hid, n_out, True), 11, batch, random_biases=True)
    W1, W2, b1, b2, X, y = (_dev(t) for t in p)
    ws = torch.empty(ulsnn.mlp_grad_workspace_bytes(n_in, n_hid, n_out, batch), dtype=torch.uint8, device=DEV)

    def fresh():
        return ulsnn.MlpGradResult(torch.empty_like(W1), torch.empty_like(W2), torch.empty(1, device=DEV),
                                   torch.empty_like(b1), torch.empty_like(b2))

    eager, replayed = fresh(), fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ulsnn.mlp_grad(W1, W2, X, y, b1, b2, out=replayed, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ulsnn.mlp_grad(W1, W2, X, y, b1, b2, out=replayed, workspace=ws)
    for _ in range(3):
        for t in (replayed.dW1, replayed.dW2, replayed.db1, replayed.db2, replayed.loss):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        ulsnn.mlp_grad(W1, W2, X, y, b1, b2, out=eager, workspace=ws)
        torch.cuda.synchronize()
        for name in ("dW1", "dW2", "db1", "db2", "loss"):
            assert torch.equal(getattr(replayed, name), getattr(eager, name)), name
    _compare(replayed, _oracle_grad(*p), f"graph replay {n_in}-{n_hid}-{n_out} B={batch}")
