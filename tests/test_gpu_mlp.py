"""Parity of ulsnn_mlp_grad / ulsnn_mlp_grad_epoch (HIP, through the C ABI) against the CPU oracle.

Bar (task statement): relative L2 error <= 1e-4 per gradient tensor against the double-precision oracle fed the
same fp32 inputs; loss within 1e-5 relative.  fp32 products summed over up to 4096..90000 patterns carry a
relative error of a few 1e-7, so beside the bar every comparison also holds
  * an element-wise bound: no entry may be off by more than ELEMENT_TOL times the sum of the absolute values of
    the terms it is made of, computed from the oracle's intermediates (a lone wrong element of 1.5 million moves
    a norm by almost nothing; and where terms cancel, an error relative to the entry itself means nothing), and
  * a regression threshold, REGRESSION_L2, on the norm of the error against the norm of those sums.
"""
import math
from types import SimpleNamespace

import numpy as np
import pytest
import torch

import oracle
import paper_1911_05181_amd as ulsnn
import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_GRAD, TOL_LOSS = 1e-4, 1e-5
ELEMENT_TOL = 1e-5          # per entry, against the sum of the absolute values of its terms
REGRESSION_L2 = 2e-6        # norm of the error against the norm of those sums


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
    """`ref` carries the oracle's gradient and, as ref.bound[name], the sum of the absolute values of the terms
    each entry is made of (see _with_bounds): fp32 rounding and the kernels' fast exp / tanh are small multiples
    of 2^-24 of THAT, whatever cancels in the sum itself."""
    torch.cuda.synchronize()
    worst = worst_el = worst_l2 = 0.0
    for name in ("dW1", "dW2", "db1", "db2"):
        g, r = getattr(res, name), getattr(ref, name)
        if r is None:
            continue
        g = g.cpu().numpy().astype(np.float64)
        assert np.isfinite(g).all(), (tag, name, "not finite")
        e = _rel(g, r)
        worst = max(worst, e)
        assert e <= TOL_GRAD, (tag, name, e)
        bound = ref.bound[name]
        assert (np.abs(r) <= bound * (1 + 1e-9) + 1e-300).all(), (tag, name, "bound below the value it bounds")
        err = np.abs(g - r)
        tiny = 1e-30
        el = (err / (bound + tiny)).max()
        l2 = np.linalg.norm(err) / (np.linalg.norm(bound) + tiny)
        worst_el, worst_l2 = max(worst_el, el), max(worst_l2, l2)
        assert el <= ELEMENT_TOL, (tag, name, "one element off", el)
        assert l2 <= REGRESSION_L2, (tag, name, "error norm far above what fp32 rounding explains", l2)
    le = abs(res.loss.item() - ref.loss) / max(abs(ref.loss), 1e-30)
    assert le <= TOL_LOSS, (tag, "loss", le)
    print(f"{tag}: worst gradient rel-L2 {worst:.2e}; against the sums of absolute terms: worst element "
          f"{worst_el:.2e}, worst norm {worst_l2:.2e}; loss rel {le:.2e}")


def _gpu_grad(W1, W2, b1, b2, X, y, **kw):
    return ulsnn.mlp_grad(_dev(W1), _dev(W2), _dev(X), _dev(y), _dev(b1), _dev(b2), **kw)


def _with_bounds(g, W1, W2, b1, X, y):
    """The oracle's result with .bound added: for every gradient entry the sum over patterns of the absolute
    values of the terms it is made of, where each factor that is itself a sum with cancellation counts with the
    absolute values of ITS terms: a hidden activation as min(1, |b1| + |x| |W1|), the output delta as P + onehot
    (what is subtracted to form it), the hidden delta as (P + onehot) |W2|^T (1 - H^2).  P and H are the
    oracle's own intermediates."""
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    n_out = g.P.shape[1]
    y = np.asarray(y)
    live = (y >= 0) & (y < n_out)
    D = g.P * live[:, None]
    D[np.nonzero(live)[0], y[live]] += 1.0
    Xa = np.abs(f64(X))
    Ha = np.minimum(1.0, Xa @ np.abs(f64(W1)) + (0.0 if b1 is None else np.abs(f64(b1))))
    E = (D @ np.abs(f64(W2)).T) * (1.0 - g.H * g.H)
    bound = {"dW2": Ha.T @ D, "db2": D.sum(axis=0), "dW1": Xa.T @ E, "db1": E.sum(axis=0)}
    return SimpleNamespace(dW1=g.dW1, dW2=g.dW2, db1=g.db1, db2=g.db2, loss=g.loss, bound=bound)


def _oracle_grad(W1, W2, b1, b2, X, y):
    g = oracle.mlp_grad(_np(W1), _np(W2), _np(X), _np(y), _np(b1), _np(b2), intermediates=True)
    return _with_bounds(g, _np(W1), _np(W2), _np(b1), _np(X), _np(y))


class _Sum:
    """Float64 sum of oracle gradients over consecutive slices of the patterns."""

    def __init__(self):
        self.dW1 = self.dW2 = self.db1 = self.db2 = None
        self.loss = 0.0
        self.bound = {}

    def add(self, g):
        for name in ("dW1", "dW2", "db1", "db2"):
            v = getattr(g, name)
            if v is not None:
                cur = getattr(self, name)
                setattr(self, name, v.astype(np.float64) if cur is None else cur + v)
                self.bound[name] = g.bound[name] if cur is None else self.bound[name] + g.bound[name]
        self.loss += g.loss


def _oracle_grad_in_slices(W1, W2, b1, b2, X, y, rows=512):
    """The oracle's gradient over many patterns as the sum of its gradients over slices of `rows` patterns:
    error and gradient are additive over patterns (section 4.3; pinned for the oracle in its own tests), and the
    oracle's weight-gradient loops walk all patterns once per weight, which for tens of thousands of patterns no
    longer fits any cache."""
    total = _Sum()
    for r0 in range(0, X.shape[0], rows):
        total.add(_oracle_grad(W1, W2, b1, b2, X[r0:r0 + rows], y[r0:r0 + rows]))
    return total


def _plan_lines(text):
    """{section: {product: (tile, splits, kchunk)}} of a plan description; sections are "pass" and "tail"."""
    out, cur = {}, None
    for line in text.strip().splitlines():
        if line.startswith("rows_per_pass="):
            cur = out.setdefault("pass", {})
        elif line.startswith("tail_rows="):
            cur = out.setdefault("tail", {})
        else:
            name, rest = line.split(": ")
            f = dict(kv.split("=") for kv in rest.split())
            cur[name] = (f["tile"], int(f["splits"]), int(f["kchunk"]))
    return out


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


def test_epoch_chunk_plans_against_the_oracle():
    """The kernels the 9,000,000-pattern epoch really runs, element by element against the oracle.

    Its last chunk has 87,104 patterns = one internal pass of 65536 (planned exactly like each of the four passes
    of a 262144-pattern chunk: large tiles with the bias / tanh' epilogues inside the products, 160-row tiles and
    long k splits for the weight gradients) + a pass of 21568 (another set of tile shapes).  The plan description
    is checked first, so this test cannot drift off those plans unnoticed."""
    shape, n = si.MLP_JOCR, 87_104
    full = _plan_lines(ulsnn.mlp_grad_describe_plan(shape.n_in, shape.n_hid, shape.n_out, 262_144))
    last = _plan_lines(ulsnn.mlp_grad_describe_plan(shape.n_in, shape.n_hid, shape.n_out, n))
    assert "tail" not in full and last["pass"] == full["pass"], (full, last)
    big_tiles = {"256x128", "128x128w8", "160x128"}
    assert {t for t, _, _ in last["pass"].values()} & big_tiles and last["pass"]["dW2"][1] > 1
    assert last["tail"] != last["pass"]
    print("pass of 65536:", last["pass"])
    print("pass of 21568:", last["tail"])
    p = _problem(shape, 2, n)
    res = _gpu_grad(*p)
    torch.cuda.synchronize()
    _compare(res, _oracle_grad_in_slices(*p), "400-480-3203 B=87104 (65536 + 21568)")
    # the same patterns through the epoch driver in chunks of 65536: the chunk call with accumulation
    ep = ulsnn.mlp_grad_epoch(_dev(p[0]), _dev(p[1]), _dev(p[4]), _dev(p[5]), 65536)
    torch.cuda.synchronize()
    assert _rel(ep.dW2.cpu().numpy(), res.dW2.cpu().numpy().astype(np.float64)) < 1e-6


def test_check_labels_counts_the_ignored_patterns():
    y = torch.tensor([0, 5, -1, 9, 10, 3, 1 << 30, -(1 << 31), 9], dtype=torch.int32)
    assert ulsnn.check_labels(_dev(y), 10).item() == 4
    assert ulsnn.check_labels(_dev(y), 11).item() == 3
    assert ulsnn.check_labels(_dev(y[:0]), 10).item() == 0
    _, big = si.mlp_patterns(si.MLP_JOCR, 2, 0, 100_000)
    assert ulsnn.check_labels(_dev(big), 3203).item() == 0
    assert ulsnn.check_labels(_dev(big), 1000).item() == int((big >= 1000).sum())


def test_call_on_a_side_stream_with_a_library_allocated_workspace():
    """stream= other than the current stream, no workspace given: the binding's temporary workspace must stay
    untouched until the queued kernels have run, whatever the caller allocates meanwhile on the current stream."""
    p = _problem(si.MlpShape(100, 130, 259, True), 5, 300, random_biases=True)
    W1, W2, b1, b2, X, y = (_dev(t) for t in p)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    res = ulsnn.mlp_grad(W1, W2, X, y, b1, b2, stream=side)
    junk = [torch.full((1 << 20,), float("nan"), device=DEV) for _ in range(16)]   # would reuse a freed block
    torch.cuda.current_stream().wait_stream(side)
    _compare(res, _oracle_grad(*p), "side stream")
    del junk


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
