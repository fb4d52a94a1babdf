"""ulsnn_mlp_grad_static (the gradient with the library's built-in scratch array, for callers that cannot allocate
or carry a workspace) against ulsnn_mlp_grad with a caller workspace, through the C ABI: two calls in a row, the
second with a smaller input, so that whatever the first call left in the shared array cannot leak into the second.
Both entry points run the same kernels with the same plans, so the results must be bit-identical; the oracle
comparison holds the usual bar (relative L2 1e-4, loss 1e-5)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1911_05181_amd as ulsnn
import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(shape, seed, batch):
    W1, W2, b1, b2 = si.mlp_weights(shape, seed)
    if shape.biases:
        b1, b2 = si.random_biases(shape, seed, 0.2)
    X, y = si.mlp_patterns(shape, seed, 0, batch)
    return W1, W2, b1, b2, X, y


def _check(p, tag):
    dev = [None if t is None else t.to(DEV) for t in p]
    W1, W2, b1, b2, X, y = dev
    got = ulsnn.mlp_grad_static(W1, W2, X, y, b1, b2)
    want = ulsnn.mlp_grad(W1, W2, X, y, b1, b2)
    torch.cuda.synchronize()
    ref = oracle.mlp_grad(*(None if t is None else t.numpy() for t in (p[0], p[1], p[4], p[5], p[2], p[3])))
    for name in ("dW1", "dW2", "db1", "db2", "loss"):
        g, w = getattr(got, name), getattr(want, name)
        if w is None:
            continue
        assert torch.equal(g, w), (tag, name)
        if name != "loss":
            r = getattr(ref, name)
            e = np.linalg.norm(g.cpu().numpy().astype(np.float64) - r) / np.linalg.norm(r)
            assert e <= 1e-4, (tag, name, e)
    assert abs(got.loss.item() - ref.loss) <= 1e-5 * ref.loss, tag


def test_static_scratch_matches_workspace_entry_on_two_calls_the_second_smaller():
    ulsnn.static_scratch_init()
    shape = si.MlpShape(100, 130, 259, True)              # general path: five products, split-k partials
    assert ulsnn.mlp_grad_workspace_bytes(100, 130, 259, 3000) <= ulsnn.static_scratch_bytes()
    _check(_case(shape, 5, 3000), "100-130-259 B=3000")
    _check(_case(shape, 6, 37), "100-130-259 B=37 after the larger call")
    _check(_case(si.MLP_SMALL, 0, 256), "64-32-10 B=256 (small-network path)")
    _check(_case(si.MLP_SMALL, 1, 16), "64-32-10 B=16 after the larger call")


def test_static_scratch_refuses_what_does_not_fit_and_accumulates():
    W1, W2, _, _, X, y = (None if t is None else t.to(DEV) for t in _case(si.MLP_JOCR, 2, 64))
    assert ulsnn.mlp_grad_workspace_bytes(400, 480, 3203, 64) > ulsnn.static_scratch_bytes()
    with pytest.raises(ulsnn.UlsnnError) as e:
        ulsnn.mlp_grad_static(W1, W2, X, y)
    assert e.value.status == 5
    p = [None if t is None else t.to(DEV) for t in _case(si.MlpShape(20, 12, 9, True), 7, 64)]
    W1, W2, b1, b2, X, y = p
    out = ulsnn.mlp_grad_static(W1, W2, X[:40], y[:40], b1, b2)
    ulsnn.mlp_grad_static(W1, W2, X[40:], y[40:], b1, b2, out=out, accumulate=True)
    whole = ulsnn.mlp_grad(W1, W2, X, y, b1, b2)
    torch.cuda.synchronize()
    for name in ("dW1", "dW2", "db1", "db2", "loss"):
        assert torch.allclose(getattr(out, name), getattr(whole, name), rtol=1e-5, atol=1e-6), name
