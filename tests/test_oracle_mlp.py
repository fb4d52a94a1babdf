"""Pins for the CPU MLP-gradient oracle.

None of these re-types the oracle's loops:
  * central finite differences of the loss for every parameter of tiny nets (ties backward to forward)
  * torch's float64 autograd of tanh / cross_entropy(reduction="sum") (a library routine; ties forward and
    backward to an independent implementation)
  * closed forms: W2 = 0 gives P = 1/n_out and loss = B ln n_out; W1 = 0 gives H = 0 and dW2 = 0
  * the one-pattern textbook case written as outer products
  * invariants: softmax rows sum to 1, dO rows sum to 0, db2 sums to 0
  * additivity over patterns (paper section 4.3), invariance under a permutation of the batch
  * a pattern with a label outside [0, n_out) is ignored
"""
import math

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


def _net(n_in, n_hid, n_out, batch, seed, biases=True, wscale=1.0):
    shape = si.MlpShape(n_in, n_hid, n_out, biases)
    W1, W2, _, _ = si.mlp_weights(shape, seed)
    X, y = si.mlp_patterns(shape, seed, 0, batch)
    b1 = b2 = None
    if biases:
        b1, b2 = si.random_biases(shape, seed, 0.3)
        b1, b2 = b1.numpy().astype(np.float64), b2.numpy().astype(np.float64)
    return ((W1.numpy() * wscale).astype(np.float64), (W2.numpy() * wscale).astype(np.float64), b1, b2,
            X.numpy().astype(np.float64), y.numpy())


@pytest.mark.parametrize("n_in,n_hid,n_out,batch,biases", [(5, 4, 3, 7, True), (3, 2, 2, 1, True),
                                                          (6, 5, 4, 9, False)])
def test_finite_differences(n_in, n_hid, n_out, batch, biases):
    W1, W2, b1, b2, X, y = _net(n_in, n_hid, n_out, batch, 21, biases, wscale=1.5)
    g = oracle.mlp_grad(W1, W2, X, y, b1, b2)
    h = 1e-5
    params = [("dW1", W1), ("dW2", W2)] + ([("db1", b1), ("db2", b2)] if biases else [])
    for name, P in params:
        G = getattr(g, name)
        flat = P.reshape(-1)
        for idx in range(flat.size):
            old = flat[idx]
            flat[idx] = old + h
            lp = oracle.mlp_loss(W1, W2, X, y, b1, b2)
            flat[idx] = old - h
            lm = oracle.mlp_loss(W1, W2, X, y, b1, b2)
            flat[idx] = old
            fd = (lp - lm) / (2 * h)
            an = G.reshape(-1)[idx]
            assert abs(fd - an) <= 1e-7 * (1 + abs(an)), (name, idx, fd, an)


def _torch_grad(W1, W2, b1, b2, X, y):
    t = lambda a: None if a is None else torch.tensor(a, dtype=torch.float64, requires_grad=True)
    W1t, W2t, b1t, b2t = t(W1), t(W2), t(b1), t(b2)
    Xt = torch.tensor(X, dtype=torch.float64)
    A1 = Xt @ W1t
    if b1t is not None:
        A1 = A1 + b1t
    H = torch.tanh(A1)
    Z = H @ W2t
    if b2t is not None:
        Z = Z + b2t
    loss = torch.nn.functional.cross_entropy(Z, torch.tensor(y, dtype=torch.int64), reduction="sum")
    loss.backward()
    g = lambda a: None if a is None else a.grad.numpy()
    return loss.item(), g(W1t), g(W2t), g(b1t), g(b2t), H.detach().numpy(), torch.softmax(Z, 1).detach().numpy()


@pytest.mark.parametrize("n_in,n_hid,n_out,batch,biases", [(64, 32, 10, 256, True), (37, 19, 53, 41, False),
                                                          (400, 48, 331, 33, True)])
def test_against_torch_autograd_float64(n_in, n_hid, n_out, batch, biases):
    W1, W2, b1, b2, X, y = _net(n_in, n_hid, n_out, batch, 4, biases)
    g = oracle.mlp_grad(W1, W2, X, y, b1, b2, intermediates=True)
    loss, dW1, dW2, db1, db2, H, P = _torch_grad(W1, W2, b1, b2, X, y)
    rel = lambda a, b: np.linalg.norm(a - b) / np.linalg.norm(b)
    assert abs(g.loss - loss) <= 1e-12 * abs(loss)
    assert rel(g.dW1, dW1) < 1e-12 and rel(g.dW2, dW2) < 1e-12
    assert rel(g.H, H) < 1e-13 and rel(g.P, P) < 1e-12
    if biases:
        assert rel(g.db1, db1) < 1e-12 and rel(g.db2, db2) < 1e-12
    assert abs(oracle.mlp_loss(W1, W2, X, y, b1, b2) - loss) <= 1e-12 * abs(loss)


def test_closed_form_zero_output_weights():
    n_in, n_hid, n_out, batch = 64, 32, 10, 256
    W1, W2, b1, b2, X, y = _net(n_in, n_hid, n_out, batch, 0, biases=False)
    W2[:] = 0.0
    g = oracle.mlp_grad(W1, W2, X, y, intermediates=True)
    assert abs(g.loss - batch * math.log(n_out)) < 1e-10          # = 256 * 2.302585...
    assert np.allclose(g.P, 1.0 / n_out, rtol=0, atol=1e-15)
    assert np.array_equal(g.dW1, np.zeros_like(g.dW1))            # dH = dO * 0
    onehot = np.eye(n_out)[y]
    assert np.allclose(g.dW2, g.H.T @ (1.0 / n_out - onehot), rtol=1e-13, atol=1e-13)


def test_closed_form_zero_input_weights():
    n_in, n_hid, n_out, batch = 12, 8, 3203, 5
    W1, W2, _, _, X, y = _net(n_in, n_hid, n_out, batch, 1, biases=False)
    W1[:] = 0.0
    g = oracle.mlp_grad(W1, W2, X, y, intermediates=True)
    assert abs(g.loss - batch * math.log(n_out)) < 1e-10          # H = 0 -> Z = 0; ln 3203 = 8.0718...
    assert abs(math.log(3203) - 8.071843) < 1e-6
    assert np.array_equal(g.H, np.zeros_like(g.H)) and np.array_equal(g.dW2, np.zeros_like(g.dW2))
    dO = 1.0 / n_out - np.eye(n_out)[y]
    assert np.allclose(g.dW1, X.T @ (dO @ W2.T), rtol=1e-12, atol=1e-15)     # tanh'(0) = 1


def test_single_pattern_textbook():
    """B = 1: dW2 = h (p - e_y)^T and dW1 = x ((W2 (p - e_y)) * (1 - h^2))^T with hand-set numbers."""
    W1 = np.array([[0.5, -1.0], [0.25, 2.0], [-0.75, 0.5]])
    W2 = np.array([[1.0, -1.0, 0.5], [0.0, 2.0, -0.5]])
    b1 = np.array([0.1, -0.2])
    b2 = np.array([0.0, 0.3, -0.3])
    x = np.array([[1.0, 2.0, -1.0]])
    y = np.array([2])
    a = np.array([0.5 + 0.5 + 0.75 + 0.1, -1.0 + 4.0 - 0.5 - 0.2])      # = [1.85, 2.3]
    h = np.tanh(a)
    z = np.array([h[0] + 0.0, -h[0] + 2 * h[1] + 0.3, 0.5 * h[0] - 0.5 * h[1] - 0.3])
    p = np.exp(z) / np.exp(z).sum()
    d = p - np.array([0.0, 0.0, 1.0])
    g = oracle.mlp_grad(W1, W2, x, y, b1, b2)
    assert abs(g.loss + math.log(p[2])) < 1e-14
    assert np.allclose(g.dW2, np.outer(h, d), rtol=1e-13, atol=1e-15)
    assert np.allclose(g.db2, d, rtol=1e-13, atol=1e-15)
    da = (W2 @ d) * (1 - h * h)
    assert np.allclose(g.dW1, np.outer(x[0], da), rtol=1e-13, atol=1e-15)
    assert np.allclose(g.db1, da, rtol=1e-13, atol=1e-15)


def test_invariants_and_float32_form():
    W1, W2, b1, b2, X, y = _net(64, 32, 10, 256, 0, biases=True)
    for dtype, tol in [(np.float64, 1e-14), (np.float32, 2e-6)]:
        g = oracle.mlp_grad(W1, W2, X, y, b1, b2, dtype=dtype, intermediates=True)
        assert np.abs(g.P.sum(axis=1) - 1).max() < tol * 10
        assert (g.P >= 0).all() and (g.P <= 1).all() and g.loss >= 0
        assert np.abs(g.dO.sum(axis=1)).max() < tol * 10
        assert abs(g.db2.sum()) < tol * 1000
        assert np.allclose(g.db2, g.dO.sum(axis=0), rtol=0, atol=tol * 300)
        assert np.abs(g.H).max() < 1
    g64 = oracle.mlp_grad(W1, W2, X, y, b1, b2)
    g32 = oracle.mlp_grad(W1, W2, X, y, b1, b2, dtype=np.float32)
    rel = lambda a, b: np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b)
    assert rel(g32.dW1, g64.dW1) < 1e-5 and rel(g32.dW2, g64.dW2) < 1e-5
    assert abs(g32.loss - g64.loss) < 1e-5 * g64.loss
    assert rel(g32.dW1, g64.dW1) > 0        # the two forms really are different arithmetic


def test_additive_and_permutation_invariant():
    W1, W2, b1, b2, X, y = _net(20, 12, 17, 50, 8, biases=True)
    g = oracle.mlp_grad(W1, W2, X, y, b1, b2)
    ga = oracle.mlp_grad(W1, W2, X[:19], y[:19], b1, b2)
    gb = oracle.mlp_grad(W1, W2, X[19:], y[19:], b1, b2)
    for name in ("dW1", "dW2", "db1", "db2"):
        assert np.allclose(getattr(ga, name) + getattr(gb, name), getattr(g, name), rtol=1e-12, atol=1e-13)
    assert abs(ga.loss + gb.loss - g.loss) < 1e-11
    perm = np.random.default_rng(0).permutation(50)
    gp = oracle.mlp_grad(W1, W2, X[perm], y[perm], b1, b2)
    for name in ("dW1", "dW2", "db1", "db2"):
        assert np.allclose(getattr(gp, name), getattr(g, name), rtol=1e-12, atol=1e-13)


def test_out_of_range_label_is_ignored():
    W1, W2, b1, b2, X, y = _net(10, 6, 5, 12, 3, biases=True)
    y2 = y.copy()
    y2[[2, 7]] = [-1, 5]
    keep = np.ones(12, bool)
    keep[[2, 7]] = False
    g = oracle.mlp_grad(W1, W2, X, y2, b1, b2)
    gk = oracle.mlp_grad(W1, W2, X[keep], y[keep], b1, b2)
    for name in ("dW1", "dW2", "db1", "db2"):
        assert np.allclose(getattr(g, name), getattr(gk, name), rtol=1e-12, atol=1e-14)
    assert abs(g.loss - gk.loss) < 1e-12
    assert abs(oracle.mlp_loss(W1, W2, X, y2, b1, b2) - gk.loss) < 1e-12


def test_empty_batch():
    W1, W2, b1, b2, X, y = _net(4, 3, 2, 1, 3, biases=True)
    g = oracle.mlp_grad(W1, W2, X[:0], y[:0], b1, b2)
    assert g.loss == 0 and not g.dW1.any() and not g.dW2.any() and not g.db1.any() and not g.db2.any()


def test_float32_loss_only_form():
    """The float build of the error-only function: inside float rounding of the double one and of the closed form
    B ln n_out (W2 = 0), equal to the loss the float gradient function reports (same steps, same order), ignores
    out-of-range labels, and is not the double arithmetic under another name."""
    W1, W2, b1, b2, X, y = _net(64, 32, 10, 256, 0, biases=True)
    l64 = oracle.mlp_loss(W1, W2, X, y, b1, b2)
    l32 = oracle.mlp_loss(W1, W2, X, y, b1, b2, dtype=np.float32)
    assert 0 < abs(l32 - l64) < 2e-6 * l64
    assert l32 == oracle.mlp_grad(W1, W2, X, y, b1, b2, dtype=np.float32).loss
    flat = oracle.mlp_loss(W1, np.zeros_like(W2), X, y, dtype=np.float32)
    assert abs(flat - 256 * math.log(10)) < 2e-6 * 256 * math.log(10)
    y2 = y.copy()
    y2[::2] = -3
    kept = oracle.mlp_loss(W1, W2, X[1::2], y[1::2], b1, b2, dtype=np.float32)
    assert abs(oracle.mlp_loss(W1, W2, X, y2, b1, b2, dtype=np.float32) - kept) < 1e-9 * kept
    assert oracle.mlp_loss(W1, W2, X[:0], y[:0], b1, b2, dtype=np.float32) == 0.0
