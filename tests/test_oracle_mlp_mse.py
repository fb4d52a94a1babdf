"""Pins for the oracle of the paper's own output stage (tanh outputs, summed squared error; sections 4.1-4.2).

  * the paper's matrix identities evaluated with numpy: Y_Delta = (1 - Y**Y)**(T - Y),
    H_Delta = (1 - H**H)**(Y_Delta * W_ho), grad_ih = H_Delta^T * X, grad_ho = Y_Delta^T * H, with
    W_ih = W1^T, W_ho = W2^T; the true gradient is -2 times them (transposed to this build's layout)
  * central finite differences of E for every parameter of tiny nets
  * torch float64 autograd of sum((tanh(tanh(X W1 + b1) W2 + b2) - T)^2)
  * closed forms: W2 = 0 gives Y = 0, E = sum T^2, dW1 = 0; T = Y gives E = 0 and zero gradients
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


def _net(n_in, n_hid, n_out, batch, seed, biases=True, wscale=1.0):
    shape = si.MlpShape(n_in, n_hid, n_out, biases)
    W1, W2, _, _ = si.mlp_weights(shape, seed)
    X, _ = si.mlp_patterns(shape, seed, 0, batch)
    T = si.mlp_targets(shape, seed, 0, batch)
    b1 = b2 = None
    if biases:
        b1, b2 = si.random_biases(shape, seed, 0.3)
        b1, b2 = b1.numpy().astype(np.float64), b2.numpy().astype(np.float64)
    return ((W1.numpy() * wscale).astype(np.float64), (W2.numpy() * wscale).astype(np.float64), b1, b2,
            X.numpy().astype(np.float64), T.numpy().astype(np.float64))


def test_paper_matrix_identities():
    """Section 4.2, with the paper's weight layout W_ih [n_h x n_i], W_ho [n_o x n_h] and no biases."""
    W1, W2, _, _, X, T = _net(20, 12, 7, 33, 3, biases=False, wscale=1.5)
    g = oracle.mlp_grad_mse(W1, W2, X, T, intermediates=True)
    W_ih, W_ho = W1.T, W2.T
    H = np.tanh(X @ W_ih.T)
    Y = np.tanh(H @ W_ho.T)
    Y_delta = (1 - Y * Y) * (T - Y)
    H_delta = (1 - H * H) * (Y_delta @ W_ho)
    grad_ih = H_delta.T @ X            # n_h x n_i, the paper's "gradient" w.r.t. W_ih
    grad_ho = Y_delta.T @ H            # n_o x n_h
    assert np.allclose(g.H, H, rtol=1e-13, atol=1e-15) and np.allclose(g.Y, Y, rtol=1e-13, atol=1e-15)
    assert abs(g.loss - ((Y - T) ** 2).sum()) < 1e-11 * g.loss              # eq. (error)
    assert np.allclose(g.dW1, -2 * grad_ih.T, rtol=1e-12, atol=1e-13)
    assert np.allclose(g.dW2, -2 * grad_ho.T, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("n_in,n_hid,n_out,batch,biases", [(5, 4, 3, 7, True), (3, 2, 2, 1, True), (6, 5, 4, 9, False)])
def test_finite_differences(n_in, n_hid, n_out, batch, biases):
    W1, W2, b1, b2, X, T = _net(n_in, n_hid, n_out, batch, 21, biases, wscale=1.5)
    g = oracle.mlp_grad_mse(W1, W2, X, T, b1, b2)
    h = 1e-5
    params = [("dW1", W1), ("dW2", W2)] + ([("db1", b1), ("db2", b2)] if biases else [])
    for name, P in params:
        G = getattr(g, name).reshape(-1)
        flat = P.reshape(-1)
        for idx in range(flat.size):
            old = flat[idx]
            flat[idx] = old + h
            lp = oracle.mlp_mse(W1, W2, X, T, b1, b2)
            flat[idx] = old - h
            lm = oracle.mlp_mse(W1, W2, X, T, b1, b2)
            flat[idx] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - G[idx]) <= 1e-7 * (1 + abs(G[idx])), (name, idx, fd, G[idx])


@pytest.mark.parametrize("n_in,n_hid,n_out,batch,biases", [(64, 32, 10, 256, True), (37, 19, 53, 41, False)])
def test_against_torch_autograd_float64(n_in, n_hid, n_out, batch, biases):
    W1, W2, b1, b2, X, T = _net(n_in, n_hid, n_out, batch, 4, biases)
    g = oracle.mlp_grad_mse(W1, W2, X, T, b1, b2)
    t = lambda a: None if a is None else torch.tensor(a, dtype=torch.float64, requires_grad=True)
    W1t, W2t, b1t, b2t = t(W1), t(W2), t(b1), t(b2)
    A1 = torch.tensor(X) @ W1t
    A1 = A1 + b1t if biases else A1
    Z = torch.tanh(A1) @ W2t
    Z = Z + b2t if biases else Z
    E = ((torch.tanh(Z) - torch.tensor(T)) ** 2).sum()
    E.backward()
    rel = lambda a, b: np.linalg.norm(a - b) / np.linalg.norm(b)
    assert abs(g.loss - E.item()) <= 1e-12 * E.item()
    assert rel(g.dW1, W1t.grad.numpy()) < 1e-12 and rel(g.dW2, W2t.grad.numpy()) < 1e-12
    if biases:
        assert rel(g.db1, b1t.grad.numpy()) < 1e-12 and rel(g.db2, b2t.grad.numpy()) < 1e-12
    assert abs(oracle.mlp_mse(W1, W2, X, T, b1, b2) - E.item()) <= 1e-12 * E.item()


def test_closed_forms_and_float32_form():
    W1, W2, _, _, X, T = _net(12, 8, 6, 20, 9, biases=False)
    g = oracle.mlp_grad_mse(W1, np.zeros_like(W2), X, T, intermediates=True)
    assert abs(g.loss - (T ** 2).sum()) < 1e-12 and not g.dW1.any()            # Y = 0
    assert np.allclose(g.dW2, g.H.T @ (-2 * T), rtol=1e-13, atol=1e-14)
    Y = oracle.mlp_grad_mse(W1, W2, X, T, intermediates=True).Y
    z = oracle.mlp_grad_mse(W1, W2, X, Y)                                      # targets = outputs
    assert z.loss == 0 and not z.dW1.any() and not z.dW2.any()
    g64 = oracle.mlp_grad_mse(W1, W2, X, T)
    g32 = oracle.mlp_grad_mse(W1, W2, X, T, dtype=np.float32)
    rel = lambda a, b: np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b)
    assert 0 < rel(g32.dW1, g64.dW1) < 1e-5 and rel(g32.dW2, g64.dW2) < 1e-5
    assert abs(g32.loss - g64.loss) < 1e-5 * g64.loss
    a = oracle.mlp_grad_mse(W1, W2, X[:8], T[:8])
    b = oracle.mlp_grad_mse(W1, W2, X[8:], T[8:])
    assert np.allclose(a.dW2 + b.dW2, g64.dW2, rtol=1e-12, atol=1e-13) and abs(a.loss + b.loss - g64.loss) < 1e-11


def test_float32_error_only_form():
    """The float build of the squared-error evaluation: inside float rounding of the double one and of the closed
    forms (W2 = 0 gives sum t^2; targets equal to the float outputs give exactly 0), equal to the error the float
    gradient function reports, and really float arithmetic."""
    W1, W2, b1, b2, X, T = _net(12, 8, 6, 20, 9, biases=True)
    e64 = oracle.mlp_mse(W1, W2, X, T, b1, b2)
    e32 = oracle.mlp_mse(W1, W2, X, T, b1, b2, dtype=np.float32)
    assert 0 < abs(e32 - e64) < 2e-6 * e64
    assert e32 == oracle.mlp_grad_mse(W1, W2, X, T, b1, b2, dtype=np.float32).loss
    t32 = T.astype(np.float32).astype(np.float64)
    flat = oracle.mlp_mse(W1, np.zeros_like(W2), X, T, dtype=np.float32)
    assert abs(flat - (t32 ** 2).sum()) < 2e-6 * (t32 ** 2).sum()
    Y32 = oracle.mlp_grad_mse(W1, W2, X, T, b1, b2, dtype=np.float32, intermediates=True).Y
    assert oracle.mlp_mse(W1, W2, X, Y32, b1, b2, dtype=np.float32) == 0.0
