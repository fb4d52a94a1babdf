"""Parity of the widened entry points against the CPU oracle:
  * ulsnn_mlp_loss       error-only evaluation (forward + loss), fp32 and bf16 operands
  * ulsnn_mlp_grad_mse   the paper's own output stage: tanh outputs, summed squared error, dense targets (fp32 and
                         bf16 operands)
  * ulsnn_mlp_mse        its error-only form
Bars as for ulsnn_mlp_grad: gradients relative L2 <= 1e-4, loss relative 1e-5 (bf16 operands: 1e-2).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_1911_05181_amd as ulsnn
import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rel(a, b):
    return np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b)


def _dev(t):
    return None if t is None else t.to(DEV)


def _np(t):
    return None if t is None else t.float().numpy()


@pytest.mark.parametrize("shape,batch", [(si.MLP_SMALL, 256), (si.MlpShape(100, 130, 259, True), 300),
                                         (si.MLP_JOCR, 4096), (si.MlpShape(64, 32, 4500, False), 37)])
def test_loss_only_fp32(shape, batch):
    W1, W2, b1, b2 = si.mlp_weights(shape, 2)
    if shape.biases:
        b1, b2 = si.random_biases(shape, 2, 0.2)
    X, y = si.mlp_patterns(shape, 2, 0, batch)
    want = oracle.mlp_loss(_np(W1), _np(W2), _np(X), y.numpy(), _np(b1), _np(b2))
    got = ulsnn.mlp_loss(_dev(W1), _dev(W2), _dev(X), _dev(y), _dev(b1), _dev(b2))
    torch.cuda.synchronize()
    assert abs(got.item() - want) <= 1e-5 * want
    # the gradient call reports the same loss, bit for bit (same kernels, same order)
    full = ulsnn.mlp_grad(_dev(W1), _dev(W2), _dev(X), _dev(y), _dev(b1), _dev(b2))
    torch.cuda.synchronize()
    assert torch.equal(full.loss, got)
    # accumulate adds
    ulsnn.mlp_loss(_dev(W1), _dev(W2), _dev(X), _dev(y), _dev(b1), _dev(b2), loss=got, accumulate=True)
    torch.cuda.synchronize()
    assert abs(got.item() - 2 * want) <= 2e-5 * want


def test_loss_only_bf16():
    shape = si.MLP_JOCR
    W1, W2, _, _ = si.mlp_weights(shape, 2)
    X, y = si.mlp_patterns(shape, 2, 0, 1000)
    W1, W2, X = (t.to(torch.bfloat16) for t in (W1, W2, X))
    want = oracle.mlp_loss(_np(W1), _np(W2), _np(X), y.numpy())
    got = ulsnn.mlp_loss(_dev(W1), _dev(W2), _dev(X), _dev(y))
    torch.cuda.synchronize()
    assert abs(got.item() - want) <= 1e-2 * want
    print(f"bf16 loss-only rel err {abs(got.item() - want) / want:.2e}")


def _mse_problem(shape, seed, batch):
    W1, W2, b1, b2 = si.mlp_weights(shape, seed)
    if shape.biases:
        b1, b2 = si.random_biases(shape, seed, 0.2)
    X, _ = si.mlp_patterns(shape, seed, 0, batch)
    T = si.mlp_targets(shape, seed, 0, batch)
    return W1, W2, b1, b2, X, T


@pytest.mark.parametrize("shape,batch", [(si.MLP_SMALL, 256), (si.MlpShape(100, 130, 259, True), 300),
                                         (si.MlpShape(17, 33, 5, True), 1), (si.MLP_JOCR, 2048),
                                         (si.MlpShape(128, 64, 40, False), 1000),    # small-network path, two launches
                                         (si.MLP_SMALL, 4097)])                      # one pattern too many for it
def test_mse_gradient(shape, batch):
    W1, W2, b1, b2, X, T = _mse_problem(shape, 2, batch)
    ref = oracle.mlp_grad_mse(_np(W1), _np(W2), _np(X), _np(T), _np(b1), _np(b2))
    res = ulsnn.mlp_grad_mse(_dev(W1), _dev(W2), _dev(X), _dev(T), _dev(b1), _dev(b2))
    torch.cuda.synchronize()
    worst = 0.0
    for name in ("dW1", "dW2", "db1", "db2"):
        r = getattr(ref, name)
        if r is None:
            continue
        e = _rel(getattr(res, name).cpu().numpy(), r)
        worst = max(worst, e)
        assert e <= 1e-4, (name, e)
    le = abs(res.loss.item() - ref.loss) / ref.loss
    assert le <= 1e-5
    print(f"mse {shape.n_in}-{shape.n_hid}-{shape.n_out} B={batch}: worst gradient rel-L2 {worst:.2e}, loss rel {le:.2e}")
    only = ulsnn.mlp_mse(_dev(W1), _dev(W2), _dev(X), _dev(T), _dev(b1), _dev(b2))
    torch.cuda.synchronize()
    assert torch.equal(only, res.loss)
    # a second call adding to the first: twice the gradient (and, on the small-network path, a ticket counter
    # that the first call left at zero)
    ulsnn.mlp_grad_mse(_dev(W1), _dev(W2), _dev(X), _dev(T), _dev(b1), _dev(b2), out=res, accumulate=True)
    torch.cuda.synchronize()
    assert _rel(res.dW2.cpu().numpy(), 2 * ref.dW2) <= 1e-4 and abs(res.loss.item() - 2 * ref.loss) <= 2e-5 * ref.loss


def test_mse_matches_the_papers_matrix_identities():
    """grad_ho = Y_Delta^T * H and grad_ih = H_Delta^T * X of section 4.2 (paper layout, no biases) = -1/2 of the
    returned derivatives, transposed; evaluated here in float64 from the same fp32 inputs."""
    shape = si.MlpShape(40, 24, 11, False)
    W1, W2, _, _, X, T = _mse_problem(shape, 5, 90)
    res = ulsnn.mlp_grad_mse(_dev(W1), _dev(W2), _dev(X), _dev(T))
    torch.cuda.synchronize()
    W_ih, W_ho, Xd, Td = W1.double().T, W2.double().T, X.double(), T.double()
    H = torch.tanh(Xd @ W_ih.T)
    Y = torch.tanh(H @ W_ho.T)
    Y_delta = (1 - Y * Y) * (Td - Y)
    H_delta = (1 - H * H) * (Y_delta @ W_ho)
    grad_ih, grad_ho = H_delta.T @ Xd, Y_delta.T @ H
    assert _rel(res.dW1.cpu().numpy(), (-2 * grad_ih.T).numpy()) < 1e-5
    assert _rel(res.dW2.cpu().numpy(), (-2 * grad_ho.T).numpy()) < 1e-5


@pytest.mark.parametrize("shape,batch", [(si.MLP_SMALL, 256), (si.MlpShape(100, 130, 259, True), 300),
                                         (si.MlpShape(104, 136, 264, False), 700), (si.MLP_JOCR, 2048),
                                         (si.MLP_SMALL, 70_000)])
def test_mse_gradient_bf16_operands(shape, batch):
    """The squared-error form with X, W1, W2 stored as bf16 (rounded once on the host; the oracle gets exactly those
    values and runs in double).  H, the output delta and the hidden delta are kept in bf16 by the library, the
    error is summed from the fp32 outputs before anything is rounded.  Bar: 1e-2, as for the softmax form."""
    W1, W2, b1, b2, X, T = _mse_problem(shape, 2, batch)
    W1, W2, X = W1.bfloat16(), W2.bfloat16(), X.bfloat16()
    ref = oracle.mlp_grad_mse(_np(W1), _np(W2), _np(X), _np(T), _np(b1), _np(b2))
    res = ulsnn.mlp_grad_mse(_dev(W1), _dev(W2), _dev(X), _dev(T), _dev(b1), _dev(b2))
    torch.cuda.synchronize()
    worst = 0.0
    for name in ("dW1", "dW2", "db1", "db2"):
        r = getattr(ref, name)
        if r is None:
            continue
        assert getattr(res, name).dtype == torch.float32
        e = _rel(getattr(res, name).cpu().numpy(), r)
        worst = max(worst, e)
        assert e <= 1e-2, (name, e)
    le = abs(res.loss.item() - ref.loss) / ref.loss
    assert le <= 1e-2
    print(f"bf16 mse {shape.n_in}-{shape.n_hid}-{shape.n_out} B={batch}: worst gradient rel-L2 {worst:.2e}, loss rel {le:.2e}")
    only = ulsnn.mlp_mse(_dev(W1), _dev(W2), _dev(X), _dev(T), _dev(b1), _dev(b2))
    torch.cuda.synchronize()
    assert abs(only.item() - ref.loss) <= 1e-2 * ref.loss and abs(only.item() - res.loss.item()) <= 1e-6 * ref.loss
    again = ulsnn.mlp_grad_mse(_dev(W1), _dev(W2), _dev(X), _dev(T), _dev(b1), _dev(b2))
    torch.cuda.synchronize()
    assert torch.equal(again.dW1, res.dW1) and torch.equal(again.dW2, res.dW2) and torch.equal(again.loss, res.loss)
