"""Parity of the optimiser-step entry points (section 4.2, last paragraph) against the numpy / C oracle:
ulsnn_dot, ulsnn_axpy, ulsnn_cg_direction, ulsnn_mlp_line_search, and a few conjugate-gradient iterations built
from them."""
import numpy as np
import pytest
import torch

import oracle
from oracle import ref_cg
import paper_1911_05181_amd as ulsnn
import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("n", [1, 63, 257, 70_001, 1_729_440])
def test_dot_axpy_direction(n):
    x = si.normal(7, si.T_A, n).to(DEV)
    y = si.normal(7, si.T_B, n).to(DEV)
    d = si.normal(7, si.T_C, n).to(DEV)
    xd, yd, dd = (t.cpu().numpy().astype(np.float64) for t in (x, y, d))
    got = ulsnn.dot(x, y)
    torch.cuda.synchronize()
    S = np.abs(xd * yd).sum()
    assert abs(got.item() - xd @ yd) <= 1e-6 * S            # double accumulation, one rounding to fp32
    again = ulsnn.dot(x, y)
    torch.cuda.synchronize()
    assert torch.equal(got, again)                          # fixed summation order
    # Polak-Ribiere: x = new gradient, y = old gradient
    want_d, want_beta = ref_cg.cg_direction(xd, yd, dd)
    d2, beta = ulsnn.cg_direction(x, y, d.clone())
    torch.cuda.synchronize()
    assert abs(beta.item() - want_beta) <= 1e-5 * max(abs(want_beta), 1e-3)
    assert np.abs(d2.cpu().numpy() - want_d).max() <= 1e-5 * np.abs(want_d).max()
    # first direction: -g, whatever d held
    d3, beta0 = ulsnn.cg_direction(x, None, torch.full_like(d, float("nan")))
    torch.cuda.synchronize()
    assert beta0.item() == 0.0 and torch.equal(d3, -x)
    # plain gradient step W := W - alpha grad E
    w = y.clone()
    ulsnn.axpy(-0.125, x, w)
    torch.cuda.synchronize()
    assert np.array_equal(w.cpu().numpy(), (yd.astype(np.float32) - np.float32(0.125) * xd.astype(np.float32)))


def test_beta_is_zero_when_the_old_gradient_is_zero():
    g = torch.ones(1000, device=DEV)
    d, beta = ulsnn.cg_direction(g, torch.zeros_like(g), torch.ones_like(g))
    torch.cuda.synchronize()
    assert beta.item() == 0.0 and torch.equal(d, -g)


def _problem(shape, seed, batch):
    W1, W2, _, _ = si.mlp_weights(shape, seed)
    X, y = si.mlp_patterns(shape, seed, 0, batch)
    return W1, W2, X, y


@pytest.mark.parametrize("shape,batch,bracket,alpha0", [(si.MlpShape(64, 32, 10, False), 256, 64, 1e-4),
                                                        (si.MlpShape(64, 32, 10, False), 256, 256, 0.05),
                                                        (si.MlpShape(64, 32, 10, False), 256, 256, 0.5),   # overshoots: step 0
                                                        (si.MlpShape(100, 130, 259, False), 300, 100, 1e-3),
                                                        (si.MLP_JOCR, 2048, 256, 1e-4)])
def test_line_search_against_the_oracle(shape, batch, bracket, alpha0):
    W1, W2, X, y = _problem(shape, 2, batch)
    g = oracle.mlp_grad(W1.numpy(), W2.numpy(), X.numpy(), y.numpy())        # direction from the oracle's gradient
    d1 = torch.from_numpy((-g.dW1).astype(np.float32))
    d2 = torch.from_numpy((-g.dW2).astype(np.float32))
    want, V1, V2 = ref_cg.mlp_line_search(W1.numpy(), W2.numpy(), d1.numpy(), d2.numpy(), X.numpy(), y.numpy(), bracket,
                                          alpha0, 30)
    gW1, gW2 = W1.to(DEV), W2.to(DEV)
    res = ulsnn.mlp_line_search(gW1, gW2, d1.to(DEV), d2.to(DEV), X.to(DEV), y.to(DEV), bracket, alpha0, 30)
    torch.cuda.synchronize()
    print(f"{shape.n_in}-{shape.n_hid}-{shape.n_out} B={batch}: alpha {res.alpha:.6g} (oracle {want.alpha:.6g}), "
          f"E {res.loss0:.6g} -> {res.loss:.6g} (oracle {want.loss:.6g}), bracket [{res.bracket_lo:.4g}, {res.bracket_hi:.4g}], "
          f"{res.error_evaluations} error + {res.gradient_evaluations} gradient evaluations")
    # the bracket is decided by signs: identical.  The vertex divides small differences of fp32 errors.
    assert res.bracket_lo == np.float32(want.lo) and res.bracket_hi == np.float32(want.hi)
    assert (res.error_evaluations, res.gradient_evaluations) == (want.error_evaluations, want.gradient_evaluations)
    assert abs(res.loss0 - want.loss0) <= 1e-5 * want.loss0
    assert abs(res.alpha - want.alpha) <= 2e-3 * want.alpha
    assert abs(res.loss - want.loss) <= 1e-5 * want.loss
    assert res.loss <= res.loss0
    # weights were updated in place with the step reported
    assert np.abs(gW1.cpu().numpy() - (W1.numpy() + np.float32(res.alpha) * d1.numpy())).max() <= 1e-6
    assert np.abs(gW2.cpu().numpy() - (W2.numpy() + np.float32(res.alpha) * d2.numpy())).max() <= 1e-6
    # and the error there is what the oracle computes at those weights
    e = oracle.mlp_loss(gW1.cpu().numpy(), gW2.cpu().numpy(), X.numpy(), y.numpy())
    assert abs(res.loss - e) <= 1e-5 * e


def test_three_conjugate_gradient_iterations_follow_the_oracle():
    shape, batch, bracket = si.MlpShape(64, 32, 10, False), 256, 128
    W1, W2, X, y = _problem(shape, 4, batch)
    # oracle trajectory, float64
    o1, o2 = W1.numpy().astype(np.float64), W2.numpy().astype(np.float64)
    og_old = od = None
    # library trajectory
    g1, g2, gX, gy = W1.to(DEV), W2.to(DEV), X.to(DEV), y.to(DEV)
    n1 = g1.numel()
    grad = torch.empty(n1 + g2.numel(), device=DEV)
    grad_old = torch.empty_like(grad)
    d = torch.empty_like(grad)
    out = ulsnn.MlpGradResult(grad[:n1].view_as(g1), grad[n1:].view_as(g2), torch.empty(1, device=DEV))
    losses = []
    for it in range(3):
        og = oracle.mlp_grad(o1, o2, X.numpy(), y.numpy())
        ogv = np.concatenate([og.dW1.ravel(), og.dW2.ravel()])
        od, obeta = ref_cg.cg_direction(ogv, og_old, od)
        orr, o1, o2 = ref_cg.mlp_line_search(o1, o2, od[:n1].reshape(o1.shape), od[n1:].reshape(o2.shape), X.numpy(),
                                             y.numpy(), bracket, 1e-3, 30)
        og_old = ogv

        ulsnn.mlp_grad(g1, g2, gX, gy, out=out)
        _, beta = ulsnn.cg_direction(grad, grad_old if it else None, d)
        res = ulsnn.mlp_line_search(g1, g2, d[:n1].view_as(g1), d[n1:].view_as(g2), gX, gy, bracket, 1e-3, 30)
        grad_old.copy_(grad)
        torch.cuda.synchronize()
        losses.append((res.loss, orr.loss))
        assert abs(beta.item() - obeta) <= 1e-2 * max(abs(obeta), 1e-2), (it, beta.item(), obeta)
        assert abs(res.loss - orr.loss) <= 1e-3 * orr.loss, (it, losses)
    assert losses[2][0] < losses[1][0] < losses[0][0]
    print("CG losses (library, oracle):", losses)
