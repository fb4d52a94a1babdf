"""Pins of the optimiser-step oracle (oracle/ref_cg.py; section 4.2, last paragraph) against what mathematics
fixes: on a convex quadratic the three-point interpolation is exact, Polak-Ribiere equals Fletcher-Reeves, the
directions are conjugate and the minimum is reached in n steps."""
import numpy as np
import pytest

import oracle
from oracle import ref_cg
import synth_inputs as si


def _spd(n, seed):
    rng = np.random.default_rng(seed)
    M = rng.normal(size=(n, n))
    return M @ M.T + n * np.eye(n), rng.normal(size=n)


def test_gradient_step_closed_form():
    w, g = np.array([1.0, -2.0, 0.5]), np.array([0.5, 0.25, -1.0])
    assert np.array_equal(ref_cg.gradient_step(w, g, 0.5), np.array([0.75, -2.125, 1.0]))


def test_line_search_is_exact_on_a_quadratic():
    A, b = _spd(5, 0)
    w = np.zeros(5)
    g = A @ w - b
    d = -g
    exact = -(g @ d) / (d @ A @ d)
    E = lambda a: 0.5 * (w + a * d) @ A @ (w + a * d) - b @ (w + a * d)
    S = lambda a: (A @ (w + a * d) - b) @ d
    for alpha0 in (exact / 37.0, exact / 2.0, exact * 0.99, exact * 3.0, exact * 100.0):
        r = ref_cg.line_search(E, S, alpha0, 20)
        assert r.lo <= exact <= r.hi
        assert abs(r.alpha - exact) <= 1e-9 * exact
        assert abs(r.loss - E(exact)) <= 1e-9 * abs(E(exact))
        assert r.loss0 == E(0.0)
    # bracket found at the first step: lo = 0, three + one evaluations of the error, one of the gradient
    r = ref_cg.line_search(E, S, exact * 3.0, 20)
    assert (r.lo, r.hi, r.error_evaluations, r.gradient_evaluations) == (0.0, exact * 3.0, 4, 1)
    # bracket found after k doublings: k + 1 gradient signs, one more error evaluation (at lo > 0)
    r = ref_cg.line_search(E, S, exact / 5.0, 20)          # 1/5, 2/5, 4/5, 8/5 -> k = 3
    assert r.gradient_evaluations == 4 and r.error_evaluations == 5
    assert r.lo == pytest.approx(exact * 0.8) and r.hi == pytest.approx(exact * 1.6)


def test_line_search_without_a_bracket_and_without_convexity():
    # E(a) = -a: never turns upward: the last two steps are the bracket, the parabola is flat, hi wins
    r = ref_cg.line_search(lambda a: -a, lambda a: -1.0, 1.0, 3)
    assert (r.lo, r.hi, r.alpha, r.loss) == (4.0, 8.0, 8.0, -8.0)
    assert r.gradient_evaluations == 4 and r.error_evaluations == 4      # E(0), E(4), E(6), E(8); no vertex
    # concave along the line with the slope test positive at once: best of lo, mid, hi
    r = ref_cg.line_search(lambda a: -(a - 1.0) ** 2, lambda a: 1.0, 4.0, 3)
    assert r.alpha == 4.0 and r.error_evaluations == 3
    # max_doublings = 0
    r = ref_cg.line_search(lambda a: (a - 10.0) ** 2, lambda a: 2 * (a - 10.0), 1.0, 0)
    assert (r.lo, r.hi) == (0.0, 1.0) and r.alpha == 1.0


def test_polak_ribiere_on_a_quadratic_conjugacy_and_finite_termination():
    n = 7
    A, b = _spd(n, 1)
    w = np.zeros(n)
    g_old = d = None
    dirs = []
    for it in range(n):
        g = A @ w - b
        d, beta = ref_cg.cg_direction(g, g_old, d)
        if it == 0:
            assert beta == 0.0 and np.array_equal(d, -g)
        else:
            # exact line searches make successive gradients orthogonal: Polak-Ribiere = |g_new|^2 / |g_old|^2
            assert beta == pytest.approx((g @ g) / (g_old @ g_old), rel=1e-3)
        E = lambda a: 0.5 * (w + a * d) @ A @ (w + a * d) - b @ (w + a * d)
        S = lambda a: (A @ (w + a * d) - b) @ d
        r = ref_cg.line_search(E, S, 1e-3, 40)
        w = w + r.alpha * d
        dirs.append(d)
        g_old = g
    assert np.linalg.norm(A @ w - b) <= 1e-7 * np.linalg.norm(b)          # n steps reach the minimum
    D = np.array(dirs)
    C = D @ A @ D.T
    off = C - np.diag(np.diag(C))
    assert np.abs(off).max() <= 1e-6 * np.abs(np.diag(C)).max()            # A-conjugate directions


def test_beta_zero_when_old_gradient_vanishes():
    d, beta = ref_cg.cg_direction(np.ones(3), np.zeros(3), np.ones(3))
    assert beta == 0.0 and np.array_equal(d, -np.ones(3))


def test_mlp_line_search_picks_the_best_evaluated_step():
    shape = si.MlpShape(20, 12, 7, False)
    W1, W2, _, _ = si.mlp_weights(shape, 3)
    X, y = si.mlp_patterns(shape, 3, 0, 96)
    W1, W2, X, y = W1.numpy(), W2.numpy(), X.numpy(), y.numpy()
    g = oracle.mlp_grad(W1, W2, X, y)
    d1, d2 = -g.dW1, -g.dW2
    r, V1, V2 = ref_cg.mlp_line_search(W1, W2, d1, d2, X, y, 32, 1e-4, 30)
    assert r.loss0 == pytest.approx(oracle.mlp_loss(W1, W2, X, y))
    assert r.loss < r.loss0 and r.lo <= r.alpha <= r.hi and r.hi == pytest.approx(2 * r.lo)
    assert np.array_equal(V1, W1 + r.alpha * d1) and np.array_equal(V2, W2 + r.alpha * d2)
    assert oracle.mlp_loss(V1, V2, X, y) == pytest.approx(r.loss, rel=1e-12)
    # the slope on the 32 bracketing patterns changes sign inside [lo, hi]
    s = lambda a: (lambda q: float((q.dW1 * d1).sum() + (q.dW2 * d2).sum()))(
        oracle.mlp_grad(W1 + a * d1, W2 + a * d2, X[:32], y[:32]))
    assert s(r.lo) < 0 <= s(r.hi)
    # no evaluated candidate is better than the one returned
    for a in (r.lo, 0.5 * (r.lo + r.hi), r.hi):
        assert oracle.mlp_loss(W1 + a * d1, W2 + a * d2, X, y) >= r.loss
