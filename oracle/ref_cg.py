"""CPU oracle for the optimiser step of section 4.2 (its last paragraph).  TEST INFRASTRUCTURE ONLY.

The paper names its ingredients without printing an algorithm: a plain gradient step `W := W - alpha grad E`,
the Polak-Ribiere conjugate-gradient rule for the search direction, and a line search made of an exponential
step-size scheme, a quadratic interpolation, and a bracketing test that needs only the SIGN of
`grad E . direction`, estimated on a few patterns.  The reading taken here (and, independently, by the library):

  direction:   beta = g_new.(g_new - g_old) / g_old.g_old  (Polak-Ribiere), d := -g_new + beta d;
               the first direction (no g_old) is -g_new; beta = 0 when g_old.g_old = 0.
  line search: E0 = E(W).  Steps alpha_k = alpha0 * 2**k, k = 0..max_doublings: the first k at which the slope
               sign( grad E_sub(W + alpha_k d) . d ) is >= 0 closes the bracket [lo, hi] = [alpha_(k-1) or 0,
               alpha_k]; if none is, the last two steps are taken as the bracket.  E is then evaluated at lo (E0 when lo = 0),
               mid = (lo + hi)/2 and hi; if the parabola through the three points is convex its vertex, clamped
               to the bracket, is evaluated as well; the step with the smallest E among those evaluated wins
               (ties: the earliest of lo, mid, hi, vertex).

Everything is float64 numpy written from the definitions; the functions take callables, so that the same code is
pinned on quadratics (where the interpolation is exact and conjugate gradients end in n steps) and then run on
the MLP oracle.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Optional

import numpy as np


def gradient_step(w: np.ndarray, g: np.ndarray, alpha: float) -> np.ndarray:
    """W := W - alpha grad E."""
    return w - alpha * g


def polak_ribiere_beta(g_new: np.ndarray, g_old: np.ndarray) -> float:
    den = float(np.dot(g_old.ravel(), g_old.ravel()))
    if den == 0.0:
        return 0.0
    return float(np.dot(g_new.ravel(), (g_new - g_old).ravel())) / den


def cg_direction(g_new: np.ndarray, g_old: Optional[np.ndarray], d: Optional[np.ndarray]):
    """Returns (new direction, beta)."""
    if g_old is None or d is None:
        return -g_new.astype(np.float64), 0.0
    beta = polak_ribiere_beta(g_new.astype(np.float64), g_old.astype(np.float64))
    return -g_new + beta * d, beta


@dataclass
class LineSearchResult:
    alpha: float
    loss: float
    loss0: float
    lo: float
    hi: float
    error_evaluations: int
    gradient_evaluations: int


def line_search(error: Callable[[float], float], slope: Callable[[float], float], alpha0: float,
                max_doublings: int) -> LineSearchResult:
    """`error(alpha)` = E(W + alpha d) on all patterns; `slope(alpha)` = grad E_sub(W + alpha d) . d."""
    assert alpha0 > 0 and max_doublings >= 0
    n_err = n_grad = 0
    e0 = error(0.0)
    n_err += 1
    lo, hi = 0.0, alpha0
    prev = 0.0
    for k in range(max_doublings + 1):
        hi = alpha0 * (2.0 ** k)
        lo = prev
        n_grad += 1
        if slope(hi) >= 0.0:
            break
        prev = hi
    mid = 0.5 * (lo + hi)
    if lo == 0.0:
        e_lo = e0
    else:
        e_lo = error(lo)
        n_err += 1
    e_mid, e_hi = error(mid), error(hi)
    n_err += 2
    cand = [(lo, e_lo), (mid, e_mid), (hi, e_hi)]
    curv = e_lo - 2.0 * e_mid + e_hi
    if curv > 0.0:
        h = 0.5 * (hi - lo)
        q = mid - h * (e_hi - e_lo) / (2.0 * curv)
        q = min(max(q, lo), hi)
        cand.append((q, error(q)))
        n_err += 1
    best = cand[0]
    for c in cand[1:]:
        if c[1] < best[1]:
            best = c
    return LineSearchResult(best[0], best[1], e0, lo, hi, n_err, n_grad)


def mlp_line_search(W1, W2, d1, d2, X, labels, bracket_batch: int, alpha0: float, max_doublings: int):
    """The line search on the softmax / cross-entropy MLP oracle (no biases).  Returns (result, W1', W2')."""
    from . import mlp_grad, mlp_loss   # the C oracle of the forward / backward passes
    W1, W2, d1, d2, X = (np.asarray(a, dtype=np.float64) for a in (W1, W2, d1, d2, X))
    labels = np.asarray(labels)
    nb = min(bracket_batch, X.shape[0])

    def error(alpha):
        return mlp_loss(W1 + alpha * d1, W2 + alpha * d2, X, labels)

    def slope(alpha):
        g = mlp_grad(W1 + alpha * d1, W2 + alpha * d2, X[:nb], labels[:nb])
        return float(np.dot(g.dW1.ravel(), d1.ravel()) + np.dot(g.dW2.ravel(), d2.ravel()))

    r = line_search(error, slope, alpha0, max_doublings)
    return r, W1 + r.alpha * d1, W2 + r.alpha * d2
