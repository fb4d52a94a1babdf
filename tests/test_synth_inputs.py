"""The seeded input generator: reproducible, sliceable, and with the stated distributions."""
import math

import numpy as np
import torch

import synth_inputs as si


def test_slices_match_whole_stream():
    whole = si.normal(2, si.T_X, 1000)
    part = si.normal(2, si.T_X, 300, start=450)
    assert torch.equal(whole[450:750], part)
    X, y = si.mlp_patterns(si.MLP_JOCR, 2, 0, 12)
    X2, y2 = si.mlp_patterns(si.MLP_JOCR, 2, 5, 4)
    assert torch.equal(X[5:9], X2) and torch.equal(y[5:9], y2)


def test_seeds_and_tensors_differ():
    a = si.uniform(1, si.T_A, 64)
    assert not torch.equal(a, si.uniform(2, si.T_A, 64))
    assert not torch.equal(a, si.uniform(1, si.T_B, 64))
    assert torch.equal(a, si.uniform(1, si.T_A, 64))


def test_distributions():
    n = 400_000
    x = si.normal(0, si.T_X, n).double().numpy()
    assert abs(x.mean()) < 4 / math.sqrt(n) and abs(x.var() - 1) < 0.01
    assert abs((np.abs(x) > 1.959964).mean() - 0.05) < 0.002
    u = si.uniform(1, si.T_A, n).double().numpy()
    assert u.min() >= -1 and u.max() <= 1 and abs(u.mean()) < 0.005 and abs(u.var() - 1 / 3) < 0.005
    lab = si.integers(2, si.T_LABELS, n, 0, 3203).numpy()
    assert lab.min() == 0 and lab.max() == 3202
    counts = np.bincount(lab, minlength=3203)
    assert abs(counts.mean() - n / 3203) < 1e-9 and counts.std() < 2 * math.sqrt(n / 3203)
    W1, W2, b1, b2 = si.mlp_weights(si.MLP_JOCR, 2)
    assert W1.shape == (400, 480) and W2.shape == (480, 3203) and b1 is None and b2 is None
    assert abs(W1.double().var().item() - 1 / 400) < 1e-4 and abs(W2.double().var().item() - 1 / 480) < 2e-5
    _, _, b1, b2 = si.mlp_weights(si.MLP_SMALL, 0)
    assert b1.shape == (32,) and b2.shape == (10,) and not b1.any() and not b2.any()


def test_small_integers():
    m = si.small_integers(3, si.T_A, 50, 60, bound=8)
    assert m.dtype == torch.float32 and m.abs().max() <= 8 and torch.equal(m, m.round())
    e = si.small_integers(3, si.T_C, 50, 60, bound=8, even=True)
    assert torch.equal(e / 2, (e / 2).round())
