"""Pins of the oracle's training-side utilities: the density regulariser (Sec. 3.5, Eq. 4) against closed forms and
automatic differentiation, one-warning-shot pruning (Sec. 3.6) against hand-worked histories and its guarantees."""
import numpy as np
import pytest
import torch

import oracle


def _feats(rows, channels, nnz, rng):
    f = np.zeros(rows * channels, dtype=np.float32)
    f[rng.choice(rows * channels, size=nnz, replace=False)] = 1.0 + rng.random(nnz).astype(np.float32)
    return f.reshape(rows, channels)


def test_bias_closed_forms_of_eq4():
    rng = np.random.default_rng(0)
    w = np.array([0.5, -0.25, 0.0, 2.0], dtype=np.float32)
    n_sites, ch = 100, 4                      # 400 possible entries
    # rho = 0.25 > rho_up = 0.10: b = o + b1 * 0.15
    rho, b, reg, grad = oracle.density_regulariser(_feats(50, ch, 100, rng), n_sites, 0.10, 0.3, 2.0, 5.0, 0.01, w)
    assert rho == 0.25 and b == pytest.approx(0.3 + 2.0 * 0.15, rel=0, abs=1e-15)
    # hand: the pruned weight (exact 0) is left out of the sum and gets no gradient
    assert reg == pytest.approx(0.01 * ((0.5 + 0.6) ** 2 + (-0.25 + 0.6) ** 2 + (2.0 + 0.6) ** 2), rel=1e-14)
    assert grad.tolist() == pytest.approx([0.02 * 1.1, 0.02 * 0.35, 0.0, 0.02 * 2.6], rel=1e-14)
    # rho = 0.05 <= rho_up = 0.10: b = -b2 * 0.05, negative: drives weights up
    rho, b, reg, grad = oracle.density_regulariser(_feats(50, ch, 20, rng), n_sites, 0.10, 0.3, 2.0, 5.0, 0.01, w)
    assert rho == 0.05 and b == pytest.approx(-0.25, abs=1e-15) and b < 0
    # exactly at the bound the second case applies: b = 0, the plain L2 regulariser
    rho, b, reg, grad = oracle.density_regulariser(_feats(50, ch, 40, rng), n_sites, 0.10, 0.3, 2.0, 5.0, 0.01, w)
    assert rho == 0.10 and b == 0.0 and reg == pytest.approx(0.01 * float((w.astype(np.float64) ** 2).sum()), rel=1e-14)
    # just above the bound the extra penalty o appears: the bias jumps by o
    rho, b, _, _ = oracle.density_regulariser(_feats(50, ch, 41, rng), n_sites, 0.10, 0.3, 2.0, 5.0, 0.01, w)
    assert b == pytest.approx(0.3 + 2.0 * (41 / 400 - 0.10), abs=1e-15)


def test_gradient_equals_autograd_of_the_regulariser():
    rng = np.random.default_rng(1)
    w = rng.normal(size=(27, 3, 5)).astype(np.float32)
    w[rng.random(w.shape) < 0.3] = 0.0
    feats = _feats(200, 5, 333, rng)
    for rho_up in (0.05, 0.9):
        rho, b, reg, grad = oracle.density_regulariser(feats, 400, rho_up, 0.2, 1.5, 0.7, 0.003, w)
        wt = torch.tensor(w.astype(np.float64), requires_grad=True)
        mask = torch.tensor(w != 0)
        r = 0.003 * (((wt + b) ** 2) * mask).sum()
        r.backward()
        assert reg == pytest.approx(float(r.detach()), rel=1e-12)
        np.testing.assert_allclose(grad, wt.grad.numpy(), rtol=1e-12, atol=0)
        assert not grad[w == 0].any()
        # the sign of the bias follows the sign of (rho - rho_up)
        assert (b > 0) == (rho > rho_up)


def test_bias_is_monotone_in_density_and_linear_on_each_side():
    rng = np.random.default_rng(2)
    w = np.ones(3, dtype=np.float32)
    bs = []
    for nnz in range(0, 401, 40):
        _, b, _, _ = oracle.density_regulariser(_feats(100, 4, nnz, rng), 100, 0.5, 0.1, 2.0, 3.0, 1.0, w)
        bs.append(b)
    assert all(x < y for x, y in zip(bs, bs[1:]))
    below, above = bs[:6], bs[6:]                      # rho = 0 .. 0.5 | 0.6 .. 1.0
    assert np.allclose(np.diff(below), 3.0 * 0.1) and np.allclose(np.diff(above), 2.0 * 0.1)


def test_pruning_hand_worked_history():
    eps = 0.1
    # weight:        0: large  1: small twice  2: small, recovers, small again  3: already pruned  4: small from epoch 2
    w = np.array([1.0, 0.05, -0.02, 0.0, 0.5], dtype=np.float32)
    warned = np.zeros(5, dtype=np.uint8)
    w, warned, removed, left = oracle.prune_weights(w, warned, eps)        # epoch 1: warnings only
    assert w.tolist() == pytest.approx([1.0, 0.05, -0.02, 0.0, 0.5]) and warned.tolist() == [0, 1, 1, 0, 0]
    assert (removed, left) == (0, 4)
    w[2], w[4] = 0.7, 0.01                                                  # training moved two weights
    w, warned, removed, left = oracle.prune_weights(w, warned, eps)        # epoch 2
    assert w.tolist() == pytest.approx([1.0, 0.0, 0.7, 0.0, 0.01]) and warned.tolist() == [0, 0, 0, 0, 1]
    assert (removed, left) == (1, 3)
    w[2] = -0.03                                                            # small again, but its warning was reset
    w, warned, removed, left = oracle.prune_weights(w, warned, eps)        # epoch 3
    assert w.tolist() == pytest.approx([1.0, 0.0, -0.03, 0.0, 0.0]) and warned.tolist() == [0, 0, 1, 0, 0]
    assert (removed, left) == (1, 2)


def test_pruning_guarantees():
    rng = np.random.default_rng(3)
    w = rng.normal(scale=0.2, size=500).astype(np.float32)
    warned = np.zeros(500, dtype=np.uint8)
    nnz = [int(np.count_nonzero(w))]
    for epoch in range(6):
        before = w.copy()
        w, warned, removed, left = oracle.prune_weights(w, warned, 0.05)
        assert left == int(np.count_nonzero(w)) and removed == nnz[-1] - left
        assert not w[before == 0].any()                          # once zero, always zero
        assert np.array_equal(w[w != 0], before[w != 0])         # survivors are untouched
        assert not warned[w == 0].any()
        nnz.append(left)
        if epoch == 0:
            assert removed == 0                                  # never without a warning shot
        w = (w + (w != 0) * rng.normal(scale=0.02, size=500)).astype(np.float32)
    assert all(a >= b for a, b in zip(nnz, nnz[1:])) and nnz[-1] < nnz[0]
    # eps = 0 never prunes
    w2, warned2, removed, _ = oracle.prune_weights(w, np.ones(500, np.uint8), 0.0)
    assert removed == 0 and np.array_equal(w2, w)
