"""Pins of the SGD oracle (Alg. 1 step 10; momentum and weight decay of Table 1): a two-step example worked by
hand, the library optimiser with the same reading of the update, and closed forms of its special cases."""

import numpy as np
import pytest
import torch

from oracle import sgd as osgd


def test_two_steps_worked_by_hand():
    # lr 0.1, momentum 0.9, weight decay 0.01, V0 = 0
    w0 = np.array([1.0, -2.0, 0.5])
    dw1 = np.array([0.5, 0.25, -1.0])
    dw2 = np.array([-0.2, 0.4, 0.1])
    # step 1: g = dW + 0.01 W = [0.51, 0.23, -0.995]; V1 = g; W1 = W0 - 0.1 V1
    w1, v1 = osgd.sgd_step(w0, np.zeros(3), dw1, 0.1, 0.9, 0.01)
    np.testing.assert_allclose(v1, [0.51, 0.23, -0.995], rtol=0, atol=1e-15)
    np.testing.assert_allclose(w1, [0.949, -2.023, 0.5995], rtol=0, atol=1e-15)
    # step 2: g = dW + 0.01 W1 = [-0.19051, 0.37977, 0.105995]; V2 = 0.9 V1 + g; W2 = W1 - 0.1 V2
    w2, v2 = osgd.sgd_step(w1, v1, dw2, 0.1, 0.9, 0.01)
    np.testing.assert_allclose(v2, [0.26849, 0.58677, -0.789505], rtol=0, atol=1e-15)
    np.testing.assert_allclose(w2, [0.922151, -2.081677, 0.6784505], rtol=0, atol=1e-15)


@pytest.mark.parametrize("momentum,wd", [(0.9, 1e-4), (0.0, 0.0), (0.5, 0.1)])
def test_matches_library_optimiser(momentum, wd):
    rng = np.random.default_rng(5)
    w = rng.standard_normal(257)
    p = torch.nn.Parameter(torch.tensor(w, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=0.05, momentum=momentum, weight_decay=wd)
    v = np.zeros_like(w)
    for step in range(4):
        dw = rng.standard_normal(257)
        p.grad = torch.tensor(dw, dtype=torch.float64)
        opt.step()
        w, v = osgd.sgd_step(w, v, dw, 0.05, momentum, wd)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-13, atol=1e-14)


def test_special_cases_closed_forms():
    rng = np.random.default_rng(6)
    w0 = rng.standard_normal(100)
    dw = rng.standard_normal(100)
    # no momentum, no decay: plain gradient descent
    w1, v1 = osgd.sgd_step(w0, np.zeros(100), dw, 0.3, 0.0, 0.0)
    np.testing.assert_allclose(w1, w0 - 0.3 * dw, rtol=1e-15)
    np.testing.assert_allclose(v1, dw, rtol=0, atol=0)
    # zero gradient, no momentum: pure decay, W_t = W_0 (1 - lr wd)^t
    w, v = w0, np.zeros(100)
    for _ in range(5):
        w, v = osgd.sgd_step(w, v, np.zeros(100), 0.1, 0.0, 0.2)
    np.testing.assert_allclose(w, w0 * (1 - 0.1 * 0.2) ** 5, rtol=1e-14)
    # constant gradient, no decay: velocity is the geometric series g (1 + m + ... + m^(t-1))
    w, v = w0, np.zeros(100)
    for _ in range(6):
        w, v = osgd.sgd_step(w, v, dw, 0.01, 0.9, 0.0)
    np.testing.assert_allclose(v, dw * (1 - 0.9 ** 6) / (1 - 0.9), rtol=1e-13)
    # the decay enters the velocity: decaying the weights beside the momentum (decoupled decay) agrees for one
    # step from V = 0 and differs from the second step on
    wa, va = osgd.sgd_step(w0, np.zeros(100), dw, 0.1, 0.9, 0.5)
    np.testing.assert_allclose(wa, w0 - 0.1 * dw - 0.1 * 0.5 * w0, rtol=1e-14)
    wb, _ = osgd.sgd_step(wa, va, dw, 0.1, 0.9, 0.5)
    w_decoupled = wa - 0.1 * (0.9 * dw + dw) - 0.1 * 0.5 * wa
    assert np.max(np.abs(wb - w_decoupled)) > 1e-3


def test_abs_sum_is_the_l1_norm():
    rng = np.random.default_rng(7)
    w = rng.standard_normal(1000).astype(np.float32)
    assert osgd.abs_sum(w) == pytest.approx(float(np.linalg.norm(w.astype(np.float64), 1)), rel=1e-14)
    assert osgd.abs_sum(np.array([-1.5, 2.0, -0.25])) == 3.75
