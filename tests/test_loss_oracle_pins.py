"""Pins of the loss-backward oracle (Alg. 3) against things other than itself: autograd of the loss
it differentiates, the textbook cross-entropy gradient, invariants, closed forms, finite differences."""
import os
import sys

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from oracle.loss_oracle import logsoftmax_loss_bwd   # noqa: E402


def case(n, v, seed, per_element=False):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, 3, (n, v))
    p = rng.random((n, v)) ** 4
    p /= p.sum(1, keepdims=True)
    g = rng.normal(0, 1, (n, v) if per_element else (n,))
    return z, p, g


@pytest.mark.parametrize("per_element", [False, True])
def test_equals_autograd_of_the_weighted_soft_target_loss(per_element):
    z, p, g = case(5, 37, 1, per_element)
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    gt = torch.tensor(g, dtype=torch.float64)
    gt = gt if per_element else gt[:, None]
    loss = -(gt * torch.tensor(p) * torch.log_softmax(zt, dim=1)).sum()
    loss.backward()
    np.testing.assert_allclose(logsoftmax_loss_bwd(z, p, g), zt.grad.numpy(), rtol=1e-12, atol=1e-14)


def test_one_hot_target_gives_the_textbook_cross_entropy_gradient():
    rng = np.random.default_rng(2)
    z = rng.normal(0, 2, (4, 11))
    tgt = np.array([3, 0, 10, 7])
    p = np.eye(11)[tgt]
    ref = torch.autograd.functional.jacobian(
        lambda t: torch.nn.functional.cross_entropy(t, torch.tensor(tgt), reduction="sum"),
        torch.tensor(z, dtype=torch.float64)).numpy()
    np.testing.assert_allclose(logsoftmax_loss_bwd(z, p, np.ones(4)), ref, rtol=1e-12, atol=1e-14)
    soft = np.exp(z - z.max(1, keepdims=True))
    soft /= soft.sum(1, keepdims=True)
    np.testing.assert_allclose(logsoftmax_loss_bwd(z, p, np.ones(4)), soft - p, rtol=1e-12, atol=1e-14)


def test_rows_sum_to_zero_and_masked_rows_vanish():
    z, p, g = case(6, 29, 3)
    g[2] = 0.0
    out = logsoftmax_loss_bwd(z, p, g)
    np.testing.assert_allclose(out.sum(1), 0.0, atol=1e-14)
    assert np.all(out[2] == 0.0)


def test_shift_of_the_logits_changes_nothing_and_scaling_g_scales_the_result():
    z, p, g = case(3, 17, 4)
    base = logsoftmax_loss_bwd(z, p, g)
    np.testing.assert_allclose(logsoftmax_loss_bwd(z + 123.456, p, g), base, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(logsoftmax_loss_bwd(z, p, -2.5 * g), -2.5 * base, rtol=1e-12, atol=1e-14)


def test_uniform_logits_closed_form_with_unnormalised_target():
    v = 13
    p = np.arange(1, v + 1, dtype=np.float64)[None, :] / 7.0      # sums to 13, not 1
    g = np.array([0.5])
    out = logsoftmax_loss_bwd(np.full((1, v), 4.0), p, g)
    # element 7 is the difference of two equal terms of size 0.5: exact zero in the closed form, one
    # rounding of exp(log(1/13)) in the oracle, hence the absolute floor of a few ulps of 0.5
    np.testing.assert_allclose(out, -(p * 0.5 - (p.sum() * 0.5) / v), rtol=1e-13, atol=1e-15)


def test_central_finite_differences_of_the_loss():
    z, p, g = case(2, 9, 5)

    def loss(zz):
        m = zz.max(1, keepdims=True)
        logsm = zz - m - np.log(np.exp(zz - m).sum(1, keepdims=True))
        return -(g[:, None] * p * logsm).sum()

    out = logsoftmax_loss_bwd(z, p, g)
    h = 1e-6
    for r, c in [(0, 0), (0, 8), (1, 4)]:
        zp, zm = z.copy(), z.copy()
        zp[r, c] += h
        zm[r, c] -= h
        assert abs((loss(zp) - loss(zm)) / (2 * h) - out[r, c]) < 1e-8
