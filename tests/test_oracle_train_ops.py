"""Pins for the oracle's loss and optimizer step (Alg. 1 lines 13, 16, 27) -- no GPU.

L1: a hand-computed example, finite differences, scale. Selective Adam: closed forms (first step, constant gradient),
the library's Adam when every point is visible, untouched rows for invisible points, and a planted-mistake check.
"""
import numpy as np
import pytest
import torch

import oracle


def test_l1_hand_example_and_finite_differences():
    img = np.array([[[1.0, 2.0, 0.5]]]); tgt = np.array([[[2.0, 0.0, 0.5]]])
    loss, g = oracle.l1_loss(img, tgt)
    assert loss == pytest.approx((1.0 + 2.0 + 0.0) / 3.0, abs=1e-15)
    assert np.array_equal(g, np.array([[[-1.0, 1.0, 0.0]]]) / 3.0)
    rng = np.random.default_rng(0)
    a = rng.uniform(size=(5, 7, 3)); b = rng.uniform(size=(5, 7, 3))
    loss, g = oracle.l1_loss(a, b)
    h = 1e-6
    for idx in [(0, 0, 0), (2, 3, 1), (4, 6, 2)]:
        ap = a.copy(); ap[idx] += h
        am = a.copy(); am[idx] -= h
        fd = (oracle.l1_loss(ap, b)[0] - oracle.l1_loss(am, b)[0]) / (2 * h)
        assert fd == pytest.approx(g[idx], abs=1e-9)
    assert np.abs(g).sum() == pytest.approx(1.0, abs=1e-12)     # every pixel differs: |dL| sums to one


def test_adam_first_step_and_constant_gradient_closed_forms():
    rng = np.random.default_rng(1)
    n = 6
    p0 = rng.normal(size=(n, 3)); g = rng.normal(size=(n, 3))
    vis = np.ones(n, dtype=np.uint8)
    lr, b1, b2, eps = 1e-2, 0.9, 0.999, 1e-8
    p, m, v = oracle.adam_selective(p0, g, np.zeros_like(p0), np.zeros_like(p0), vis, lr, b1, b2, eps, 1)
    np.testing.assert_allclose(p, p0 - lr * g / (np.abs(g) + eps), rtol=1e-12)
    np.testing.assert_allclose(m, (1 - b1) * g, rtol=1e-15); np.testing.assert_allclose(v, (1 - b2) * g * g, rtol=1e-15)
    # constant gradient: bias-corrected moments stay (g, g^2), so every step moves by lr g / (|g| + eps)
    for t in range(2, 8):
        p, m, v = oracle.adam_selective(p, g, m, v, vis, lr, b1, b2, eps, t)
    np.testing.assert_allclose(p, p0 - 7 * lr * g / (np.abs(g) + eps), rtol=1e-10)


def test_adam_matches_library_when_all_visible_and_skips_invisible_rows():
    rng = np.random.default_rng(2)
    n = 16
    p0 = rng.normal(size=(n, 4)); lr, b1, b2, eps = 3e-3, 0.85, 0.99, 1e-6
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tp], lr=lr, betas=(b1, b2), eps=eps)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for t in range(1, 6):
        g = rng.normal(size=(n, 4))
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = oracle.adam_selective(p, g, m, v, np.ones(n), lr, b1, b2, eps, t)
    np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-10, atol=1e-13)
    # selective: invisible rows keep parameter and both moments bit for bit, visible rows move as before
    vis = (np.arange(n) % 3 == 0).astype(np.uint8)
    g = rng.normal(size=(n, 4))
    p2, m2, v2 = oracle.adam_selective(p, g, m, v, vis, lr, b1, b2, eps, 6)
    pa, ma, va = oracle.adam_selective(p, g, m, v, np.ones(n), lr, b1, b2, eps, 6)
    hid = vis == 0
    assert np.array_equal(p2[hid], p[hid]) and np.array_equal(m2[hid], m[hid]) and np.array_equal(v2[hid], v[hid])
    assert np.array_equal(p2[~hid], pa[~hid]) and np.array_equal(m2[~hid], ma[~hid]) and np.array_equal(v2[~hid], va[~hid])
    # a step with the moments decayed for invisible rows (plain Adam with zero gradient) is a different thing
    pz, mz, vz = oracle.adam_selective(p, np.where(hid[:, None], 0.0, g), m, v, np.ones(n), lr, b1, b2, eps, 6)
    assert not np.allclose(pz[hid], p[hid])
