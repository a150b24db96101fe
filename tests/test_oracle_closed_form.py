"""Pins of the CPU oracle against closed forms and rule scenes (no GPU).

Single on-axis Gaussian: every step of cull/project/blend collapses to a formula one can write by hand
(paper Sec. 2.1 pipeline; thresholds per the benchmark contract: clamp 0.99, skip < 1/255, stop T < 1e-4).
"""
import math

import numpy as np
import pytest

import oracle
from helpers import one_point_scene, simple_camera, splat_state

W = H = 64
F = 50.0
ZC = 4.0


def _single(s=(0.4, 0.4, 0.4), logit=0.3, rgb=(0.9, 0.5, 0.2), quat=(1, 0, 0, 0), mean=(0, 0, 0)):
    scene = one_point_scene(mean, np.log(s), quat, logit, rgb=rgb)
    cam = simple_camera(W, H, F, ZC)
    return scene, cam


def test_head_on_axis_aligned_covariance_and_conic():
    s = (0.4, 0.25, 0.7)
    scene, cam = _single(s=s)
    sp = oracle.preprocess(scene, cam)
    va = (F * s[0] / ZC) ** 2 + 0.3
    vc = (F * s[1] / ZC) ** 2 + 0.3
    assert sp["radius"][0] > 0
    np.testing.assert_allclose(sp["cov2d"][0], [va, 0.0, vc], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(sp["conic"][0], [1 / va, 0.0, 1 / vc], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(sp["mean2d"][0], [W / 2, H / 2], atol=1e-12)
    np.testing.assert_allclose(sp["depth"][0], ZC, atol=1e-14)
    np.testing.assert_allclose(sp["opacity"][0], 1 / (1 + math.exp(-0.3)), rtol=1e-14)
    np.testing.assert_allclose(sp["color"][0], [0.9, 0.5, 0.2], rtol=1e-12)
    # extent: 3 sigma of the larger eigenvalue, discriminant floored at 0.1
    m = 0.5 * (va + vc)
    lam = m + math.sqrt(max(0.1, m * m - va * vc))
    assert sp["radius"][0] == math.ceil(3 * math.sqrt(lam))


def test_isotropic_rotation_irrelevant():
    a, _ = _single(quat=(1, 0, 0, 0))
    b, cam = _single(quat=(0.3, -0.7, 0.2, 0.9))
    sa, sb = oracle.preprocess(a, cam), oracle.preprocess(b, cam)
    np.testing.assert_allclose(sa["cov2d"], sb["cov2d"], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("logit,bg", [(0.3, (0.0, 0.0, 0.0)), (-1.0, (0.2, 0.7, 0.4)), (6.0, (1.0, 1.0, 1.0))])
def test_single_gaussian_image_closed_form(logit, bg):
    rgb = np.array([0.9, 0.5, 0.2])
    scene, cam = _single(s=(0.9, 0.9, 0.9), logit=logit, rgb=rgb)
    out = oracle.forward(scene, cam, bg, splat_dtype=np.float64)
    var = (F * 0.9 / ZC) ** 2 + 0.3
    o = 1 / (1 + math.exp(-logit))
    assert out["splats"]["radius"][0] >= 32  # the splat's tile rectangle covers the whole 64x64 image
    ys, xs = np.mgrid[0:H, 0:W]
    d2 = (xs + 0.5 - W / 2) ** 2 + (ys + 0.5 - H / 2) ** 2
    alpha = np.minimum(0.99, o * np.exp(-d2 / (2 * var)))
    alpha = np.where(alpha < 1 / 255, 0.0, alpha)
    img = alpha[..., None] * rgb + (1 - alpha)[..., None] * np.asarray(bg)
    np.testing.assert_allclose(out["image"], img, rtol=0, atol=1e-13)
    np.testing.assert_allclose(out["final_T"], 1 - alpha, rtol=0, atol=1e-13)
    assert np.array_equal(out["last_idx"], (alpha > 0).astype(np.uint32))
    if logit == 6.0:
        assert (alpha == 0.99).sum() > 0  # the clamp is exercised


def test_single_gaussian_gradients_by_hand():
    s = np.array([0.9, 0.7, 0.5])
    rgb = np.array([0.9, 0.5, 0.2]); bg = np.array([0.1, 0.2, 0.3]); logit = -0.4
    scene, cam = _single(s=s, logit=logit, rgb=rgb)
    rng = np.random.default_rng(5)
    G = rng.normal(size=(H, W, 3))
    fwd = oracle.forward(scene, cam, bg, splat_dtype=np.float64)
    g = oracle.backward(scene, cam, bg, fwd, G)
    o = 1 / (1 + math.exp(-logit))
    va = (F * s[0] / ZC) ** 2 + 0.3; vc = (F * s[1] / ZC) ** 2 + 0.3
    ys, xs = np.mgrid[0:H, 0:W]
    dx = xs + 0.5 - W / 2; dy = ys + 0.5 - H / 2
    gauss = np.exp(-dx * dx / (2 * va) - dy * dy / (2 * vc))
    alpha = o * gauss
    assert alpha.max() < 0.99
    live = alpha >= 1 / 255
    # tile rectangle: the splat reaches every tile here
    assert fwd["splats"]["rect"][0].tolist() == [0, 0, 4, 4]
    A = np.where(live, (G * (rgb - bg)).sum(-1), 0.0)          # dL/dalpha per pixel
    np.testing.assert_allclose(g["logit"][0], (A * gauss).sum() * o * (1 - o), rtol=1e-11)
    dc = (np.where(live, alpha, 0.0)[..., None] * G).sum((0, 1))
    np.testing.assert_allclose(g["sh"][0, 0], dc * 0.28209479177387814, rtol=1e-11)
    ux = (F * s[0] / ZC) ** 2; uy = (F * s[1] / ZC) ** 2
    np.testing.assert_allclose(g["log_scale"][0, 0], (A * alpha * dx * dx * ux / va ** 2).sum(), rtol=1e-10)
    np.testing.assert_allclose(g["log_scale"][0, 1], (A * alpha * dy * dy * uy / vc ** 2).sum(), rtol=1e-10)
    assert abs(g["log_scale"][0, 2]) < 1e-12 * abs(g["log_scale"][0, 0])
    np.testing.assert_allclose(g["mean"][0, 0], (A * alpha * dx / va).sum() * F / ZC, rtol=1e-10)
    np.testing.assert_allclose(g["mean"][0, 1], (A * alpha * dy / vc).sum() * F / ZC, rtol=1e-10)
    # depth: only the footprint shrinks (the centre stays on the axis)
    dva = -2 * ux / ZC; dvc = -2 * uy / ZC
    gz = (A * alpha * (dx * dx / (2 * va ** 2) * dva + dy * dy / (2 * vc ** 2) * dvc)).sum()
    np.testing.assert_allclose(g["mean"][0, 2], gz, rtol=1e-10)


# ---------------------------------------------------------------- rule scenes on hand-made splat states
def _render_state(st, depth, w=16, h=16, bg=(0, 0, 0)):
    lists = oracle.bin_sort(st["mean2d"], st["radius"], np.asarray(depth, dtype=np.float32), w, h)
    return oracle.render_fwd(st, lists, w, h, bg), lists


def test_alpha_clamp_is_099():
    st = splat_state([[8.5, 8.5]], [[0.05, 0.0, 0.05]], [1.0], [[1.0, 1.0, 1.0]], [8])
    out, _ = _render_state(st, [1.0])
    assert out["final_T"][8, 8] == 1.0 - 0.99
    assert out["image"][8, 8, 0] == 0.99
    assert out["last_idx"][8, 8] == 1


def test_skip_below_1_over_255():
    for o, blended in [(1 / 255 - 1e-9, False), (1 / 255 + 1e-9, True)]:
        st = splat_state([[8.5, 8.5]], [[0.05, 0.0, 0.05]], [o], [[1.0, 1.0, 1.0]], [8])
        out, _ = _render_state(st, [1.0])
        assert (out["last_idx"][8, 8] == 1) == blended
        assert (out["final_T"][8, 8] < 1.0) == blended
        assert out["fragile"][8, 8] & 1  # and the oracle knows this pixel sits on the threshold


def test_stop_before_transmittance_below_1e4():
    k = 20
    st = splat_state([[8.5, 8.5]] * k, [[0.05, 0.0, 0.05]] * k, [0.5] * k, [[0.8, 0.4, 0.2]] * k, [8] * k)
    out, _ = _render_state(st, np.arange(1, k + 1, dtype=np.float32))
    assert out["last_idx"][8, 8] == 13                 # 0.5^13 = 1.22e-4 kept, 0.5^14 = 6.1e-5 would stop
    assert out["final_T"][8, 8] == 0.5 ** 13
    np.testing.assert_allclose(out["image"][8, 8], np.array([0.8, 0.4, 0.2]) * (1 - 0.5 ** 13), rtol=1e-14)
    assert (out["final_T"] >= 1e-4).all()


def test_negative_exponent_is_skipped():
    st = splat_state([[8.5, 8.5]], [[-0.05, 0.0, -0.05]], [0.5], [[1.0, 1.0, 1.0]], [8])
    out, _ = _render_state(st, [1.0])
    assert out["last_idx"][3, 3] == 0 and out["final_T"][3, 3] == 1.0
    assert out["last_idx"][8, 8] == 1   # sigma == 0 exactly at the centre is not negative


def test_depth_order_front_to_back():
    # two opaque-ish splats at the same pixel; the nearer one must dominate, whatever the index order
    for depths in ([1.0, 2.0], [2.0, 1.0]):
        st = splat_state([[8.5, 8.5]] * 2, [[0.05, 0.0, 0.05]] * 2, [0.9, 0.9], [[1, 0, 0], [0, 1, 0]], [8, 8])
        out, lists = _render_state(st, depths)
        near = int(np.argmin(depths))
        assert lists["vals"].tolist() == [near, 1 - near]
        exp = np.zeros(3); exp[near] = 0.9; exp[1 - near] = 0.9 * 0.1
        np.testing.assert_allclose(out["image"][8, 8], exp, rtol=1e-14)


def test_near_far_and_radius_clip_cull():
    scene, cam = _single()
    assert oracle.preprocess(scene, dict(cam, near=5.0))["radius"][0] == 0
    assert oracle.preprocess(scene, dict(cam, far=3.0))["radius"][0] == 0
    r = oracle.preprocess(scene, cam)["radius"][0]
    assert oracle.preprocess(scene, dict(cam, radius_clip=float(r)))["radius"][0] == 0
    assert oracle.preprocess(scene, dict(cam, radius_clip=float(r) - 1))["radius"][0] == r
    # a splat wholly off-screen is culled
    off, _ = _single(mean=(40.0, 0, 0))
    assert oracle.preprocess(off, cam)["radius"][0] == 0


def test_skip_flag_covers_float32_evaluations_of_alpha():
    """The width of the 'within rounding of the 1/255 threshold' flag is derived from fp32 arithmetic (about 1e-6 of
    relative error from log / exp / product, 2.5e-7 per unit of sigma's terms, doubled). Here: one splat per tile, its
    opacity chosen so that one pixel of the tile lands within a few 1e-6 (relative) of the threshold; alpha of that
    pixel is then evaluated in float32 in two ways (o exp(-sigma), and 2^(log2 o - sigma log2 e) with pre-scaled conic).
    Wherever either float32 decision differs from the oracle's, the oracle must have flagged the pixel; and the flag
    must not be so wide that it swallows samples 1e-4 away."""
    rng = np.random.default_rng(5)
    tx = ty = 64
    w, h = 16 * tx, 16 * ty
    n = tx * ty
    cx = (np.arange(n) % tx) * 16 + rng.uniform(2, 14, n)
    cy = (np.arange(n) // tx) * 16 + rng.uniform(2, 14, n)
    a = rng.uniform(0.02, 0.6, n); c = rng.uniform(0.02, 0.6, n); b = rng.uniform(-0.9, 0.9, n) * np.sqrt(a * c)
    px = (np.arange(n) % tx) * 16 + rng.integers(0, 16, n) + 0.5
    py = (np.arange(n) // tx) * 16 + rng.integers(0, 16, n) + 0.5
    mean2d = np.stack([cx, cy], 1).astype(np.float32).astype(np.float64)
    conic = np.stack([a, b, c], 1).astype(np.float32).astype(np.float64)
    dx, dy = px - mean2d[:, 0], py - mean2d[:, 1]
    sigma = 0.5 * (conic[:, 0] * dx * dx + conic[:, 2] * dy * dy) + conic[:, 1] * dx * dy
    keep = sigma < 5.0                                     # so that the opacity below stays under 1
    delta = rng.uniform(-4e-6, 4e-6, n)
    delta[::7] = rng.choice([-1e-4, 1e-4], len(delta[::7]))   # some samples clearly off the threshold
    o = np.where(keep, np.exp(sigma) / 255.0 * (1.0 + delta), 0.5).astype(np.float32).astype(np.float64)
    st = splat_state(mean2d, conic, o, np.ones((n, 3)), np.full(n, 7))
    # the radius keeps every splat inside its own tile's 3 x 3 neighbourhood; only the designated pixel is looked at
    lists = oracle.bin_sort(st["mean2d"], st["radius"], np.ones(n, dtype=np.float32), w, h)
    out = oracle.render_fwd(st, lists, w, h, (0, 0, 0))
    iy, ix = (py - 0.5).astype(int), (px - 0.5).astype(int)
    # float32 evaluations (this test's own restatement of the blend rule of Sec. 2.1 in single precision)
    f = np.float32
    m32, q32, o32 = mean2d.astype(f), conic.astype(f), o.astype(f)
    dx32, dy32 = px.astype(f) - m32[:, 0], py.astype(f) - m32[:, 1]
    s32 = f(0.5) * (q32[:, 0] * dx32 * dx32 + q32[:, 2] * dy32 * dy32) + q32[:, 1] * dx32 * dy32
    alpha_a = np.minimum(f(0.99), o32 * np.exp(-s32))
    l2e = f(1.4426950408889634)
    A, Bq, Cq = f(0.5) * l2e * q32[:, 0], l2e * q32[:, 1], f(0.5) * l2e * q32[:, 2]
    alpha_b = np.minimum(f(0.99), np.exp2(np.log2(o32) - ((A * dx32 + Bq * dy32) * dx32 + Cq * dy32 * dy32)))
    thr = f(1.0 / 255.0)
    # the designated pixel sees only its own tile's splats; its own is the one whose index is the tile's
    alpha64 = np.minimum(0.99, o * np.exp(-sigma))
    dec64 = alpha64 >= 1.0 / 255.0
    flagged = (out["fragile"][iy, ix] & 1) != 0
    differs = keep & (((alpha_a >= thr) != dec64) | ((alpha_b >= thr) != dec64))
    assert differs.sum() > 20                               # the sample does reach the knife edge
    assert flagged[differs].all()
    far = keep & (np.abs(delta) > 5e-5)
    alone = np.array([(lists["ranges"][t, 1] - lists["ranges"][t, 0]) == 1 for t in range(n)])
    assert far.sum() > 100 and not flagged[far & alone].any()
