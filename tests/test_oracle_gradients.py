"""Finite-difference pins of the oracle's analytic backward (Alg. 1 lines 17-18 and 22-24), no GPU.

L(theta) = sum(G * image(theta)) for a fixed random G. Central differences in fp64 over every parameter of every
point; a sample is dropped when any discrete decision (visibility, extent, tile lists, last blended index, clamp
state) differs between theta-eps and theta+eps, since the derivative is defined with those decisions frozen.
"""
import numpy as np
import pytest

import oracle
from helpers import to_f64
from paper_2512_20017_amd import synth

BG = np.array([0.2, 0.5, 0.3])


def _loss_and_decisions(sc, cam, G):
    f = oracle.forward(sc, cam, BG, splat_dtype=np.float64)
    sig = (f["splats"]["radius"].tobytes(), f["lists"]["vals"].tobytes(), f["lists"]["ranges"].tobytes(),
           f["last_idx"].tobytes(), (f["splats"]["color"] > 0).tobytes())
    return float((f["image"] * G).sum()), sig, f


def _fd_check(sc, cam, seed, eps=1e-6, rtol=2e-5, min_checked=0.7):
    W, H = cam["width"], cam["height"]
    G = np.random.default_rng(seed).normal(size=(H, W, 3))
    L0, sig0, f0 = _loss_and_decisions(sc, cam, G)
    g = oracle.backward(sc, cam, BG, f0, G)
    assert (f0["fragile"] == 0).all()
    checked = total = 0
    for name in ("mean", "log_scale", "quat", "logit", "sh"):
        a = sc[name]
        scale = max(np.abs(g[name]).max(), 1e-12)
        for idx in np.ndindex(a.shape):
            total += 1
            old = a[idx]
            a[idx] = old + eps; Lp, sp, _ = _loss_and_decisions(sc, cam, G)
            a[idx] = old - eps; Lm, sm, _ = _loss_and_decisions(sc, cam, G)
            a[idx] = old
            if sp != sig0 or sm != sig0:
                continue
            checked += 1
            fd = (Lp - Lm) / (2 * eps)
            assert abs(fd - g[name][idx]) <= rtol * scale + 1e-9, (name, idx, fd, g[name][idx])
    assert checked >= min_checked * total, (checked, total)
    return g, f0


@pytest.mark.parametrize("seed,deg", [(0, 3), (1, 2), (2, 0)])
def test_finite_differences_random_scene(seed, deg):
    sc = to_f64(synth.random_small_scene(seed, 10, deg))
    cam = synth.pinhole(32, 32, 50.0, np.eye(3), [0.03, -0.04, 2.2])
    g, f = _fd_check(sc, cam, seed)
    assert (f["splats"]["radius"] > 0).sum() >= 8
    assert f["n_blend"] > 500
    for k in ("mean", "log_scale", "quat", "logit", "sh"):
        assert np.abs(g[k]).max() > 0


def test_finite_differences_rotated_offcentre_camera():
    sc = to_f64(synth.random_small_scene(7, 8, 1))
    R, t = synth.look_at([1.5, 0.8, -1.6], [0.1, 0.0, 0.0], [0.0, 1.0, 0.0])
    cam = synth.pinhole(48, 32, 45.0, R, t)
    cam["cx"] += 1.7; cam["cy"] -= 0.9; cam["fy"] *= 1.1
    _fd_check(sc, cam, 11)


def test_finite_differences_with_alpha_clamp_and_colour_clamp():
    """Opaque, overlapping splats (alpha saturates at 0.99 on many pixels) and dark colours (the max(0,.) clamp
    is active on some channels): both must pass zero gradient where active."""
    sc = to_f64(synth.random_small_scene(3, 6, 1, spread=0.3, ls_mu=-1.6))
    sc["logit"][:] = 7.0
    sc["sh"][:3, 0, :] = -2.5      # 0.5 + 0.282*(-2.5) < 0  -> clamped to 0
    cam = synth.pinhole(32, 32, 50.0, np.eye(3), [0.0, 0.0, 2.0])
    g, f = _fd_check(sc, cam, 5, min_checked=0.5)
    assert (f["splats"]["color"][:3] == 0).any()
    assert (f["state"]["opacity"] > 0.99).all()   # every splat saturates alpha around its centre
    # where the DC colour is clamped its gradient is exactly zero
    for i in range(3):
        for c in range(3):
            if f["splats"]["color"][i, c] == 0:
                assert (g["sh"][i, :, c] == 0).all()


def test_finite_differences_in_guard_band():
    """A big splat whose centre is outside 1.3 x half-FoV horizontally: the clamped slope passes no gradient."""
    cam = synth.pinhole(32, 32, 60.0, np.eye(3), [0.0, 0.0, 0.0])
    lim = 1.3 * 16 / cam["fx"]
    sc = dict(mean=np.array([[1.6 * lim * 3.0, 0.2, 3.0], [0.1, 0.1, 2.5]]), log_scale=np.log([[1.4, 0.9, 1.1], [0.3, 0.2, 0.25]]),
              quat=np.array([[0.9, 0.1, -0.3, 0.2], [1.0, 0.2, 0.1, 0.0]]), logit=np.array([0.5, 0.0]),
              sh=np.random.default_rng(0).normal(0, 0.5, size=(2, 4, 3)), sh_degree=1)
    g, f = _fd_check(sc, cam, 9, min_checked=0.9)
    assert f["splats"]["radius"][0] > 0 and f["n_blend"] > 100


def test_gradients_accumulate():
    sc = to_f64(synth.random_small_scene(4, 6, 1))
    cam = synth.pinhole(32, 32, 50.0, np.eye(3), [0.0, 0.0, 2.2])
    G = np.random.default_rng(0).normal(size=(32, 32, 3))
    f = oracle.forward(sc, cam, BG)
    once = oracle.backward(sc, cam, BG, f, G)
    acc = oracle.preprocess_bwd(sc, cam, once["d_splats"])
    acc = oracle.preprocess_bwd(sc, cam, once["d_splats"], accumulate_into=acc)
    for k in ("mean", "log_scale", "quat", "logit", "sh"):
        np.testing.assert_allclose(acc[k], 2 * once[k], rtol=1e-14)
