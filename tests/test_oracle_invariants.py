"""Invariants the blending and projection must satisfy whatever the scene (no GPU).

White furnace / partition of unity, monotone transmittance, tile lists == their definition over the global
sorted list, rigid-motion invariance, permutation invariance, projection Jacobian as the push-forward of the
pinhole map, conic = inverse covariance.
"""
import numpy as np
import pytest
from scipy.spatial.transform import Rotation

import oracle
from helpers import to_f64
from paper_2512_20017_amd import synth


def _scene(seed, n=48, deg=0):
    sc = to_f64(synth.random_small_scene(seed, n, deg))
    cam = synth.pinhole(80, 56, 55.0, np.eye(3), [0.05, -0.02, 2.5])
    return sc, cam


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_white_furnace_partition_of_unity(seed):
    sc, cam = _scene(seed)
    f = oracle.forward(sc, cam, [1, 1, 1])
    st = dict(f["state"]); st["color"] = np.ones_like(st["color"])
    out = oracle.render_fwd(st, f["lists"], cam["width"], cam["height"], [1.0, 1.0, 1.0])
    np.testing.assert_allclose(out["image"], 1.0, rtol=0, atol=1e-13)
    assert (out["final_T"] <= 1.0).all() and (out["final_T"] >= 1e-4).all()
    assert out["n_blend"] > 1000  # not a trivial scene


def test_transmittance_monotone_along_the_list():
    sc, cam = _scene(3, n=64)
    cam = dict(cam, width=16, height=16, cx=8.0, cy=8.0)
    f = oracle.forward(sc, cam, [0, 0, 0])
    P = f["lists"]["P"]
    assert P > 20
    prev = np.ones((16, 16))
    for k in range(P + 1):
        lists = dict(vals=f["lists"]["vals"], ranges=np.array([[0, k]], dtype=np.uint32))
        T = oracle.render_fwd(f["state"], lists, 16, 16, [0, 0, 0])["final_T"]
        assert (T <= prev + 1e-16).all()
        prev = T


@pytest.mark.parametrize("seed", [0, 4])
def test_tile_lists_equal_definition_over_global_list(seed):
    sc, cam = _scene(seed, n=40)
    f = oracle.forward(sc, cam, [0.3, 0.1, 0.2])
    sp = f["splats"]
    vis = np.nonzero(sp["radius"] > 0)[0]
    bits = f["depth32"].view(np.uint32)
    order = np.array(sorted(vis.tolist(), key=lambda i: (int(bits[i]), i)), dtype=np.uint32)
    rect = np.stack([oracle.tile_rect(f["state"]["mean2d"][i, 0], f["state"]["mean2d"][i, 1], sp["radius"][i],
                                      cam["width"], cam["height"]) for i in range(len(bits))])
    g = oracle.render_fwd_global(f["state"], order, rect, cam["width"], cam["height"], [0.3, 0.1, 0.2])
    assert np.array_equal(g["image"], f["image"])
    assert np.array_equal(g["final_T"], f["final_T"])


def test_rigid_motion_invariance():
    sc, cam = _scene(5, n=32)
    base = oracle.forward(sc, cam, [0.1, 0.1, 0.1], splat_dtype=np.float64)
    rot = Rotation.from_rotvec([0.3, -0.5, 0.2])
    Q = rot.as_matrix(); d = np.array([0.4, -0.3, 0.2])
    sc2 = dict(sc)
    sc2["mean"] = sc["mean"] @ Q.T + d
    qs = Rotation.from_quat(sc["quat"][:, [1, 2, 3, 0]] / np.linalg.norm(sc["quat"], axis=1, keepdims=True))
    q2 = (rot * qs).as_quat()           # scipy: (x,y,z,w)
    sc2["quat"] = q2[:, [3, 0, 1, 2]] * 1.7   # scale: normalisation must not matter
    cam2 = dict(cam); cam2["R"] = cam["R"] @ Q.T; cam2["t"] = cam["t"] - cam["R"] @ Q.T @ d
    moved = oracle.forward(sc2, cam2, [0.1, 0.1, 0.1], splat_dtype=np.float64)
    np.testing.assert_allclose(moved["image"], base["image"], rtol=0, atol=1e-11)
    assert np.array_equal(moved["splats"]["radius"], base["splats"]["radius"])


def test_permutation_invariance():
    sc, cam = _scene(6, n=48)
    base = oracle.forward(sc, cam, [0, 0, 0])
    perm = np.random.default_rng(1).permutation(48)
    sc2 = {k: (v[perm] if isinstance(v, np.ndarray) else v) for k, v in sc.items()}
    out = oracle.forward(sc2, cam, [0, 0, 0])
    assert len(np.unique(base["depth32"][base["splats"]["radius"] > 0])) == (base["splats"]["radius"] > 0).sum()
    np.testing.assert_allclose(out["image"], base["image"], rtol=0, atol=1e-14)
    assert np.array_equal(out["last_idx"], base["last_idx"])


def test_depth_ties_break_by_index():
    st = dict(mean2d=np.full((3, 2), 8.5), conic=np.tile([0.05, 0.0, 0.05], (3, 1)), opacity=np.full(3, 0.5),
              color=np.eye(3), radius=np.full(3, 8, dtype=np.int32))
    lists = oracle.bin_sort(st["mean2d"], st["radius"], np.array([2.0, 1.0, 1.0], dtype=np.float32), 16, 16)
    assert lists["vals"].tolist() == [1, 2, 0]


@pytest.mark.parametrize("seed", [0, 1])
def test_cov2d_is_pushforward_of_projection_and_conic_is_inverse(seed):
    """cov2d - 0.3 I = A Sigma A^T with A = d(mean2d)/d(mean) taken by finite differences of the projection
    itself and Sigma built with a library rotation: pins the Jacobian, R_q, the scale activation."""
    sc, cam = _scene(seed, n=24)
    sp = oracle.preprocess(sc, cam)
    eps = 1e-6
    A = np.zeros((24, 2, 3))
    for a in range(3):
        hi = dict(sc); hi["mean"] = sc["mean"].copy(); hi["mean"][:, a] += eps
        lo = dict(sc); lo["mean"] = sc["mean"].copy(); lo["mean"][:, a] -= eps
        A[:, :, a] = (oracle.preprocess(hi, cam)["mean2d"] - oracle.preprocess(lo, cam)["mean2d"]) / (2 * eps)
    Rq = Rotation.from_quat(sc["quat"][:, [1, 2, 3, 0]]).as_matrix()     # scipy normalises
    S = np.exp(sc["log_scale"])
    Sigma = np.einsum("nij,nj,nkj->nik", Rq, S * S, Rq)
    cov = np.einsum("nia,nab,njb->nij", A, Sigma, A)
    vis = sp["radius"] > 0
    assert vis.sum() >= 12
    got = sp["cov2d"][vis]
    np.testing.assert_allclose(got[:, 0], cov[vis, 0, 0] + 0.3, rtol=1e-6)
    np.testing.assert_allclose(got[:, 1], cov[vis, 0, 1], rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(got[:, 2], cov[vis, 1, 1] + 0.3, rtol=1e-6)
    a, b, c = got.T
    qa, qb, qc = sp["conic"][vis].T
    np.testing.assert_allclose(qa * a + qb * b, 1.0, rtol=1e-12)
    np.testing.assert_allclose(qb * b + qc * c, 1.0, rtol=1e-12)
    np.testing.assert_allclose(qa * b + qb * c, 0.0, atol=1e-12)


def test_guard_band_clamps_ray_slope():
    """A large splat centred far outside the image: the Jacobian uses the slope clamped to 1.3 x half-FoV, so its
    footprint equals that of the same point moved (at equal depth) onto the guard-band edge."""
    cam = synth.pinhole(64, 64, 60.0, np.eye(3), [0.0, 0.0, 0.0])
    lim = 1.3 * 32 / cam["fx"]
    base = dict(log_scale=np.log([[1.3, 0.9, 1.1]]), quat=np.array([[0.9, 0.1, -0.3, 0.2]]), logit=np.array([0.0]),
                sh=np.zeros((1, 1, 3)), sh_degree=0)
    far_out = dict(base, mean=np.array([[2.0 * lim * 3.0, 0.1, 3.0]]))
    on_edge = dict(base, mean=np.array([[lim * 3.0, 0.1, 3.0]]))
    a = oracle.preprocess(far_out, cam); b = oracle.preprocess(on_edge, cam)
    assert a["radius"][0] > 0 and b["radius"][0] > 0
    np.testing.assert_allclose(a["cov2d"], b["cov2d"], rtol=1e-13)
    assert abs(a["mean2d"][0, 0] - b["mean2d"][0, 0]) > 10  # the centre itself is not clamped
