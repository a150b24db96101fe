"""Pins for the oracle's point-group frustum culling (paper App. D.1; groups of Sec. 4.2.1) -- no GPU.

The group test must never change a result: a dropped group may only hold points that the per-point culls drop
anyway. That is checked by brute force (grouped == ungrouped preprocessing, element for element) on scenes built
to stress each clause of the rule -- cameras inside the cloud, boxes straddling the near plane and the image
border, large splats whose centre is off screen but whose extent reaches it -- and the rule's usefulness is
checked on boxes whose fate is known from geometry alone.
"""
import numpy as np
import pytest

import oracle
from helpers import simple_camera, to_f64
from paper_2512_20017_amd import synth

STATE = ("mean2d", "conic", "opacity", "color", "radius", "depth")


def _street_like(seed, n=6000, scale_mu=-3.0):
    """A slab of points around cameras placed inside it (most groups out of view), stored in Z-order."""
    rng = np.random.default_rng(seed)
    mean = rng.uniform([-20, -20, 0], [20, 20, 4], size=(n, 3))
    sc = dict(mean=mean, log_scale=rng.normal(scale_mu, 0.6, size=(n, 3)), quat=rng.normal(size=(n, 4)),
              logit=rng.normal(size=n), sh=rng.uniform(-1, 1, size=(n, 1, 3)), sh_degree=0)
    perm = synth.zorder_permutation(mean.astype(np.float32))
    return {k: (v[perm] if isinstance(v, np.ndarray) else v) for k, v in sc.items()}


def _street_cam(seed, width=160, height=96, far=1e10, radius_clip=0.0):
    rng = np.random.default_rng(1000 + seed)
    pos = np.array([rng.uniform(-15, 15), rng.uniform(-15, 15), 2.0])
    yaw = rng.uniform(0, 2 * np.pi)
    R, t = synth.look_at(pos, pos + np.array([np.cos(yaw), np.sin(yaw), 0.0]), [0, 0, 1.0])
    return synth.pinhole(width, height, 70.0, R, t, far=far, radius_clip=radius_clip)


def test_bounds_are_min_max_of_each_group():
    sc = _street_like(0, n=1000)
    G = 64
    b = oracle.group_bounds(sc, G)
    assert b.shape == (16, 7)
    for g in range(16):
        sl = slice(g * G, min((g + 1) * G, 1000))
        np.testing.assert_array_equal(b[g, 0:3], sc["mean"][sl].min(axis=0))
        np.testing.assert_array_equal(b[g, 3:6], sc["mean"][sl].max(axis=0))
        np.testing.assert_allclose(b[g, 6], np.exp(sc["log_scale"][sl].max()), rtol=1e-15)


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("G", [32, 256])
def test_grouped_equals_ungrouped_inside_the_cloud(seed, G):
    sc = _street_like(seed)
    cam = _street_cam(seed, far=25.0 if seed % 2 else 1e10, radius_clip=2.0 if seed == 3 else 0.0)
    ref = oracle.preprocess(sc, cam)
    got = oracle.preprocess_grouped(sc, cam, G)
    for k in STATE:
        vis = ref["radius"] > 0
        assert np.array_equal(got["radius"], ref["radius"])
        np.testing.assert_array_equal(got[k][vis], ref[k][vis])
    # the rule is worth something here: a good share of the groups goes, and no kept group is needed by accident only
    keep = got["keep"].astype(bool)
    assert keep.sum() < (0.9 if G == 32 else 1.01) * keep.size
    vis_groups = np.unique(np.nonzero(ref["radius"] > 0)[0] // G)
    assert keep[vis_groups].all()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_grouped_equals_ungrouped_with_large_offscreen_splats(seed):
    # big splats (sigma ~ 0.4 m) close to the camera: many centres project far off screen while the extent still
    # reaches the image; groups of such points must be kept
    sc = _street_like(10 + seed, n=3000, scale_mu=-1.0)
    cam = _street_cam(seed, width=96, height=64)
    ref = oracle.preprocess(sc, cam)
    got = oracle.preprocess_grouped(sc, cam, 16)
    assert np.array_equal(got["radius"], ref["radius"])
    off = (ref["radius"] > 0) & ((ref["mean2d"][:, 0] < 0) | (ref["mean2d"][:, 0] > cam["width"]))
    assert off.sum() > 10       # the case is exercised


def test_known_boxes():
    cam = simple_camera(128, 96, 100.0, 0.0, near=0.2, far=50.0)      # camera at the origin looking down +z
    s = 0.01

    def keep(lo, hi, smax=s):
        b = np.array([[*lo, *hi, smax]], dtype=np.float64)
        r = oracle.group_cull(b, cam)
        return int(r["keep"][0])

    assert keep([-1, -1, 5], [1, 1, 6]) == 1                 # in view
    assert keep([-1, -1, -6], [1, 1, -5]) == 0               # behind the camera
    assert keep([-1, -1, 60], [1, 1, 70]) == 0               # beyond the far plane
    assert keep([-1, -1, 49], [1, 1, 51]) == 1               # straddles the far plane
    assert keep([-1, -1, -1], [1, 1, 1]) == 1                # straddles the near plane: always kept
    assert keep([20, -1, 5], [22, 1, 6]) == 0                # far to the right: x/z >= 3.3, image edge at 0.64
    assert keep([-22, -1, 5], [-20, 1, 6]) == 0
    assert keep([-1, 20, 5], [1, 22, 6]) == 0
    assert keep([-1, -22, 5], [1, -20, 6]) == 0
    assert keep([3.0, -1, 5], [3.4, 1, 5.2]) == 1            # centre-to-edge 0.6..0.68: touches the right border
    # a box off to the side whose corners are all outside the image, but which spans the whole view in depth: kept
    # because its projected rectangle crosses the image (the eight-corner test of the paper would drop it)
    assert keep([-40, -0.5, 1], [40, 0.5, 1.5]) == 1
    # off screen by 60 px at depth 5, scale small: dropped; same box with 1 m splats (extent ~ 3 * 100 * 1 / 5 px
    # times the guard-band factor): kept
    assert keep([6.6, -0.2, 5], [7.0, 0.2, 5.2]) == 0
    assert keep([6.6, -0.2, 5], [7.0, 0.2, 5.2], smax=1.0) == 1


def test_extent_bound_really_bounds_every_radius():
    # k1 s_max / z + k0 of the rule against the radii the per-point path produces, over random anisotropic, rotated
    # splats at every position of the guard band
    rng = np.random.default_rng(7)
    n = 4000
    sc = dict(mean=rng.uniform([-6, -4, 1], [6, 4, 12], size=(n, 3)), log_scale=rng.normal(-2.0, 1.0, size=(n, 3)),
              quat=rng.normal(size=(n, 4)), logit=np.zeros(n), sh=np.zeros((n, 1, 3)), sh_degree=0)
    cam = simple_camera(200, 120, 150.0, 0.0)
    sp = oracle.preprocess(sc, cam)
    lim_x, lim_y = 1.3 * 100 / 150.0, 1.3 * 60 / 150.0
    k1 = 3 * np.sqrt(150.0 ** 2 * (1 + lim_x ** 2) + 150.0 ** 2 * (1 + lim_y ** 2))
    k0 = 3 * np.sqrt(0.3 + np.sqrt(0.1)) + 1
    smax = np.exp(sc["log_scale"]).max(axis=1)
    z = sc["mean"][:, 2]
    vis = sp["radius"] > 0
    assert vis.sum() > 1000
    assert (sp["radius"][vis] <= (k1 * smax / z + k0)[vis]).all()
    # and it is not absurdly loose: within a factor ~2.5 (the Frobenius norm over both image axes) for round splats
    iso = dict(sc, log_scale=np.repeat(sc["log_scale"][:, :1], 3, axis=1))
    sp2 = oracle.preprocess(iso, cam)
    v2 = sp2["radius"] > 20
    bound2 = k1 * np.exp(iso["log_scale"][:, 0]) / z + k0
    assert (bound2[v2] / sp2["radius"][v2]).max() < 2.5


def test_near_tie_flags_only_boxes_at_a_threshold():
    cam = simple_camera(128, 96, 100.0, 0.0, near=0.2, far=50.0)
    b = np.array([[-1, -1, 5, 1, 1, 6, 0.01],                 # clearly kept
                  [-1, -1, -6, 1, 1, -5, 0.01],               # clearly dropped
                  [-1, -1, 50.0 + 1e-7, 1, 1, 70, 0.01],      # zmin within 2e-9 relative of the far plane
                  [-1, -1, -3, 1, 1, 0.2 - 1e-9, 0.01]])      # zmax just under the near plane
    r = oracle.group_cull(b, cam, tau=1e-6)
    assert r["near_tie"].tolist() == [0, 0, 1, 1]


def test_planted_mistakes_are_caught():
    # the brute-force comparison above must be able to fail: rules that ignore the splat extent, or that test the
    # eight corners against the frustum, lose visible points on the large-splat scene
    sc = _street_like(11, n=3000, scale_mu=-1.0)
    cam = _street_cam(1, width=96, height=64)
    ref = oracle.preprocess(sc, cam)
    G = 16
    b = oracle.group_bounds(sc, G)
    R, t = np.asarray(cam["R"]), np.asarray(cam["t"])
    lost_no_extent = lost_corners = 0
    for g in range(b.shape[0]):
        corners = np.array([[b[g, 3 * ((k >> a) & 1) + a] for a in range(3)] for k in range(8)])
        p = corners @ R.T + t
        members = ref["radius"][g * G:(g + 1) * G]
        if p[:, 2].min() < cam["near"]:
            continue
        mx = cam["fx"] * p[:, 0] / p[:, 2] + cam["cx"]; my = cam["fy"] * p[:, 1] / p[:, 2] + cam["cy"]
        no_extent_drop = mx.max() < 0 or mx.min() > cam["width"] or my.max() < 0 or my.min() > cam["height"]
        inside = (mx >= 0) & (mx <= cam["width"]) & (my >= 0) & (my <= cam["height"])
        if no_extent_drop and (members > 0).any():
            lost_no_extent += 1
        if not inside.any() and (members > 0).any():
            lost_corners += 1
    assert lost_no_extent > 0 and lost_corners > 0
