"""GPU parity for 2D Gaussian surfels: the HIP path (through the C ABI) against the CPU oracle, element by element.

Staged like the 3D-Gaussian tests:
  A. preprocess: fp32 vs fp64 with tolerances; visibility and extent exact except where the oracle flags the decision
     as within 2e-5 of flipping (or the extent as ill-conditioned).
  B. tile lists bit-exact, oracle binning fed with the GPU's own fp32 (mean2d, radius, depth).
  C. compositing forward / backward: oracle fed with the GPU's fp32 state and the identical lists; image within 1e-4
     absolute, gradients within 1e-3 relative + floor; pixels the oracle flags as fragile carry no loss gradient.
  D. splatting backward: oracle fed with the GPU's splat-state gradient.
  E. a full-size view of the 1M-surfel configuration.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_pipeline import to_chw_dev, to_hwc
from helpers import grad_close, to_f64
from paper_2512_20017_amd import binding as B
from paper_2512_20017_amd import synth

pytestmark = pytest.mark.gpu

BG = [0.1, 0.3, 0.2]
IMG_ATOL = 1e-4
GRAD_RTOL = 1e-3
STATE_KEYS = ("mean2d", "T", "opacity", "color")
PARAM_KEYS = ("mean", "tan_u", "tan_v", "log_scale", "logit", "sh")


class SurfelView:
    def __init__(self, n, cam, cap):
        self.n, self.cam, self.cap = n, cam, int(cap)
        self.W, self.H = cam["width"], cam["height"]
        self.splats = B.Splats2D.empty(n)
        self.ws = B.alloc_workspace2d(n, self.W, self.H, self.cap)
        self.image = torch.empty((3, self.H, self.W), dtype=torch.float32, device="cuda")
        self.final_T = torch.empty((self.H, self.W), dtype=torch.float32, device="cuda")
        self.last_idx = torch.empty((self.H, self.W), dtype=torch.int32, device="cuda")
        self.g_splats = B.SplatGrads2D.empty(n)

    def preprocess(self, scene):
        B.pbdr2d_preprocess(scene, self.cam, self.splats)
        torch.cuda.synchronize()
        return self.splats.to_numpy()

    def render_fwd(self, bg):
        B.pbdr2d_render_fwd(self.splats, self.cam, bg, self.cap, self.image, self.final_T, self.last_idx, self.ws)
        torch.cuda.synchronize()
        return dict(image=to_hwc(self.image), final_T=self.final_T.cpu().numpy(),
                    last_idx=self.last_idx.cpu().numpy().astype(np.uint32))

    def lists(self):
        return B.pbdr2d_lists_view(self.ws, self.n, self.W, self.H, self.cap)

    def render_bwd(self, bg, G_hwc, scene=None, grads=None):
        B.pbdr2d_render_bwd(scene, self.splats, self.cam, bg, self.cap, self.final_T, self.last_idx, to_chw_dev(G_hwc),
                            self.g_splats, grads, self.ws)
        torch.cuda.synchronize()
        return self.g_splats.to_numpy()


def _state64(sp):
    return {k: sp[k].astype(np.float64) for k in STATE_KEYS} | {"radius": sp["radius"]}


def _grad_close(name, got, ref):
    grad_close("surfels " + name, got, ref)


def _check_preprocess(sp, ref, cam, sc, max_tie=0.01):
    # S: magnitude of the world coordinates entering p = R x + t (fp32 leaves ~4e-7 S absolute error in p)
    S = float(np.abs(sc["mean"]).max() + np.abs(cam["t"]).max())
    tie = ref["near_tie"] != 0
    assert tie.mean() < max_tie
    assert np.array_equal(sp["radius"][~tie], ref["radius"][~tie])
    vis = (sp["radius"] > 0) & (ref["radius"] > 0)
    if vis.any():
        f = max(cam["fx"], cam["fy"])
        z = ref["depth"][vis]
        # the centre comes through p = R x + t and a perspective divide, the transform through products with f and c
        slope = np.abs(ref["mean2d"][vis] - np.array([cam["cx"], cam["cy"]])) / f
        m_tol = 1e-4 + 3e-7 * np.abs(ref["mean2d"][vis]) + 4e-7 * S * f * (1.0 + slope) / z[:, None]
        m_err = np.abs(sp["mean2d"][vis] - ref["mean2d"][vis])
        assert (m_err <= m_tol).all(), (int((m_err > m_tol).sum()), float(m_err.max()))
        # rows of T are sums of products of size (f + c) x |p|; compare against the row's size and that floor
        scale = np.abs(ref["T"][vis]).reshape(-1, 3, 3).max(axis=2, keepdims=True)
        t_tol = (3e-6 * scale + 6e-7 * (f + max(cam["cx"], cam["cy"])) * S) * np.ones((1, 1, 3))
        t_tol[:, 2, :] = 3e-6 * scale[:, 2, :] + 6e-7 * S
        t_err = np.abs(sp["T"][vis].reshape(-1, 3, 3) - ref["T"][vis].reshape(-1, 3, 3))
        assert (t_err <= t_tol).all(), (int((t_err > t_tol).sum()), float(t_err.max()))
        np.testing.assert_allclose(sp["opacity"][vis], ref["opacity"][vis], rtol=2e-6, atol=1e-7)
        np.testing.assert_allclose(sp["color"][vis], ref["color"][vis], rtol=2e-5, atol=4e-6)
        np.testing.assert_allclose(sp["depth"][vis], ref["depth"][vis], rtol=2e-6, atol=2e-6 + 6e-7 * S)
        # Gram-Schmidt loses accuracy as the raw tangents approach parallel: error ~ eps / sin(angle between them)
        a, b = np.asarray(sc["tan_u"], dtype=np.float64)[vis], np.asarray(sc["tan_v"], dtype=np.float64)[vis]
        sin = np.linalg.norm(np.cross(a, b), axis=1) / (np.linalg.norm(a, axis=1) * np.linalg.norm(b, axis=1))
        n_err = np.abs(sp["normal"][vis] - ref["normal"][vis]).max(axis=1)
        assert (n_err <= 2e-6 / sin).all(), float((n_err * sin).max())
    return tie, vis


CASES = [
    ("deg3_ragged", lambda: (synth.random_small_surfels(21, 500, 3, spread=1.2, ls_mu=-2.4),
                             synth.pinhole(200, 120, 60.0, *synth.look_at([0.4, 0.3, -3.0], [0, 0, 0], [0, 1, 0])))),
    ("deg2_ragged", lambda: (synth.random_small_surfels(22, 300, 2, spread=0.9),
                             synth.pinhole(75, 51, 50.0, np.eye(3), [0.0, 0.1, 2.6]))),
    ("deg1_dense", lambda: (synth.random_small_surfels(23, 2000, 1, spread=0.5, ls_mu=-2.0),
                            synth.pinhole(64, 64, 50.0, np.eye(3), [0.0, 0.0, 2.0]))),
    ("deg0_small_disks", lambda: (synth.random_small_surfels(24, 3000, 0, spread=1.0, ls_mu=-4.5),     # low-pass dominated
                                  synth.pinhole(160, 96, 55.0, np.eye(3), [0.0, 0.0, 2.5]))),
]


@pytest.fixture(scope="module", params=CASES, ids=[c[0] for c in CASES])
def case(request):
    sc, cam = request.param[1]()
    n = sc["mean"].shape[0]
    scene = B.Scene2D.from_numpy(sc)
    ref = oracle.preprocess2d(to_f64(sc), cam)
    probe = SurfelView(n, cam, 1)
    sp = probe.preprocess(scene)
    lists = oracle.bin_sort(sp["mean2d"].astype(np.float64), sp["radius"], sp["depth"], cam["width"], cam["height"])
    view = SurfelView(n, cam, lists["P"] + 17)
    sp2 = view.preprocess(scene)
    for k in sp:
        assert np.array_equal(sp[k][sp["radius"] > 0], sp2[k][sp["radius"] > 0])
    return dict(sc=sc, cam=cam, n=n, scene=scene, ref=ref, view=view, sp=sp, lists=lists)


def test_a_preprocess(case):
    _check_preprocess(case["sp"], case["ref"], case["cam"], case["sc"], max_tie=0.02)
    assert (case["sp"]["radius"] > 0).sum() > 0.3 * case["n"]


def test_b_lists_bit_exact(case):
    view, lists = case["view"], case["lists"]
    view.render_fwd(BG)
    gl = view.lists()
    assert gl["P_raw"] == lists["P"]
    assert np.array_equal(gl["keys"], lists["keys"])
    assert np.array_equal(gl["vals"], lists["vals"])
    assert np.array_equal(gl["ranges"], lists["ranges"])


def test_c_compositing(case):
    view, lists, cam, sp = case["view"], case["lists"], case["cam"], case["sp"]
    W, H = cam["width"], cam["height"]
    got = view.render_fwd(BG)
    st = _state64(sp)
    ref = oracle.render_fwd2d(st, lists, W, H, BG)
    ok = ref["fragile"] == 0
    assert (~ok).mean() < 0.02
    assert np.abs(got["image"] - ref["image"])[ok].max() <= IMG_ATOL
    assert np.abs(got["final_T"] - ref["final_T"])[ok].max() <= IMG_ATOL
    assert np.array_equal(got["last_idx"][ok], ref["last_idx"][ok])
    assert ref["n_blend"] > 10 * W * H / 256
    G = np.random.default_rng(5).normal(size=(H, W, 3)).astype(np.float32)
    G[~ok] = 0.0
    gs = view.render_bwd(BG, G)
    ref_b = oracle.render_bwd2d(st, lists, W, H, BG, G.astype(np.float64))
    v = sp["radius"] > 0
    assert np.abs(ref_b["T"]).max() > 0 and np.abs(ref_b["mean2d"]).max() > 0
    # the transform's gradient is judged row by row against that row's own magnitude (rows differ by the focal length)
    for r in range(3):
        _grad_close(f"T{r}", gs["T"][v][:, 3 * r:3 * r + 3], ref_b["T"][v][:, 3 * r:3 * r + 3])
    for k in ("mean2d", "opacity", "color"):
        _grad_close(k, gs[k][v], ref_b[k][v])


def test_d_splatting_backward(case):
    view, cam, sp, sc, scene = case["view"], case["cam"], case["sp"], case["sc"], case["scene"]
    W, H = cam["width"], cam["height"]
    view.render_fwd(BG)
    G = np.random.default_rng(6).normal(size=(H, W, 3)).astype(np.float32)
    grads = scene.zeros_like()
    gs = view.render_bwd(BG, G, scene=scene, grads=grads)
    got = grads.to_numpy()
    ref = oracle.preprocess_bwd2d(to_f64(sc), cam, {k: gs[k].astype(np.float64) for k in STATE_KEYS})
    both = (sp["radius"] > 0) & (case["ref"]["radius"] > 0) & (case["ref"]["near_tie"] == 0)
    for k in PARAM_KEYS:
        _grad_close(k, got[k][both], ref[k][both])
    # accumulation: a second backward doubles the parameter gradient (up to the order of the in-tile float sums)
    view.render_bwd(BG, G, scene=scene, grads=grads)
    got2 = grads.to_numpy()
    for k in PARAM_KEYS:
        np.testing.assert_allclose(got2[k], 2.0 * got[k], rtol=1e-4, atol=1e-5 * np.abs(got[k]).max())


def test_edge_empty_and_all_culled():
    cam = synth.pinhole(48, 40, 50.0, np.eye(3), [0.0, 0.0, 2.0])
    # no points at all
    view = SurfelView(0, cam, 1)
    scene = B.Scene2D.from_numpy(dict(mean=np.zeros((0, 3)), tan_u=np.zeros((0, 3)), tan_v=np.zeros((0, 3)),
                                      log_scale=np.zeros((0, 2)), logit=np.zeros(0), sh=np.zeros((0, 1, 3)), sh_degree=0))
    view.preprocess(scene)
    out = view.render_fwd(BG)
    assert np.allclose(out["image"], np.asarray(BG, dtype=np.float32)[None, None, :])
    assert (out["final_T"] == 1).all() and (out["last_idx"] == 0).all()
    # every point behind the camera
    sc = synth.random_small_surfels(31, 100, 1)
    sc["mean"][:, 2] -= 10.0
    scene = B.Scene2D.from_numpy(sc)
    view = SurfelView(100, cam, 64)
    sp = view.preprocess(scene)
    assert (sp["radius"] == 0).all()
    out = view.render_fwd(BG)
    assert np.allclose(out["image"], np.asarray(BG, dtype=np.float32)[None, None, :])
    assert view.lists()["P_raw"] == 0
    grads = scene.zeros_like()
    view.render_bwd(BG, np.ones((40, 48, 3), dtype=np.float32), scene=scene, grads=grads)
    assert all(not v.any() for k, v in grads.to_numpy().items() if k != "sh_degree")


def test_edge_capacity_overflow_is_contained():
    sc = synth.random_small_surfels(23, 2000, 1, spread=0.5, ls_mu=-2.0)
    cam = synth.pinhole(64, 64, 50.0, np.eye(3), [0.0, 0.0, 2.0])
    scene = B.Scene2D.from_numpy(sc)
    view = SurfelView(2000, cam, 500)
    view.preprocess(scene)
    out = view.render_fwd(BG)
    gl = view.lists()
    assert gl["P_raw"] > 500 and gl["P"] == 500
    assert np.isfinite(out["image"]).all()
    gs = view.render_bwd(BG, np.ones((64, 64, 3), dtype=np.float32))
    v = view.splats.radius.cpu().numpy() > 0
    assert all(np.isfinite(gs[k][v]).all() for k in STATE_KEYS)


@pytest.mark.timeout(600)
def test_e_full_size_view():
    """1M surfels, SH3, 1920x1080 (the surfel benchmark configuration), every stage over the whole image."""
    sc = synth.scene_surfels(0)
    cam = synth.cameras_sphere()[0]
    n = sc["mean"].shape[0]
    W, H = cam["width"], cam["height"]
    scene = B.Scene2D.from_numpy(sc)
    cap = 8_000_000
    view = SurfelView(n, cam, cap)
    sp = view.preprocess(scene)
    sc64 = to_f64(sc)
    ref = oracle.preprocess2d(sc64, cam)
    tie, vis = _check_preprocess(sp, ref, cam, sc)
    lists = oracle.bin_sort(sp["mean2d"].astype(np.float64), sp["radius"], sp["depth"], W, H)
    assert lists["P"] <= cap
    got = view.render_fwd([0.0, 0.0, 0.0])
    gl = view.lists()
    assert gl["P_raw"] == lists["P"]
    assert np.array_equal(gl["keys"], lists["keys"])
    assert np.array_equal(gl["vals"], lists["vals"])
    assert np.array_equal(gl["ranges"], lists["ranges"])
    st = _state64(sp)
    ref_f = oracle.render_fwd2d(st, lists, W, H, [0.0, 0.0, 0.0])
    ok = ref_f["fragile"] == 0
    assert (~ok).mean() < 0.02
    assert np.abs(got["image"] - ref_f["image"])[ok].max() <= IMG_ATOL
    assert np.abs(got["final_T"] - ref_f["final_T"])[ok].max() <= IMG_ATOL
    assert np.array_equal(got["last_idx"][ok], ref_f["last_idx"][ok])
    G = np.random.default_rng(0).normal(size=(H, W, 3)).astype(np.float32)
    G[~ok] = 0.0
    grads = scene.zeros_like()
    gs = view.render_bwd([0.0, 0.0, 0.0], G, scene=scene, grads=grads)
    ref_b = oracle.render_bwd2d(st, lists, W, H, [0.0, 0.0, 0.0], G.astype(np.float64))
    v = sp["radius"] > 0
    for r in range(3):
        _grad_close(f"T{r}", gs["T"][v][:, 3 * r:3 * r + 3], ref_b["T"][v][:, 3 * r:3 * r + 3])
    for k in ("mean2d", "opacity", "color"):
        _grad_close(k, gs[k][v], ref_b[k][v])
    ref_g = oracle.preprocess_bwd2d(sc64, cam, {k: gs[k].astype(np.float64) for k in STATE_KEYS})
    got_g = grads.to_numpy()
    both = vis & ~tie
    for k in PARAM_KEYS:
        _grad_close(k, got_g[k][both], ref_g[k][both])


def test_first_view_writes_what_zero_then_accumulate_leaves():
    """Surfel twin of the 3D test: first_view stores instead of accumulating and zeroes the points the view skips."""
    sc = synth.random_small_surfels(41, 400, 2, spread=1.2)
    cam = synth.pinhole(96, 64, 45.0, *synth.look_at([0.3, 0.1, -2.5], [0, 0, 0], [0, 1, 0]))
    scene = B.Scene2D.from_numpy(sc)
    view = SurfelView(400, cam, 200000)
    sp = view.preprocess(scene)
    assert 0 < (sp["radius"] > 0).sum() < 400
    view.render_fwd(BG)
    G = np.random.default_rng(2).normal(size=(64, 96, 3)).astype(np.float32)
    ref = scene.zeros_like()
    view.render_bwd(BG, G, scene=scene, grads=ref)
    got = scene.zeros_like()
    for t in (got.mean, got.tan_u, got.tan_v, got.log_scale, got.logit, got.sh):
        t.fill_(float("nan"))
    B.pbdr2d_render_bwd(scene, view.splats, cam, BG, view.cap, view.final_T, view.last_idx, to_chw_dev(G), view.g_splats, got,
                        view.ws, first_view=True)
    torch.cuda.synchronize()
    a, b = got.to_numpy(), ref.to_numpy()
    unused = sp["radius"] <= 0
    for k in PARAM_KEYS:
        assert np.isfinite(a[k]).all(), k
        np.testing.assert_allclose(a[k], b[k], rtol=4e-6, atol=1e-6 * np.abs(b[k]).max())
        assert not a[k][unused].any(), k


def test_backward_without_splat_gradient_output():
    """g_splats = NULL with a scene: the splatting backward reads the per-point records in the workspace instead of the
    planes; the parameter gradient is the one the two-step path gives (same values and formulas; the two compositing runs
    differ by the rounding of their LDS adds and the two kernel variants by the compiler's choice of fused multiply-adds:
    4e-6 relative, as between the store and accumulate variants), as a store and as an accumulation, for the whole image
    and for a patch."""
    sc = synth.random_small_surfels(43, 3000, 2, spread=1.2)
    cam = synth.pinhole(160, 96, 50.0, *synth.look_at([0.3, 0.1, -2.5], [0, 0, 0], [0, 1, 0]))
    scene = B.Scene2D.from_numpy(sc)
    view = SurfelView(3000, cam, 400000)
    sp = view.preprocess(scene)
    assert 0 < (sp["radius"] > 0).sum() < 3000
    view.render_fwd(BG)
    G = to_chw_dev(np.random.default_rng(3).normal(size=(96, 160, 3)).astype(np.float32))
    for first in (True, False):
        ref, got = scene.zeros_like(), scene.zeros_like()
        if not first:
            for t in (ref, got):
                t.mean.fill_(0.25); t.sh.fill_(-0.5)
        B.pbdr2d_render_bwd(scene, view.splats, cam, BG, view.cap, view.final_T, view.last_idx, G, view.g_splats, ref, view.ws,
                            first_view=first)
        B.pbdr2d_render_bwd(scene, view.splats, cam, BG, view.cap, view.final_T, view.last_idx, G, None, got, view.ws,
                            first_view=first)
        torch.cuda.synchronize()
        a, b = got.to_numpy(), ref.to_numpy()
        for k in PARAM_KEYS:
            np.testing.assert_allclose(a[k], b[k], rtol=4e-6, atol=1e-6 * np.abs(b[k]).max(), err_msg=f"{k} {first}")
            assert np.array_equal(a[k] == 0, b[k] == 0) or first is False, k      # the same points get exact zeros
        assert np.abs(b["mean"]).max() > 0
    # a patch
    patch = (37, 10, 140, 81)
    w, h = patch[2] - patch[0], patch[3] - patch[1]
    splats = B.Splats2D.empty(3000)
    B.pbdr2d_preprocess_patch(scene, cam, patch, splats)
    image = torch.empty((3, h, w), device="cuda"); T = torch.empty((h, w), device="cuda")
    last = torch.empty((h, w), dtype=torch.int32, device="cuda")
    B.pbdr2d_render_fwd_patch(splats, cam, patch, BG, view.cap, image, T, last, view.ws)
    Gp = G[:, patch[1]:patch[3], patch[0]:patch[2]].contiguous()
    ref, got = scene.zeros_like(), scene.zeros_like()
    B.pbdr2d_render_bwd_patch(scene, splats, cam, patch, BG, view.cap, T, last, Gp, view.g_splats, ref, view.ws, first_view=True)
    B.pbdr2d_render_bwd_patch(scene, splats, cam, patch, BG, view.cap, T, last, Gp, None, got, view.ws, first_view=True)
    torch.cuda.synchronize()
    a, b = got.to_numpy(), ref.to_numpy()
    for k in PARAM_KEYS:
        np.testing.assert_allclose(a[k], b[k], rtol=4e-6, atol=1e-6 * np.abs(b[k]).max(), err_msg=k)
    # no output at all is still an error
    with pytest.raises(B.PbdrError):
        B.pbdr2d_render_bwd(None, view.splats, cam, BG, view.cap, view.final_T, view.last_idx, G, None, None, view.ws)


def test_backward_writes_every_per_pair_record_itself():
    """The backward pass needs no cleared workspace: records of pairs that lie behind the last splat their tile blended are
    written as zeros by the compositing kernel. A dense scene (most lists end early on transmittance) is rendered with
    the whole workspace poisoned with NaN bit patterns before the forward pass; the gradient equals that of a clean run."""
    sc = synth.random_small_surfels(47, 6000, 1, spread=0.5, ls_mu=-1.6)     # large, overlapping disks
    sc["logit"] = np.full(6000, 4.0, dtype=np.float32)                       # nearly opaque: pixels saturate early
    cam = synth.pinhole(160, 96, 50.0, *synth.look_at([0.2, 0.1, -2.5], [0, 0, 0], [0, 1, 0]))
    scene = B.Scene2D.from_numpy(sc)
    G = np.random.default_rng(9).normal(size=(96, 160, 3)).astype(np.float32)
    out = []
    for poison in (False, True):
        view = SurfelView(6000, cam, 600000)
        view.ws.fill_(0xFF if poison else 0)
        vis = view.preprocess(scene)["radius"] > 0
        fw = view.render_fwd(BG)
        lists = view.lists()
        grads = scene.zeros_like()
        g2 = view.render_bwd(BG, G, scene=scene, grads=grads)
        out.append((g2, grads.to_numpy(), fw, lists))
    (g2a, ga, fwa, la), (g2b, gb, fwb, lb) = out
    # the case is what it claims: many pairs lie behind the last blended splat of their tile
    tiles = la["ranges"]
    walked = 0
    last = fwa["last_idx"]
    for t in range(tiles.shape[0]):
        ty, tx = divmod(t, 10)
        walked += int(last[ty * 16:(ty + 1) * 16, tx * 16:(tx + 1) * 16].max())
    assert walked < 0.8 * la["P"], (walked, la["P"])
    assert np.array_equal(fwa["image"], fwb["image"])
    for k in g2a:      # the splat-state gradient is written for the listed points only
        assert np.isfinite(g2b[k][vis]).all(), k
        np.testing.assert_allclose(g2b[k][vis], g2a[k][vis], rtol=1e-5, atol=1e-6 * np.abs(g2a[k][vis]).max(), err_msg=k)
    for k in PARAM_KEYS:
        assert np.isfinite(gb[k]).all(), k
        np.testing.assert_allclose(gb[k], ga[k], rtol=1e-5, atol=1e-6 * np.abs(ga[k]).max(), err_msg=k)
