"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

mid   : 1M Gaussians, SH3, 1920x1080 -- every stage against the oracle over the whole image / all points.
batch : the same scene from 16 cameras -- tile lists bit-exact for every view, images and accumulated gradients for two.
large : 8M Gaussians, 3840x2160 street-level views where most points are culled -- lists for four views, image and
        gradients for one.
The oracle finishes each of these in seconds (OpenMP over the host's cores).
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_pipeline import GpuView, to_chw_dev
from helpers import IMG_ATOL, grad_close
from paper_2512_20017_amd import binding as B
from paper_2512_20017_amd import synth

pytestmark = pytest.mark.gpu

BG = [0.0, 0.0, 0.0]


def _state64(sp):
    st = {k: sp[k].astype(np.float64) for k in ("mean2d", "conic", "opacity", "color")}
    st["radius"] = sp["radius"]
    return st



def _run_view(scene, sc, cam, n, cap, check_image=True, grads_into=None, G_seed=0, tag="view"):
    """One view through the HIP path with staged checks against the oracle. Returns the oracle's parameter gradient."""
    W, H = cam["width"], cam["height"]
    view = GpuView(n, cam, cap)
    sp = view.preprocess(scene)
    ref_sp = oracle.preprocess(sc, cam)
    tie = ref_sp["near_tie"] != 0
    assert tie.mean() < 0.01
    assert np.array_equal(sp["radius"][~tie], ref_sp["radius"][~tie])
    vis = (sp["radius"] > 0) & (ref_sp["radius"] > 0)
    # fp32 forms p = R x + t from inputs of magnitude S, so p carries ~4e-7 S absolute error; through the perspective
    # divide that is ~4e-7 S f (1 + |slope|) / z pixels (small at z = 15, larger near the camera), plus the rounding of
    # the pixel coordinate itself
    f = max(cam["fx"], cam["fy"])
    S = float(np.abs(sc["mean"]).max() + np.abs(cam["t"]).max())
    z = ref_sp["depth"][vis]
    slope = np.abs(ref_sp["mean2d"][vis] - np.array([cam["cx"], cam["cy"]])) / f
    tol = 1e-4 + 3e-7 * np.abs(ref_sp["mean2d"][vis]) + 4e-7 * S * f * (1.0 + slope) / z[:, None]
    e_m = np.abs(sp["mean2d"][vis] - ref_sp["mean2d"][vis]) / tol
    assert e_m.max() <= 1.0
    np.testing.assert_allclose(sp["color"][vis], ref_sp["color"][vis], rtol=2e-5, atol=4e-6)
    # depth = row 2 of R . mean + t: the same ~4e-7 S of absolute error, plus its own rounding
    e_d = np.abs(sp["depth"][vis] - z) / (2e-7 * z + 4e-7 * S)
    assert e_d.max() <= 1.0
    np.testing.assert_allclose(sp["opacity"][vis], ref_sp["opacity"][vis], rtol=1e-5, atol=1e-30)
    # conic, entry by entry, against the largest entry of the splat's conic: it inherits the relative error of p (the
    # Jacobian is built from p: ~4e-7 S / z per entry, twice for the product J . J^T) on top of its own rounding
    scale = np.abs(ref_sp["conic"][vis]).max(axis=1)
    e_c = np.abs(sp["conic"][vis] - ref_sp["conic"][vis]).max(axis=1) / ((1e-5 + 2e-6 * S / z) * scale)
    assert e_c.max() <= 1.0
    print(f"[parity] {tag} preprocess: worst |err|/tol mean2d {e_m.max():.3f}, depth {e_d.max():.3f}, conic {e_c.max():.3f}; "
          f"near-tie points {int(tie.sum())} of {n}")
    # lists, bit-exact, from the GPU's own fp32 splat state
    lists = oracle.bin_sort(sp["mean2d"].astype(np.float64), sp["radius"], sp["depth"], W, H)
    assert lists["P"] <= cap
    got_f = view.render_fwd(BG)
    gl = view.lists()
    assert gl["P_raw"] == lists["P"]
    assert np.array_equal(gl["keys"], lists["keys"])
    assert np.array_equal(gl["vals"], lists["vals"])
    assert np.array_equal(gl["ranges"], lists["ranges"])
    if not check_image:
        return None
    st = _state64(sp)
    ref_f = oracle.render_fwd(st, lists, W, H, BG)
    ok = ref_f["fragile"] == 0
    assert (~ok).mean() < 1e-3
    e_img = float(np.abs(got_f["image"] - ref_f["image"])[ok].max()); e_T = float(np.abs(got_f["final_T"] - ref_f["final_T"])[ok].max())
    print(f"[parity] {tag} forward: max |image err| {e_img:.2e}, max |final_T err| {e_T:.2e} (tolerance {IMG_ATOL:.0e}); "
          f"fragile pixels {int((~ok).sum())} of {ok.size}")
    assert e_img <= IMG_ATOL and e_T <= IMG_ATOL
    assert np.array_equal(got_f["last_idx"][ok], ref_f["last_idx"][ok])
    ex, bl = B.pbdr_render_stats(cam, n, cap, view.ws)
    assert abs(ex - ref_f["n_eval"]) <= 1e-6 * ref_f["n_eval"] + 100 and abs(bl - ref_f["n_blend"]) <= 1e-6 * ref_f["n_blend"] + 100
    # backward
    G = np.random.default_rng(G_seed).normal(size=(H, W, 3)).astype(np.float32)
    G[~ok] = 0.0
    gs = view.render_bwd(BG, G, scene=scene, grads=grads_into)
    ref_b = oracle.render_bwd(st, lists, W, H, BG, G.astype(np.float64))
    v = sp["radius"] > 0
    for k in ("mean2d", "conic", "opacity", "color"):
        grad_close(f"{tag} composite bwd {k}", gs[k][v], ref_b[k][v])
    # splatting backward: oracle fed with the GPU's splat-state gradient
    ref_g = oracle.preprocess_bwd(sc, cam, {k: gs[k].astype(np.float64) for k in ("mean2d", "conic", "opacity", "color")})
    both = vis & ~tie
    return ref_g, both


@pytest.fixture(scope="module")
def mid():
    sc = synth.scene_mid(0)
    return sc, B.Scene.from_numpy(sc), synth.cameras_sphere()


@pytest.mark.timeout(300)
def test_mid_full_view(mid):
    sc, scene, cams = mid
    n = scene.n
    grads = scene.zeros_like()
    ref_g, both = _run_view(scene, sc, cams[0], n, 3_700_000, grads_into=grads, tag="mid")
    torch.cuda.synchronize()
    got = grads.to_numpy()
    for k in ("mean", "log_scale", "quat", "logit", "sh"):
        grad_close(f"splatting bwd {k}", got[k][both], ref_g[k][both])


@pytest.mark.timeout(600)
def test_batch_of_sixteen_views(mid):
    sc, scene, cams = mid
    n = scene.n
    grads = scene.zeros_like()
    total = None
    both_all = None
    for ci, cam in enumerate(cams):
        full = ci in (3, 11)
        out = _run_view(scene, sc, cam, n, 6_000_000, check_image=full, grads_into=grads if full else None, G_seed=ci, tag=f"batch view {ci}")
        if full:
            ref_g, both = out
            total = ref_g if total is None else {k: total[k] + ref_g[k] for k in ("mean", "log_scale", "quat", "logit", "sh")}
            both_all = both if both_all is None else (both_all | both)
    torch.cuda.synchronize()
    got = grads.to_numpy()     # gradients of the two fully checked views, accumulated into one buffer (Alg. 1 l.22-24)
    for k in ("mean", "log_scale", "quat", "logit", "sh"):
        grad_close(f"two views accumulated {k}", got[k][both_all], total[k][both_all])


@pytest.fixture(scope="module")
def large():
    sc = synth.scene_large(0)
    return sc, B.Scene.from_numpy(sc), synth.cameras_street(0)


@pytest.mark.timeout(600)
def test_large_street_views(large):
    sc, scene, cams = large
    n = scene.n
    grads = scene.zeros_like()
    for ci in (0, 1, 2, 5):
        full = ci == 2
        out = _run_view(scene, sc, cams[ci], n, 12_000_000, check_image=full, grads_into=grads if full else None, G_seed=ci, tag=f"street view {ci}")
        if full:
            ref_g, both = out
            torch.cuda.synchronize()
            got = grads.to_numpy()
            for k in ("mean", "log_scale", "quat", "logit", "sh"):
                grad_close(f"splatting bwd {k}", got[k][both], ref_g[k][both])


@pytest.mark.timeout(900)
def test_large_batch_of_eight_views_accumulated(large):
    """The 8M-point street scene as the batch it is meant to be (App. D.1; Alg. 1 lines 2-4 and 21-24 over a batch): all
    eight 4K views preprocessed in one pass with point-group culling, rendered, and their gradients summed into one buffer
    by the batched splatting backward. Per view the loss lives on a seeded sample of 256 tiles (dL/dimage is zero
    elsewhere), which keeps the oracle's backward affordable; the oracle's per-view gradients, summed, must equal the
    accumulated buffer."""
    sc, scene, cams = large
    n = scene.n
    W, H = cams[0]["width"], cams[0]["height"]
    TX, TY = (W + 15) // 16, (H + 15) // 16
    group = 1024
    ng = B.pbdr_group_count(n, group)
    bounds = torch.empty((7, ng), dtype=torch.float32, device="cuda")
    keep = torch.empty((len(cams), ng), dtype=torch.uint8, device="cuda")
    B.pbdr_group_bounds(scene, group, bounds)
    splats = [B.Splats.empty(n) for _ in cams]
    g_splats = [B.SplatGrads.empty(n) for _ in cams]
    B.pbdr_preprocess_batch(scene, cams, splats, group, bounds, keep)
    cap = 7_000_000
    view = GpuView(n, cams[0], cap)
    total = None
    used = np.zeros(n, dtype=bool)
    ties = np.zeros(n, dtype=bool)
    for v, cam in enumerate(cams):
        view.cam = cam
        sp = splats[v].to_numpy()
        got_f = view.render_fwd(BG, splats=splats[v])
        lists = oracle.bin_sort(sp["mean2d"].astype(np.float64), sp["radius"], sp["depth"], W, H)
        assert lists["P"] <= cap
        gl = view.lists()
        assert gl["P_raw"] == lists["P"] and np.array_equal(gl["vals"], lists["vals"]) and np.array_equal(gl["ranges"], lists["ranges"])
        st = _state64(sp)
        ref_f = oracle.render_fwd(st, lists, W, H, BG)
        ok = ref_f["fragile"] == 0
        assert np.abs(got_f["image"] - ref_f["image"])[ok].max() <= IMG_ATOL
        # the loss: N(0,1) dL/dimage on 256 seeded tiles, among those that hold splats where the view has that many
        rng = np.random.default_rng(100 + v)
        lens = lists["ranges"][:, 1] - lists["ranges"][:, 0]
        busy = np.nonzero(lens > 0)[0]
        pool = busy if len(busy) >= 256 else np.arange(TX * TY)
        G = np.zeros((H, W, 3), dtype=np.float32)
        for t in rng.choice(pool, 256, replace=False):
            ty, tx = divmod(int(t), TX)
            y0, x0 = 16 * ty, 16 * tx
            G[y0:y0 + 16, x0:x0 + 16] = rng.normal(size=(min(16, H - y0), min(16, W - x0), 3)).astype(np.float32)
        G[~ok] = 0.0
        B.pbdr_render_bwd(None, splats[v], cam, BG, cap, view.final_T, view.last_idx, to_chw_dev(G), g_splats[v], None, view.ws)
        torch.cuda.synchronize()
        gs = g_splats[v].to_numpy()
        ref_b = oracle.render_bwd(st, lists, W, H, BG, G.astype(np.float64))
        vis = sp["radius"] > 0
        for k in ("mean2d", "conic", "opacity", "color"):
            grad_close(f"street view {v} (256 tiles) composite bwd {k}", gs[k][vis], ref_b[k][vis], report=(v == 2))
        ref_sp = oracle.preprocess(sc, cam)
        ties |= ref_sp["near_tie"] != 0
        assert np.array_equal(sp["radius"][ref_sp["near_tie"] == 0] > 0, ref_sp["radius"][ref_sp["near_tie"] == 0] > 0)
        used |= vis
        ref_g = oracle.preprocess_bwd(sc, cam, {k: gs[k].astype(np.float64) for k in ("mean2d", "conic", "opacity", "color")})
        total = ref_g if total is None else {k: total[k] + ref_g[k] for k in ("mean", "log_scale", "quat", "logit", "sh")}
    grads = scene.zeros_like()
    for k in ("mean", "log_scale", "quat", "logit", "sh"):
        getattr(grads, k).fill_(float("nan"))          # first_view: the call writes every entry
    B.pbdr_preprocess_bwd_batch(scene, cams, splats, g_splats, grads, first_view=True)
    torch.cuda.synchronize()
    got = grads.to_numpy()
    sel = used & ~ties
    for k in ("mean", "log_scale", "quat", "logit", "sh"):
        assert not got[k][~used].any()                  # points no view uses: exact zeros
        grad_close(f"eight street views accumulated {k}", got[k][sel], total[k][sel])
