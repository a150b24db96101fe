"""GPU parity for image-patch rendering (paper Sec. 4.2.2 patches of H/p x W/p; App. D.2 kernels restricted to a patch).

What a patch must be is fixed by the whole-image path, which the other GPU tests pin to the oracle:
  * forward: image / final_T / last_idx of the patch are the crop of the whole-image outputs, bit for bit;
  * visibility: a point is visible for the patch iff it is visible for the image and its tile rectangle meets the tiles
    of the patch (integer interval arithmetic, written out below); its other fields are those of the whole-image state;
  * backward: the oracle's whole-image backward fed with dL/dimage that is zero outside the patch;
  * the parameter gradients of the patches of a partition, accumulated into one buffer, are the whole-image gradient.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_pipeline import to_chw_dev, to_hwc
from helpers import IMG_ATOL, grad_close
from paper_2512_20017_amd import binding as B
from paper_2512_20017_amd import synth

pytestmark = pytest.mark.gpu
BG = [0.2, 0.1, 0.3]


def _partition(W, H, p):
    xs = [round(i * W / p) for i in range(p + 1)]
    ys = [round(i * H / p) for i in range(p + 1)]
    return [(xs[i], ys[j], xs[i + 1], ys[j + 1]) for j in range(p) for i in range(p)]


class Full:
    """Whole-image render through the HIP path, kept for cropping."""

    def __init__(self, scene, cam, cap):
        n, W, H = scene.n, cam["width"], cam["height"]
        self.cam, self.cap = cam, cap
        self.splats = B.Splats.empty(n)
        self.ws = B.alloc_workspace(n, W, H, cap)
        self.image = torch.empty((3, H, W), device="cuda"); self.final_T = torch.empty((H, W), device="cuda")
        self.last_idx = torch.empty((H, W), dtype=torch.int32, device="cuda")
        B.pbdr_preprocess(scene, cam, self.splats)
        B.pbdr_render_fwd(self.splats, cam, BG, cap, self.image, self.final_T, self.last_idx, self.ws)
        P, over = B.pbdr_query_lists(self.ws, n, W, H, cap)
        assert not over
        self.sp = self.splats.to_numpy()


def _touches(sp, patch):
    """Points whose tile rectangle (16 x 16 tiles of the image grid) meets the tiles of the patch."""
    x0, y0, x1, y1 = patch
    tx0, ty0, tx1, ty1 = x0 // 16, y0 // 16, (x1 + 15) // 16, (y1 + 15) // 16
    ix = np.floor(sp["mean2d"][:, 0]).astype(np.int64); iy = np.floor(sp["mean2d"][:, 1]).astype(np.int64)
    r = sp["radius"].astype(np.int64)
    ax0, ax1 = (ix - r) >> 4, (ix + r + 15) >> 4            # [ax0, ax1) before clamping
    ay0, ay1 = (iy - r) >> 4, (iy + r + 15) >> 4
    return (sp["radius"] > 0) & (np.maximum(ax0, tx0) < np.minimum(ax1, tx1)) & (np.maximum(ay0, ty0) < np.minimum(ay1, ty1))


def _render_patch(scene, full, patch, ws):
    x0, y0, x1, y1 = patch
    w, h = x1 - x0, y1 - y0
    n = scene.n
    splats = B.Splats.empty(n)
    splats.radius.fill_(-3)
    image = torch.full((3, h, w), -1.0, device="cuda"); final_T = torch.full((h, w), -1.0, device="cuda")
    last_idx = torch.full((h, w), -1, dtype=torch.int32, device="cuda")
    B.pbdr_preprocess_patch(scene, full.cam, patch, splats)
    B.pbdr_render_fwd_patch(splats, full.cam, patch, BG, full.cap, image, final_T, last_idx, ws)
    torch.cuda.synchronize()
    # forward: the crop, bit for bit
    assert torch.equal(image, full.image[:, y0:y1, x0:x1])
    assert torch.equal(final_T, full.final_T[y0:y1, x0:x1])
    assert torch.equal(last_idx, full.last_idx[y0:y1, x0:x1])
    # visibility and state
    sp = splats.to_numpy()
    want = _touches(full.sp, patch)
    assert np.array_equal(sp["radius"] > 0, want)
    for k in ("mean2d", "conic", "opacity", "color", "radius", "depth"):
        assert np.array_equal(sp[k][want], full.sp[k][want]), k
    return splats, sp, final_T, last_idx, want


@pytest.mark.parametrize("seed,W,H,deg", [(0, 200, 120, 1), (1, 97, 83, 0), (2, 160, 160, 3)])
def test_patches_small(seed, W, H, deg):
    sc = synth.random_small_scene(seed, 300, deg)
    cam = synth.pinhole(W, H, 55.0, np.eye(3), [0.03, -0.02, 2.4])
    scene = B.Scene.from_numpy(sc)
    n, cap = scene.n, 1 << 18
    full = Full(scene, cam, cap)
    ws = B.alloc_workspace(n, W, H, cap)
    # oracle lists / compositing on the GPU's own whole-image fp32 state
    st = {k: full.sp[k].astype(np.float64) for k in ("mean2d", "conic", "opacity", "color")}
    st["radius"] = full.sp["radius"]
    lists = oracle.bin_sort(st["mean2d"], st["radius"], full.sp["depth"], W, H)
    ref_f = oracle.render_fwd(st, lists, W, H, BG)
    ok = ref_f["fragile"] == 0
    # the whole-image render the patches are cropped from, against the oracle (the crops themselves are bit-exact)
    whole_img = full.image.permute(1, 2, 0).cpu().numpy()
    assert np.abs(whole_img - ref_f["image"])[ok].max() <= IMG_ATOL
    assert np.abs(full.final_T.cpu().numpy() - ref_f["final_T"])[ok].max() <= IMG_ATOL
    assert np.array_equal(full.last_idx.cpu().numpy().astype(np.uint32)[ok], ref_f["last_idx"][ok])
    rng = np.random.default_rng(seed)
    G = rng.normal(size=(H, W, 3)).astype(np.float32)
    G[~ok] = 0.0
    patches = _partition(W, H, 2) + _partition(W, H, 3) + [(17, 5, 18, 6), (W - 40, H - 33, W, H), (0, 0, W, H)]
    acc = {2: scene.zeros_like(), 3: scene.zeros_like(), "2, no splat-gradient output": scene.zeros_like()}
    for pi, patch in enumerate(patches):
        x0, y0, x1, y1 = patch
        splats, sp, final_T, last_idx, vis = _render_patch(scene, full, patch, ws)
        Gp = np.zeros_like(G); Gp[y0:y1, x0:x1] = G[y0:y1, x0:x1]
        ref_b = oracle.render_bwd(st, lists, W, H, BG, Gp.astype(np.float64))
        g_sp = B.SplatGrads.empty(n)
        grads = acc[2] if pi < 4 else (acc[3] if pi < 13 else scene.zeros_like())
        B.pbdr_render_bwd_patch(scene, splats, cam, patch, BG, cap, final_T, last_idx,
                                to_chw_dev(G[y0:y1, x0:x1]), g_sp, grads, ws)
        if pi < 4:      # the 2 x 2 partition once more, the splat-state gradient left in the workspace
            B.pbdr_render_bwd_patch(scene, splats, cam, patch, BG, cap, final_T, last_idx, to_chw_dev(G[y0:y1, x0:x1]), None,
                                    acc["2, no splat-gradient output"], ws)
        torch.cuda.synchronize()
        got = g_sp.to_numpy()
        for k in ("mean2d", "conic", "opacity", "color"):
            grad_close(f"patch {pi} composite bwd {k}", got[k][vis], ref_b[k][vis], report=(pi == 0))
            hidden = (full.sp["radius"] > 0) & ~vis          # visible in the image, not in the patch: no gradient
            assert not np.abs(ref_b[k][hidden]).any()
    # Alg. 1 lines 22-24 over the patches of a partition = the whole image
    whole = scene.zeros_like()
    g_sp = B.SplatGrads.empty(n)
    B.pbdr_render_bwd(scene, full.splats, cam, BG, cap, full.final_T, full.last_idx, to_chw_dev(G), g_sp, whole, full.ws)
    torch.cuda.synchronize()
    ref = whole.to_numpy()
    for p in acc:
        got = acc[p].to_numpy()
        for k in ("mean", "log_scale", "quat", "logit", "sh"):
            grad_close(f"patches summed {k}", got[k], ref[k])


def test_invalid_patches():
    sc = synth.random_small_scene(0, 64, 0)
    cam = synth.pinhole(64, 48, 55.0, np.eye(3), [0, 0, 2.4])
    scene = B.Scene.from_numpy(sc)
    out = B.Splats.empty(scene.n)
    for bad in [(-1, 0, 10, 10), (0, 0, 65, 10), (10, 10, 10, 20), (20, 10, 10, 20), (0, 0, 10, 49)]:
        with pytest.raises(B.PbdrError):
            B.pbdr_preprocess_patch(scene, cam, bad, out)


@pytest.mark.timeout(300)
def test_patches_full_size():
    sc = synth.scene_mid(0)
    scene = B.Scene.from_numpy(sc)
    cam = synth.cameras_sphere()[0]
    W, H = cam["width"], cam["height"]
    cap = 3_700_000
    full = Full(scene, cam, cap)
    ws = B.alloc_workspace(scene.n, W, H, cap)
    seen = np.zeros(scene.n, dtype=bool)
    for patch in _partition(W, H, 2) + [_partition(W, H, 8)[27]]:
        _, sp, _, _, vis = _render_patch(scene, full, patch, ws)
        seen |= vis
    assert np.array_equal(seen, full.sp["radius"] > 0)      # every visible point belongs to some patch of the partition


@pytest.mark.parametrize("seed,W,H,deg", [(0, 150, 100, 1), (3, 96, 96, 3)])
def test_surfel_patches(seed, W, H, deg):
    """2D Gaussian surfels through the same patch mechanism: crop of the whole-image forward bit for bit, backward
    against the oracle's whole-image backward with dL/dimage zero outside the patch, partition sums to the whole."""
    sc = synth.random_small_surfels(seed, 250, deg)
    cam = synth.pinhole(W, H, 55.0, np.eye(3), [0.03, -0.02, 2.4])
    scene = B.Scene2D.from_numpy(sc)
    n, cap = scene.n, 1 << 18
    full_sp = B.Splats2D.empty(n)
    full_ws = B.alloc_workspace2d(n, W, H, cap)
    image = torch.empty((3, H, W), device="cuda"); final_T = torch.empty((H, W), device="cuda")
    last_idx = torch.empty((H, W), dtype=torch.int32, device="cuda")
    B.pbdr2d_preprocess(scene, cam, full_sp)
    B.pbdr2d_render_fwd(full_sp, cam, BG, cap, image, final_T, last_idx, full_ws)
    torch.cuda.synchronize()
    fsp = full_sp.to_numpy()
    st = {k: fsp[k].astype(np.float64) for k in ("mean2d", "T", "opacity", "color")}
    st["radius"] = fsp["radius"]
    lists = oracle.bin_sort(st["mean2d"], st["radius"], fsp["depth"], W, H)
    ref_f = oracle.render_fwd2d(st, lists, W, H, BG)
    ok = ref_f["fragile"] == 0
    assert np.abs(to_hwc(image) - ref_f["image"])[ok].max() <= IMG_ATOL      # what the patches are crops of
    assert np.array_equal(last_idx.cpu().numpy().astype(np.uint32)[ok], ref_f["last_idx"][ok])
    G = np.random.default_rng(seed).normal(size=(H, W, 3)).astype(np.float32)
    G[~ok] = 0.0
    ws = B.alloc_workspace2d(n, W, H, cap)
    acc = scene.zeros_like()
    for patch in _partition(W, H, 2) + [(33, 21, 90, 64)]:
        x0, y0, x1, y1 = patch
        w, h = x1 - x0, y1 - y0
        sp = B.Splats2D.empty(n)
        img = torch.empty((3, h, w), device="cuda"); fT = torch.empty((h, w), device="cuda")
        li = torch.empty((h, w), dtype=torch.int32, device="cuda")
        B.pbdr2d_preprocess_patch(scene, cam, patch, sp)
        B.pbdr2d_render_fwd_patch(sp, cam, patch, BG, cap, img, fT, li, ws)
        torch.cuda.synchronize()
        assert torch.equal(img, image[:, y0:y1, x0:x1])
        assert torch.equal(fT, final_T[y0:y1, x0:x1])
        assert torch.equal(li, last_idx[y0:y1, x0:x1])
        psp = sp.to_numpy()
        vis = _touches(fsp, patch)
        assert np.array_equal(psp["radius"] > 0, vis)
        for k in ("mean2d", "T", "opacity", "color", "radius", "depth", "normal"):
            assert np.array_equal(psp[k][vis], fsp[k][vis]), k
        Gp = np.zeros_like(G); Gp[y0:y1, x0:x1] = G[y0:y1, x0:x1]
        ref_b = oracle.render_bwd2d(st, lists, W, H, BG, Gp.astype(np.float64))
        g_sp = B.SplatGrads2D.empty(n)
        grads = acc if patch != (33, 21, 90, 64) else scene.zeros_like()
        B.pbdr2d_render_bwd_patch(scene, sp, cam, patch, BG, cap, fT, li, to_chw_dev(G[y0:y1, x0:x1]), g_sp, grads, ws)
        torch.cuda.synchronize()
        got = g_sp.to_numpy()
        for k in ("mean2d", "opacity", "color"):
            grad_close(f"surfel patch {patch} composite bwd {k}", got[k][vis], ref_b[k][vis], report=False)
        for row in range(3):      # the rows of T differ by the focal length in magnitude
            grad_close(f"surfel patch {patch} T{row}", got["T"][vis][:, 3 * row:3 * row + 3], ref_b["T"][vis][:, 3 * row:3 * row + 3],
                       report=False)
    whole = scene.zeros_like()
    g_sp = B.SplatGrads2D.empty(n)
    B.pbdr2d_render_bwd(scene, full_sp, cam, BG, cap, final_T, last_idx, to_chw_dev(G), g_sp, whole, full_ws)
    torch.cuda.synchronize()
    ref, got = whole.to_numpy(), acc.to_numpy()
    for k in ("mean", "tan_u", "tan_v", "log_scale", "logit", "sh"):
        grad_close(f"patches summed {k}", got[k], ref[k])


@pytest.mark.parametrize("surfels", [False, True])
def test_whole_image_state_through_a_patch_ignores_unlisted_splat_gradients(surfels):
    """A state written by the whole-image preprocessing call has radius > 0 for points whose tiles miss the patch.
    Binning for the patch never lists them, so their g_splats entries are not written by the backward; the parameter
    gradient must not depend on what those entries held (here: NaN), and must equal the one from the patch's own state."""
    W, H, n, cap = 240, 180, 600, 1 << 18
    patch = (100, 70, 130, 90)
    x0, y0, x1, y1 = patch
    cam = synth.pinhole(W, H, 55.0, np.eye(3), [0.03, -0.02, 2.4])
    if surfels:
        sc = synth.random_small_surfels(7, n, 2, spread=1.0, ls_mu=-3.2); scene = B.Scene2D.from_numpy(sc)
        mk_sp, mk_g, alloc = B.Splats2D.empty, B.SplatGrads2D.empty, B.alloc_workspace2d
        pre, pre_p, fwd_p, bwd_p = B.pbdr2d_preprocess, B.pbdr2d_preprocess_patch, B.pbdr2d_render_fwd_patch, B.pbdr2d_render_bwd_patch
        keys, state_keys = ("mean", "tan_u", "tan_v", "log_scale", "logit", "sh"), ("mean2d", "T", "opacity", "color")
    else:
        sc = synth.random_small_scene(7, n, 2, spread=1.0, ls_mu=-3.4); scene = B.Scene.from_numpy(sc)
        mk_sp, mk_g, alloc = B.Splats.empty, B.SplatGrads.empty, B.alloc_workspace
        pre, pre_p, fwd_p, bwd_p = B.pbdr_preprocess, B.pbdr_preprocess_patch, B.pbdr_render_fwd_patch, B.pbdr_render_bwd_patch
        keys, state_keys = ("mean", "log_scale", "quat", "logit", "sh"), ("mean2d", "conic", "opacity", "color")
    G = to_chw_dev(np.random.default_rng(1).normal(size=(y1 - y0, x1 - x0, 3)).astype(np.float32))
    results = []
    for whole_state in (False, True):
        sp = mk_sp(n)
        if whole_state:
            pre(scene, cam, sp)
        else:
            pre_p(scene, cam, patch, sp)
        ws = alloc(n, W, H, cap)
        image = torch.empty((3, y1 - y0, x1 - x0), device="cuda"); fT = torch.empty((y1 - y0, x1 - x0), device="cuda")
        li = torch.empty((y1 - y0, x1 - x0), dtype=torch.int32, device="cuda")
        fwd_p(sp, cam, patch, BG, cap, image, fT, li, ws)
        g_sp = mk_g(n)
        for k in state_keys:
            getattr(g_sp, "T" if k == "T" else k).fill_(float("nan"))
        grads = scene.zeros_like()
        for k in keys:
            getattr(grads, k).fill_(float("nan"))          # first_view: every entry is written
        bwd_p(scene, sp, cam, patch, BG, cap, fT, li, G, g_sp, grads, ws, first_view=True)
        torch.cuda.synchronize()
        results.append((sp.to_numpy()["radius"] > 0, image.clone(), grads.to_numpy(), g_sp.to_numpy()))
    (vis_p, img_p, g_p, _), (vis_w, img_w, g_w, gsp_w) = results
    assert (vis_w & ~vis_p).sum() > 10                      # points the patch does not list although radius > 0
    assert torch.equal(img_p, img_w)
    for k in keys:
        assert np.isfinite(g_w[k]).all(), k
        # (not bit for bit: the order of a tile's four wavefronts' adds into the shared accumulators is not fixed)
        np.testing.assert_allclose(g_w[k], g_p[k], rtol=1e-5, atol=1e-6 * np.abs(g_p[k]).max(), err_msg=k)
        assert not g_w[k][~vis_p].any(), k                  # no gradient for points the patch does not use
    for k in state_keys:                                    # unlisted points: left untouched, as the header says
        assert np.isnan(gsp_w[k][vis_w & ~vis_p]).all() and np.isfinite(gsp_w[k][vis_p]).all(), k
