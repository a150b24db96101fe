"""GPU parity for the loss and the optimizer step (paper Alg. 1 lines 13, 16, 27) through the C ABI, against the oracle.

Tolerances: dL/dimage is a sign times 1/(3HW): exact up to the fp32 rounding of that constant (the sign of a
difference of two fp32 numbers is the same in fp32 and fp64). The loss is a sum of ~1e7 fp32 terms formed pairwise per
workgroup and by float atomics across workgroups: 2e-6 relative. Adam: each of m, v is two roundings per step
(2e-7 relative + the same of the increment); the parameter moves by at most about lr per step, computed to ~1e-6
relative, on top of its own rounding.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_20017_amd import binding as B
from paper_2512_20017_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("W,H", [(1, 1), (5, 3), (64, 48), (333, 77), (1920, 1080)])
def test_l1_loss(W, H):
    rng = np.random.default_rng(W * 7 + H)
    img = rng.uniform(size=(3, H, W)).astype(np.float32)
    tgt = rng.uniform(size=(3, H, W)).astype(np.float32)
    eq = rng.uniform(size=(3, H, W)) < 0.1
    tgt[eq] = img[eq]                                      # equal values: zero gradient
    d_img, d_tgt = torch.from_numpy(img).cuda(), torch.from_numpy(tgt).cuda()
    loss = torch.full((1,), 0.25, device="cuda")          # accumulates
    dL = torch.full((3, H, W), 9.0, device="cuda")
    B.pbdr_l1_loss(d_img, d_tgt, loss, dL)
    B.pbdr_l1_loss(d_img, d_tgt, loss, dL)
    torch.cuda.synchronize()
    ref_loss, ref_g = oracle.l1_loss(img.transpose(1, 2, 0), tgt.transpose(1, 2, 0))
    assert float(loss.item()) == pytest.approx(0.25 + 2 * ref_loss, rel=2e-6)
    got = dL.cpu().numpy().transpose(1, 2, 0)
    np.testing.assert_allclose(got, ref_g, rtol=1e-7, atol=0)
    assert (got[eq.transpose(1, 2, 0)] == 0).all()


def _adam_case(n, planes, steps, seed, zero_grad):
    rng = np.random.default_rng(seed)
    # the boundary takes the hyper-parameters as fp32: the oracle gets the same (rounded) numbers
    lr, b1, b2, eps = (float(np.float32(x)) for x in (1.6e-3, 0.9, 0.999, 1e-8))
    p = rng.normal(size=(planes, n)).astype(np.float32)
    m = np.zeros_like(p); v = np.zeros_like(p)
    dp, dm, dv = (torch.from_numpy(a.copy()).cuda() for a in (p, m, v))
    for t in range(1, steps + 1):
        g = (rng.normal(size=(planes, n)) * 10.0 ** rng.uniform(-4, 0, size=(planes, 1))).astype(np.float32)
        vis = (rng.uniform(size=n) < (0.5 if t != 2 else 0.02)).astype(np.uint8)
        if t == 3:
            vis[:] = 0
            vis[n // 2] = 1
        g[:, vis == 0] = 0.0          # nothing accumulates into points no view used
        dg = torch.from_numpy(g.copy()).cuda()
        dvis = torch.from_numpy(vis).cuda()
        p0, m0, v0 = dp.cpu().numpy(), dm.cpu().numpy(), dv.cpu().numpy()
        B.pbdr_adam_selective(dp, dg, dm, dv, dvis, lr, b1, b2, eps, t, zero_grad=zero_grad)
        torch.cuda.synchronize()
        rp, rm, rv = oracle.adam_selective(p0.T, g.T, m0.T, v0.T, vis, lr, b1, b2, eps, t)
        gp, gm, gv = dp.cpu().numpy(), dm.cpu().numpy(), dv.cpu().numpy()
        hid = vis == 0
        assert np.array_equal(gp[:, hid], p0[:, hid]) and np.array_equal(gm[:, hid], m0[:, hid]) and np.array_equal(gv[:, hid], v0[:, hid])
        # m is a sum of two terms that may cancel: the bound is relative to their magnitudes, not to the result
        assert (np.abs(gm - rm.T) <= 3e-7 * (b1 * np.abs(m0) + (1 - b1) * np.abs(g)) + 1e-30).all()
        np.testing.assert_allclose(gv, rv.T, rtol=4e-7, atol=1e-20)
        assert (np.abs(gp - rp.T) <= 2e-6 * lr + 1.2e-7 * np.abs(rp.T)).all()
        if zero_grad:
            assert not dg.any().item()
        else:
            assert torch.equal(dg.cpu(), torch.from_numpy(g))


@pytest.mark.parametrize("n,planes,zero_grad", [(4096, 3, False), (100003, 1, True), (100000, 48, True), (7, 4, False), (1, 1, True)])
def test_adam_selective(n, planes, zero_grad):
    _adam_case(n, planes, 4, n + planes, zero_grad)


def test_mark_visible_is_the_union_over_views():
    sc = synth.random_small_scene(5, 3000, 0)
    scene = B.Scene.from_numpy(sc)
    visible = torch.zeros(scene.n, dtype=torch.uint8, device="cuda")
    want = np.zeros(scene.n, dtype=bool)
    seen_by = []
    for k, shift in enumerate(((-0.45, 0.0), (0.45, 0.0), (0.0, 0.45))):
        cam = synth.pinhole(64 + 16 * k, 48, 12.0, np.eye(3), [shift[0], shift[1], 2.4])
        sp = B.Splats.empty(scene.n)
        B.pbdr_preprocess(scene, cam, sp)
        B.pbdr_mark_visible(sp.radius, visible)
        seen_by.append(sp.radius.cpu().numpy() > 0)
        want |= seen_by[-1]
    torch.cuda.synchronize()
    assert np.array_equal(visible.cpu().numpy() != 0, want)
    assert all(0 < s.sum() < want.sum() for s in seen_by) and want.sum() < scene.n


def test_invalid_arguments():
    t = torch.zeros(16, device="cuda")
    vis = torch.ones(16, dtype=torch.uint8, device="cuda")
    for kw in [dict(step=0), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=0.0), dict(lr=-1.0)]:
        args = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, step=1)
        args.update(kw)
        with pytest.raises(B.PbdrError):
            B.pbdr_adam_selective(t, t.clone(), t.clone(), t.clone(), vis, **args)


@pytest.mark.timeout(300)
def test_training_iteration_full_size():
    """Alg. 1 on one GPU for one view of the 1M-point scene: splat, render, loss, backward, selective Adam with the
    gradient zeroed for the next iteration; parameters against the oracle's Adam fed with the GPU's own gradient."""
    sc = synth.scene_mid(0)
    scene = B.Scene.from_numpy(sc)
    cam = synth.cameras_sphere()[0]
    W, H, n, cap = cam["width"], cam["height"], scene.n, 3_700_000
    splats = B.Splats.empty(n); g_sp = B.SplatGrads.empty(n); ws = B.alloc_workspace(n, W, H, cap)
    image = torch.empty((3, H, W), device="cuda"); final_T = torch.empty((H, W), device="cuda")
    last_idx = torch.empty((H, W), dtype=torch.int32, device="cuda")
    target = torch.from_numpy(np.ascontiguousarray(synth.target_image(0, W, H).transpose(2, 0, 1))).cuda()
    dL = torch.empty_like(image); loss = torch.zeros(1, device="cuda")
    grads = scene.zeros_like(); m1 = scene.zeros_like(); m2 = scene.zeros_like()
    visible = torch.zeros(n, dtype=torch.uint8, device="cuda")
    bg = [0.0, 0.0, 0.0]
    B.pbdr_preprocess(scene, cam, splats)
    B.pbdr_mark_visible(splats.radius, visible)
    B.pbdr_render_fwd(splats, cam, bg, cap, image, final_T, last_idx, ws)
    B.pbdr_l1_loss(image, target, loss, dL)
    B.pbdr_render_bwd(scene, splats, cam, bg, cap, final_T, last_idx, dL, g_sp, grads, ws)
    torch.cuda.synchronize()
    ref_loss, ref_dL = oracle.l1_loss(image.permute(1, 2, 0).cpu().numpy(), target.permute(1, 2, 0).cpu().numpy())
    assert float(loss.item()) == pytest.approx(ref_loss, rel=2e-6)
    np.testing.assert_allclose(dL.permute(1, 2, 0).cpu().numpy(), ref_dL, rtol=1e-7)
    vis = visible.cpu().numpy()
    assert np.array_equal(vis != 0, splats.radius.cpu().numpy() > 0)
    lrs = dict(mean=1.6e-4, log_scale=5e-3, quat=1e-3, logit=5e-2, sh=2.5e-3)
    for k, lr in lrs.items():
        p, g = getattr(scene, k), getattr(grads, k)
        p0, g0 = p.cpu().numpy(), g.cpu().numpy()
        lr, b1, b2, eps = (float(np.float32(x)) for x in (lr, 0.9, 0.999, 1e-15))
        B.pbdr_adam_selective(p, g, getattr(m1, k), getattr(m2, k), visible, lr, b1, b2, eps, 1, zero_grad=True)
        torch.cuda.synchronize()
        P0 = p0.reshape(-1, n).T; G0 = g0.reshape(-1, n).T
        rp, rm, rv = oracle.adam_selective(P0, G0, np.zeros_like(P0), np.zeros_like(P0), vis, lr, b1, b2, eps, 1)
        got = p.cpu().numpy().reshape(-1, n).T
        assert (np.abs(got - rp) <= 2e-6 * lr + 1.2e-7 * np.abs(rp)).all(), k
        assert np.array_equal(got[vis == 0], P0[vis == 0])
        assert not g.any().item()
        assert (np.abs(got - P0)[vis != 0].max() > 0.5 * lr)       # the step really moved the visible points


@pytest.mark.parametrize("deg,n,views", [(1, 1500, 1), (3, 2500, 4), (0, 777, 16)])
def test_fused_batch_backward_and_adam_is_the_unfused_sequence(deg, n, views):
    """pbdr_preprocess_bwd_batch_adam against pbdr_preprocess_bwd_batch (first view) + pbdr_mark_visible per view +
    pbdr_adam_selective per attribute: parameters and both moments bit for bit, over two consecutive steps; points no
    view uses keep their parameters and moments."""
    sc = synth.random_small_scene(40 + deg, n, deg, spread=1.3, ls_mu=-2.8)
    cams = []
    for k in range(views):
        a = 2 * np.pi * k / views + 0.2
        cams.append(synth.pinhole(160, 96, 55.0, *synth.look_at([3 * np.cos(a), 0.3, 3 * np.sin(a)], [0, 0, 0], [0, 1, 0])))
    rng = np.random.default_rng(12)
    lrs = (1.6e-4, 5e-3, 1e-3, 5e-2, 2.5e-3)
    names = ("mean", "log_scale", "quat", "logit", "sh")

    def fresh():
        scene = B.Scene.from_numpy(sc)
        m, v = scene.zeros_like(), scene.zeros_like()
        m.flat.copy_(torch.from_numpy(np.random.default_rng(1).normal(size=m.flat.shape).astype(np.float32) * 1e-3).cuda())
        v.flat.copy_(torch.from_numpy(np.random.default_rng(2).uniform(size=v.flat.shape).astype(np.float32) * 1e-4).cuda())
        return scene, m, v

    s_ref, m_ref, v_ref = fresh()
    s_got, m_got, v_got = fresh()
    start = s_ref.to_numpy()
    used_any = np.zeros(n, dtype=bool)
    for step in (1, 2):
        g2_np = []
        for _ in cams:
            d = dict(mean2d=rng.normal(size=(n, 2)), conic=rng.normal(size=(n, 3)) * 10, opacity=rng.normal(size=n),
                     color=rng.normal(size=(n, 3)))
            g2_np.append({k: x.astype(np.float32) for k, x in d.items()})
        # unfused
        splats = []
        visible = torch.zeros(n, dtype=torch.uint8, device="cuda")
        for cam in cams:
            sp = B.Splats.empty(n)
            B.pbdr_preprocess(s_ref, cam, sp)
            B.pbdr_mark_visible(sp.radius, visible)
            splats.append(sp)
        g2s = [B.SplatGrads.from_numpy(d) for d in g2_np]
        grads = s_ref.zeros_like()
        grads.flat.fill_(float("nan"))
        B.pbdr_preprocess_bwd_batch(s_ref, cams, splats, g2s, grads, first_view=True)
        for k, lr in zip(names, lrs):
            B.pbdr_adam_selective(getattr(s_ref, k), getattr(grads, k), getattr(m_ref, k), getattr(v_ref, k), visible, lr, 0.9, 0.999,
                                  1e-15, step)
        used_any |= visible.cpu().numpy() != 0
        # fused (its own preprocessing: its parameters must follow the same trajectory)
        splats2 = []
        for cam in cams:
            sp = B.Splats.empty(n)
            B.pbdr_preprocess(s_got, cam, sp)
            splats2.append(sp)
        B.pbdr_preprocess_bwd_batch_adam(s_got, cams, splats2, g2s, m_got, v_got, lrs, 0.9, 0.999, 1e-15, step)
        torch.cuda.synchronize()
        for k in names:
            assert torch.equal(getattr(s_got, k), getattr(s_ref, k)), (step, k)
            assert torch.equal(getattr(m_got, k), getattr(m_ref, k)), (step, k)
            assert torch.equal(getattr(v_got, k), getattr(v_ref, k)), (step, k)
    assert 0 < used_any.sum() < n
    end = s_got.to_numpy()
    for k in names:
        assert np.array_equal(end[k][~used_any], start[k][~used_any]), k
        assert not np.array_equal(end[k][used_any], start[k][used_any]), k
