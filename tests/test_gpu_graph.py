"""A whole training step recorded once into a HIP graph and replayed: the library's calls are kernel launches on the
caller's stream and nothing else (no allocation, no host read-back, no memset node, every count that sizes later work
stays on the device), so a captured step must give on every replay what the same calls give when issued one by one.

The step is Alg. 1's per-view part: splat, render, L1 loss, backward (lines 2-4, 5-12, 13, 16-24), optionally followed by
the selective Adam step (line 27). Between replays the inputs change in place (target image, point parameters) and the
program does its own eager work and synchronisations; every replay is compared with the eager result for the same inputs.
Image, final transmittance and last index: bit for bit. Gradients: to the rounding of the backward kernel's LDS adds,
whose order among a tile's four wavefronts is not fixed (1e-5 of the largest entry), as in the test of views in flight
on separate streams.
"""
import numpy as np
import pytest
import torch

from paper_2512_20017_amd import binding as B
from paper_2512_20017_amd import synth

pytestmark = pytest.mark.gpu

W, H, N, CAP = 640, 360, 20000, 2_000_000


def _cam(eye=(0.3, -0.2, -3.0)):
    R, t = synth.look_at(eye, (0.0, 0.0, 0.0), (0.0, 1.0, 0.0))
    return synth.pinhole(W, H, 55.0, R, t)


def _params(scene):
    return torch.cat([t.reshape(-1) for t in (scene.mean, scene.log_scale, scene.quat, scene.logit, scene.sh)])


def _buffers(scene):
    return dict(splats=B.Splats.empty(N), grads=scene.zeros_like(), image=torch.empty((3, H, W), device="cuda"),
                T=torch.empty((H, W), device="cuda"), last=torch.empty((H, W), dtype=torch.int32, device="cuda"),
                dL=torch.empty((3, H, W), device="cuda"), loss=torch.zeros((1,), device="cuda"),
                ws=B.alloc_workspace(N, W, H, CAP))


def _step(scene, cam, bg, target, c):
    B.pbdr_preprocess(scene, cam, c["splats"])
    B.pbdr_render_fwd(c["splats"], cam, bg, CAP, c["image"], c["T"], c["last"], c["ws"])
    B.pbdr_l1_loss(c["image"], target, c["loss"], c["dL"])
    B.pbdr_render_bwd(scene, c["splats"], cam, bg, CAP, c["T"], c["last"], c["dL"], None, c["grads"], c["ws"], first_view=True)


def _same(got, ref):
    assert torch.equal(got["image"], ref["image"])
    assert torch.equal(got["T"], ref["T"])
    assert torch.equal(got["last"], ref["last"])
    assert torch.equal(got["dL"], ref["dL"])
    a, b = got["grads"].flat, ref["grads"].flat
    assert float(b.abs().max()) > 0
    assert float((a - b).abs().max()) <= 1e-5 * float(b.abs().max())


def test_captured_step_replays_like_the_eager_step():
    sc = synth.random_small_scene(17, N, 2, spread=1.0, ls_mu=-3.2)
    scene = B.Scene.from_numpy(sc)
    cam, bg = _cam(), [0.1, 0.2, 0.3]
    rng = np.random.default_rng(5)
    target = torch.from_numpy(rng.uniform(size=(3, H, W)).astype(np.float32)).cuda()
    ref, got = _buffers(scene), _buffers(scene)

    _step(scene, cam, bg, target, got)             # every kernel has run once before anything is recorded
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _step(scene, cam, bg, target, got)
    torch.cuda.synchronize()

    for rep in range(4):
        if rep:                                     # new inputs, written in place: the graph holds addresses only
            target.copy_(torch.from_numpy(rng.uniform(size=(3, H, W)).astype(np.float32)).cuda())
            scene.mean.add_(torch.from_numpy(rng.normal(scale=0.01, size=(3, N)).astype(np.float32)).cuda())
            for k in ("image", "T", "dL"):         # stale outputs must not pass for new ones
                got[k].fill_(-7.0)
            got["last"].fill_(-7)
            got["grads"].flat.fill_(-7.0)
        got["loss"].zero_()
        ref["loss"].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _step(scene, cam, bg, target, ref)
        torch.cuda.synchronize()
        _same(got, ref)
        assert float(got["loss"].item()) == pytest.approx(float(ref["loss"].item()), rel=2e-6)
        assert float(ref["loss"].item()) > 0


def test_captured_training_iteration_with_fused_adam():
    """Batched preprocessing, two views rendered one after the other, and the backward pass that ends in the Adam step:
    replays advance the parameters exactly as the same calls issued eagerly do on a copy of the state."""
    sc = synth.random_small_scene(23, N, 1, spread=1.0, ls_mu=-3.2)
    cams = [_cam(), _cam((2.0, 0.4, -2.2))]
    bg = [0.0, 0.0, 0.0]
    rng = np.random.default_rng(6)
    targets = [torch.from_numpy(rng.uniform(size=(3, H, W)).astype(np.float32)).cuda() for _ in cams]
    lrs = [1.6e-4, 5e-3, 1e-3, 5e-2, 2.5e-3]            # mean, log-scale, rotation, opacity logit, SH

    def state():
        scene = B.Scene.from_numpy(sc)
        return dict(scene=scene, m=scene.zeros_like(), v=scene.zeros_like(),
                    views=[dict(_buffers(scene), g2=B.SplatGrads.empty(N)) for _ in cams])

    def iteration(s, step):
        splats = [c["splats"] for c in s["views"]]
        B.pbdr_preprocess_batch(s["scene"], cams, splats)
        for cam, tgt, c in zip(cams, targets, s["views"]):
            B.pbdr_render_fwd(c["splats"], cam, bg, CAP, c["image"], c["T"], c["last"], c["ws"])
            B.pbdr_l1_loss(c["image"], tgt, c["loss"], c["dL"])
            B.pbdr_render_bwd(None, c["splats"], cam, bg, CAP, c["T"], c["last"], c["dL"], c["g2"], None, c["ws"])
        B.pbdr_preprocess_bwd_batch_adam(s["scene"], cams, splats, [c["g2"] for c in s["views"]], s["m"], s["v"], lrs,
                                         0.9, 0.999, 1e-8, step)

    ref, got, warm = state(), state(), state()
    start = _params(ref["scene"]).clone()
    iteration(warm, 1)                              # every kernel has run once before anything is recorded
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        iteration(got, 1)
    torch.cuda.synchronize()
    assert torch.equal(_params(got["scene"]), start)            # capture records, it does not run

    def reset(s):
        for name in ("mean", "log_scale", "quat", "logit", "sh"):
            getattr(s["scene"], name).copy_(getattr(warm0, name))
        s["m"].flat.zero_()
        s["v"].flat.zero_()

    warm0 = B.Scene.from_numpy(sc)
    for rep in range(3):
        # the step number is a kernel argument (Adam's bias correction), so a recorded iteration is "step 1" for good:
        # each replay starts from the initial parameters and zero moments, as does the eager run it is compared with
        reset(got)
        reset(ref)
        for c in got["views"]:
            c["image"].fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        iteration(ref, 1)
        torch.cuda.synchronize()
        for a, b in zip(got["views"], ref["views"]):
            assert torch.equal(a["image"], b["image"]) and torch.equal(a["last"], b["last"])
        p, q = _params(got["scene"]), _params(ref["scene"])
        moved = (q != start)
        assert int(moved.sum()) > 1000
        # the first Adam step moves an entry by lr * g / (|g| + eps): the two sides' gradients differ by the rounding of
        # the backward kernel's LDS adds, which matters only where the gradient is itself rounding noise (|g| near eps)
        differ = (p - q).abs() > 1e-6
        assert float((p - q).abs().max()) <= 2.2 * max(lrs)
        assert int(differ.sum()) <= 0.01 * int(moved.sum())
