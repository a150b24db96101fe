"""The order in which the compositing kernels take the tiles (an implementation detail of the launch: Sec. 2.1
composites every tile independently, so no result depends on it; the parity tests cover that). Checked here against
its definition in the header: a permutation of the call's tiles, longer lists first by class of list length, image
order within a class. The expected order is computed from the tile ranges with numpy."""
import numpy as np
import pytest
import torch

from paper_2512_20017_amd import binding as B
from paper_2512_20017_amd import synth

pytestmark = pytest.mark.gpu


def _classes(length):
    x = length.astype(np.int64) + 1
    e = np.floor(np.log2(x)).astype(np.int64)
    e = np.where((1 << (e + 1)) <= x, e + 1, e)           # guard the floating-point log at powers of two
    e = np.where((1 << e) > x, e - 1, e)
    half = np.where(e > 0, (x >> np.maximum(e - 1, 0)) & 1, 0)
    return np.minimum(2 * e + half, 39)


def _expected(ranges, tiles):
    cls = _classes(ranges[:tiles, 1].astype(np.int64) - ranges[:tiles, 0].astype(np.int64))
    return np.lexsort((np.arange(tiles), -cls)).astype(np.uint32)


def _camera(W, H, eye=(0.2, -0.1, -3.0)):
    R, t = synth.look_at(eye, (0.0, 0.0, 0.0), (0.0, 1.0, 0.0))
    return synth.pinhole(W, H, 55.0, R, t)


@pytest.mark.parametrize("W,H,n", [(16, 16, 50), (128, 128, 4096), (640, 360, 20000), (1031, 517, 30000), (2050, 1030, 50000),
                                   (3840, 2160, 20000)])
def test_order_is_the_definition(W, H, n):
    sc = synth.random_small_scene(W + n, n, 0, spread=1.2, ls_mu=-3.0)
    scene = B.Scene.from_numpy(sc)
    cam = _camera(W, H)
    cap = 4_000_000
    splats = B.Splats.empty(n)
    ws = B.alloc_workspace(n, W, H, cap)
    B.pbdr_preprocess(scene, cam, splats)
    B.pbdr_bin_sort(splats, cam, cap, ws)
    tiles = ((W + 15) // 16) * ((H + 15) // 16)
    lv = B.pbdr_lists_view(ws, n, W, H, cap)
    got = B.pbdr_tile_order_view(ws, n, W, H, cap, tiles)
    assert np.array_equal(np.sort(got), np.arange(tiles, dtype=np.uint32))
    assert np.array_equal(got, _expected(lv["ranges"], tiles))
    if tiles > 64:
        assert len(np.unique(_classes(lv["ranges"][:, 1].astype(np.int64) - lv["ranges"][:, 0]))) > 2      # the case orders something


def test_order_of_a_patch_covers_the_patch_grid_only():
    W, H, n = 640, 360, 20000
    sc = synth.random_small_scene(3, n, 0, spread=1.2, ls_mu=-3.0)
    scene = B.Scene.from_numpy(sc)
    cam = _camera(W, H)
    cap = 2_000_000
    patch = (100, 40, 371, 233)
    w, h = patch[2] - patch[0], patch[3] - patch[1]
    splats = B.Splats.empty(n)
    ws = B.alloc_workspace(n, W, H, cap)
    image = torch.empty((3, h, w), device="cuda")
    T = torch.empty((h, w), device="cuda")
    last = torch.empty((h, w), dtype=torch.int32, device="cuda")
    B.pbdr_preprocess_patch(scene, cam, patch, splats)
    B.pbdr_render_fwd_patch(splats, cam, patch, [0, 0, 0], cap, image, T, last, ws)
    tx = (patch[2] + 15) // 16 - patch[0] // 16
    ty = (patch[3] + 15) // 16 - patch[1] // 16
    lv = B.pbdr_lists_view(ws, n, W, H, cap)
    got = B.pbdr_tile_order_view(ws, n, W, H, cap, tx * ty)
    assert np.array_equal(got, _expected(lv["ranges"], tx * ty))


def test_no_points_gives_the_image_order():
    W, H = 200, 100
    cam = _camera(W, H)
    ws = B.alloc_workspace(0, W, H, 1000)
    ws.fill_(0xAB)
    image = torch.empty((3, H, W), device="cuda")
    T = torch.empty((H, W), device="cuda")
    last = torch.empty((H, W), dtype=torch.int32, device="cuda")
    splats = B.Splats.empty(0)
    B.pbdr_render_fwd(splats, cam, [0.5, 0.25, 0.125], 1000, image, T, last, ws)
    tiles = 13 * 7
    assert np.array_equal(B.pbdr_tile_order_view(ws, 0, W, H, 1000, tiles), np.arange(tiles, dtype=np.uint32))
    assert float(image[0].min()) == 0.5 and float(image[2].max()) == 0.125 and float(T.min()) == 1.0


def test_surfel_workspace_has_its_own_order():
    W, H, n = 320, 200, 5000
    ss = synth.random_small_surfels(4, n, 0)
    scene = B.Scene2D.from_numpy(ss)
    cam = _camera(W, H)
    cap = 2_000_000
    splats = B.Splats2D.empty(n)
    ws = B.alloc_workspace2d(n, W, H, cap)
    image = torch.empty((3, H, W), device="cuda")
    T = torch.empty((H, W), device="cuda")
    last = torch.empty((H, W), dtype=torch.int32, device="cuda")
    B.pbdr2d_preprocess(scene, cam, splats)
    B.pbdr2d_render_fwd(splats, cam, [0, 0, 0], cap, image, T, last, ws)
    tiles = 20 * 13
    lv = B.pbdr2d_lists_view(ws, n, W, H, cap)
    got = B.pbdr_tile_order_view(ws, n, W, H, cap, tiles, surfels=True)
    assert np.array_equal(got, _expected(lv["ranges"], tiles))
