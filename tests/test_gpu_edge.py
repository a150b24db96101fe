"""GPU edge cases through the C ABI: empty and degenerate inputs, adversarial sort keys, capacity overflow."""
import numpy as np
import pytest
import torch

import oracle
from gpu_pipeline import GpuView
from helpers import grad_close
from paper_2512_20017_amd import binding as B
from paper_2512_20017_amd import synth

pytestmark = pytest.mark.gpu


def _cam(w, h):
    return synth.pinhole(w, h, 60.0, np.eye(3), [0.0, 0.0, 3.0])


def _lists_case(st, depth, w, h, cap=None):
    """st: host splat dict (mean2d[n,2], conic, opacity, color, radius); returns (gpu lists, oracle lists, view)."""
    st = dict(st); st["depth"] = np.asarray(depth, dtype=np.float32)
    n = len(st["opacity"])
    ref = oracle.bin_sort(np.asarray(st["mean2d"], dtype=np.float32).astype(np.float64), np.asarray(st["radius"], dtype=np.int32),
                          st["depth"], w, h)
    view = GpuView(n, _cam(w, h), cap if cap is not None else max(ref["P"], 1))
    view.splats = B.Splats.from_numpy(st)
    B.pbdr_bin_sort(view.splats, view.cam, view.cap, view.ws)
    return view.lists(), ref, view


def _rand_state(rng, n, w, h, rmax=60):
    return dict(mean2d=np.stack([rng.uniform(-20, w + 20, n), rng.uniform(-20, h + 20, n)], 1).astype(np.float32),
                conic=np.tile([0.02, 0.0, 0.02], (n, 1)).astype(np.float32), opacity=rng.uniform(0.05, 0.9, n).astype(np.float32),
                color=rng.uniform(0, 1, (n, 3)).astype(np.float32), radius=rng.integers(0, rmax, n).astype(np.int32))


@pytest.mark.parametrize("w,h,n,seed", [(64, 64, 500, 0), (200, 120, 3000, 1), (33, 17, 100, 2), (1920, 1080, 20000, 3)])
def test_lists_random_states_with_ties(w, h, n, seed):
    rng = np.random.default_rng(seed)
    st = _rand_state(rng, n, w, h)
    depth = rng.uniform(0.3, 50, n).astype(np.float32)
    depth[rng.integers(0, n, n // 3)] = depth[0]         # many exact ties -> order must fall back to the index
    got, ref, _ = _lists_case(st, depth, w, h)
    assert got["P_raw"] == ref["P"]
    assert np.array_equal(got["keys"], ref["keys"])
    assert np.array_equal(got["vals"], ref["vals"])
    assert np.array_equal(got["ranges"], ref["ranges"])


@pytest.mark.parametrize("n", [262144, 262145, 263000, 1048577 + 256, 2097152 + 300])
def test_lists_point_counts_around_a_scan_chunk(n):
    """The block scan and the packing order are made by one workgroup per 1,024 blocks of 256 points, each adding up what
    precedes its chunk by itself: point counts of exactly one chunk, one point more, a short second chunk, and a fifth
    chunk of two blocks, and just past two million points (from where a workgroup takes 4,096 blocks), with heavy and
    light blocks mixed (a few splats of large radius)."""
    rng = np.random.default_rng(n % 1000)
    w, h = 640, 360
    st = _rand_state(rng, n, w, h, rmax=3)
    big = rng.integers(0, n, 40)
    st["radius"][big] = rng.integers(100, 400, 40)
    st["radius"][rng.integers(0, n, n // 2)] = 0
    depth = rng.uniform(0.3, 50, n).astype(np.float32)
    got, ref, _ = _lists_case(st, depth, w, h)
    assert got["P_raw"] == ref["P"]
    assert np.array_equal(got["vals"], ref["vals"])
    assert np.array_equal(got["keys"], ref["keys"])
    assert np.array_equal(got["ranges"], ref["ranges"])


def test_lists_all_equal_depth_one_tile():
    n = 5000                                               # one tile, one depth: pure index order, several sort blocks
    st = dict(mean2d=np.full((n, 2), 8.0, dtype=np.float32), conic=np.tile([0.1, 0, 0.1], (n, 1)), opacity=np.full(n, 0.01),
              color=np.zeros((n, 3)), radius=np.full(n, 3, dtype=np.int32))
    got, ref, _ = _lists_case(st, np.full(n, 2.5), 16, 16)
    assert got["vals"].tolist() == list(range(n))
    assert got["ranges"].tolist() == [[0, n]]
    assert np.array_equal(got["keys"], ref["keys"])


@pytest.mark.parametrize("n", [2, 3, 63, 64, 65, 257, 511, 600, 1021, 1022, 1023, 2048, 2049, 4097, 6400, 6401, 9000, 70001])
@pytest.mark.parametrize("kind", ["narrow", "wide", "two_values", "wide_short_runs"])
def test_one_crowded_tile_depth_order(n, kind):
    """Every splat in one tile: the list's depth order is made by one workgroup - by counting up to 256 entries, in LDS up
    to 2048, through the global scratch arrays beyond - over the bit positions in which the depths differ: depths from a
    narrow band (few differing bits), from many octaves (all exponent bits differ), and only two distinct values; a
    third of the entries tied in each of these, so that the order among equals (point index) is exercised too; and depths over
    many octaves with short runs of near-equal values out of point order."""
    rng = np.random.default_rng(n * 7 + len(kind))
    st = dict(mean2d=rng.uniform(17.0, 30.0, (n, 2)).astype(np.float32), conic=np.tile([0.1, 0, 0.1], (n, 1)),
              opacity=np.full(n, 0.01), color=np.zeros((n, 3)), radius=np.full(n, 1, dtype=np.int32))
    if kind == "narrow":
        depth = rng.uniform(7.0, 7.01, n).astype(np.float32)
    elif kind == "wide":
        depth = np.exp(rng.uniform(np.log(1e-3), np.log(1e9), n)).astype(np.float32)
    elif kind == "wide_short_runs":
        # many bit positions differ, and entries that agree in the top 16 of them come in runs of two to eight: exact
        # ties, and neighbours a few units in the last place apart, out of order by point index
        depth = np.exp(rng.uniform(np.log(0.5), np.log(300.0), n)).astype(np.float32)
        for start in rng.integers(0, max(n - 8, 1), max(n // 6, 1)):
            run = int(rng.integers(2, 9))
            bits = depth[start:start + 1].view(np.uint32)[0] + rng.integers(0, 40, run).astype(np.uint32)
            where = rng.integers(0, n, run)
            depth[where] = bits.view(np.float32)
    else:
        depth = rng.choice(np.array([2.5, 2.5000002], dtype=np.float32), n)
    if kind != "wide_short_runs":
        depth[rng.integers(0, n, n // 3)] = depth[0]
    got, ref, _ = _lists_case(st, depth, 48, 48)
    assert ref["ranges"][4].tolist() == [0, n]             # tile (1, 1) of the 3 x 3 grid holds them all
    assert np.array_equal(got["vals"], ref["vals"])
    assert np.array_equal(got["keys"], ref["keys"])
    assert np.array_equal(got["ranges"], ref["ranges"])


def test_lists_empty_single_and_adversarial_bits():
    # nothing visible
    st = dict(mean2d=np.zeros((7, 2)), conic=np.zeros((7, 3)), opacity=np.zeros(7), color=np.zeros((7, 3)), radius=np.zeros(7, dtype=np.int32))
    got, ref, view = _lists_case(st, np.ones(7), 48, 32)
    assert got["P_raw"] == 0 and (got["ranges"] == 0).all()
    out = view.render_fwd([0.25, 0.5, 0.75])
    assert (out["image"] == np.array([0.25, 0.5, 0.75], dtype=np.float32)).all() and (out["final_T"] == 1).all()
    assert (out["last_idx"] == 0).all()
    # a single pair
    st = dict(mean2d=[[40.0, 20.0]], conic=[[0.1, 0, 0.1]], opacity=[0.5], color=[[1, 1, 1]], radius=[2])
    got, ref, _ = _lists_case(st, [1.0], 48, 32)
    assert got["P_raw"] == 1 and got["vals"].tolist() == [0] and got["ranges"][2 + 3 * 1].tolist() == [0, 1]
    # depth bit patterns that differ only in one byte each, plus denormal-small and huge values
    depths = np.array([1.0, np.nextafter(np.float32(1.0), np.float32(2)), 256.0, 65536.0, 1.6e7, 1e-30, 3.4e38, 0.5, 0.5], dtype=np.float32)
    n = len(depths)
    st = dict(mean2d=np.full((n, 2), 20.0), conic=np.tile([0.1, 0, 0.1], (n, 1)), opacity=np.full(n, 0.5), color=np.zeros((n, 3)),
              radius=np.full(n, 30, dtype=np.int32))
    got, ref, _ = _lists_case(st, depths, 48, 32)
    assert np.array_equal(got["keys"], ref["keys"]) and np.array_equal(got["vals"], ref["vals"])


def test_zero_points():
    cam = _cam(32, 32)
    view = GpuView(0, cam, 16)
    scene = B.Scene.from_numpy(dict(mean=np.zeros((0, 3)), log_scale=np.zeros((0, 3)), quat=np.zeros((0, 4)), logit=np.zeros(0),
                                    sh=np.zeros((0, 1, 3)), sh_degree=0))
    B.pbdr_preprocess(scene, cam, view.splats)
    out = view.render_fwd([1.0, 0.0, 0.5])
    assert (out["image"][..., 0] == 1).all() and (out["image"][..., 2] == 0.5).all()
    grads = scene.zeros_like()
    view.render_bwd([1.0, 0.0, 0.5], np.ones((32, 32, 3), dtype=np.float32), scene=scene, grads=grads)
    # the same without a splat-state gradient output, and the batched calls on an empty cloud
    G = torch.ones((3, 32, 32), device="cuda")
    B.pbdr_render_bwd(scene, view.splats, cam, [1.0, 0.0, 0.5], view.cap, view.final_T, view.last_idx, G, None, grads, view.ws,
                      first_view=True)
    torch.cuda.synchronize()


def _untouched(st, w, h):
    """Points with radius > 0 whose tile rectangle misses the image (binning does not list them)."""
    r = np.asarray(st["radius"], dtype=np.int64)
    ix = np.floor(np.asarray(st["mean2d"], dtype=np.float32)[:, 0]).astype(np.int64)
    iy = np.floor(np.asarray(st["mean2d"], dtype=np.float32)[:, 1]).astype(np.int64)
    tx, ty = (w + 15) // 16, (h + 15) // 16
    x0, x1 = np.clip((ix - r) >> 4, 0, tx), np.clip((ix + r + 15) >> 4, 0, tx)
    y0, y1 = np.clip((iy - r) >> 4, 0, ty), np.clip((iy + r + 15) >> 4, 0, ty)
    return int(((r > 0) & ((x1 - x0) * (y1 - y0) == 0)).sum())


def test_capacity_overflow_is_reported_and_in_bounds():
    rng = np.random.default_rng(5)
    n, w, h = 2000, 128, 96
    st = _rand_state(rng, n, w, h)
    depth = rng.uniform(0.3, 50, n).astype(np.float32)
    full, ref, roomy = _lists_case(st, depth, w, h)
    assert np.array_equal(full["vals"], ref["vals"])
    cap = ref["P"] // 3
    got, _, view = _lists_case(st, depth, w, h, cap=cap)
    n_dup, over = B.pbdr_query_lists(view.ws, n, w, h, cap)
    assert over and n_dup == ref["P"]
    assert got["P"] == cap
    # the same through the status words a caller can poll without a synchronising call: {pairs found, overflow, listed}
    words = B.pbdr_status_view(view.ws, n, w, h, cap).cpu().numpy()
    assert words.tolist() == [ref["P"], 1, int((np.asarray(st["radius"]) > 0).sum() - _untouched(st, w, h))]
    words_ok = B.pbdr_status_view(roomy.ws, n, w, h, roomy.cap).cpu().numpy()      # the run with room for every pair
    assert words_ok[0] == ref["P"] and words_ok[1] == 0
    # what was kept is a sorted subset of the true pairs, and ranges stay inside the capacity
    assert (np.diff(got["keys"].astype(np.uint64).astype(object)) >= 0).all()
    assert got["ranges"].max() <= cap
    true_pairs = set(zip(ref["keys"].tolist(), ref["vals"].tolist()))
    assert set(zip(got["keys"].tolist(), got["vals"].tolist())) <= true_pairs
    # rendering from truncated lists must still run and stay finite
    out = view.render_fwd([0, 0, 0])
    assert np.isfinite(out["image"]).all()


def test_large_radius_covers_whole_image():
    w, h = 200, 120
    st = dict(mean2d=[[100.0, 60.0], [10.0, 10.0]], conic=[[1e-4, 0, 1e-4], [0.05, 0, 0.05]], opacity=[0.6, 0.9],
              color=[[1, 0, 0], [0, 1, 0]], radius=[100000, 9])
    got, ref, view = _lists_case(st, [2.0, 1.0], w, h)
    assert np.array_equal(got["keys"], ref["keys"]) and np.array_equal(got["ranges"], ref["ranges"])
    out = view.render_fwd([0, 0, 0])
    sp64 = {k: np.asarray(st[k], dtype=np.float32).astype(np.float64) for k in ("mean2d", "conic", "opacity", "color")}
    r = oracle.render_fwd(sp64, ref, w, h, [0, 0, 0])
    assert np.abs(out["image"] - r["image"]).max() < 1e-5


def test_caller_supplied_conics_that_are_not_positive_definite():
    """pbdr_render_fwd / pbdr_render_bwd accept any splat state. A conic that is not positive definite makes the
    quadratic form negative on part of the image, where the rule is "skip" (no blend); the compositing kernels leave that
    test out only for batches whose conics are all safely positive definite, so a scene that mixes indefinite,
    near-degenerate and ordinary conics over several staging batches exercises both loops, forward and backward."""
    rng = np.random.default_rng(17)
    w, h, n = 96, 80, 900                                   # ~40 splats per tile on average, several batches of 256 in the busy ones
    st = dict(mean2d=np.stack([rng.uniform(0, w, n), rng.uniform(0, h, n)], 1).astype(np.float32),
              conic=np.zeros((n, 3), dtype=np.float32), opacity=rng.uniform(0.05, 0.6, n).astype(np.float32),
              color=rng.uniform(0, 1, (n, 3)).astype(np.float32), radius=rng.integers(4, 40, n).astype(np.int32))
    a = rng.uniform(0.01, 0.08, n); c = rng.uniform(0.01, 0.08, n)
    b = rng.uniform(-0.9, 0.9, n) * np.sqrt(a * c)          # positive definite ...
    kind = rng.integers(0, 4, n)
    b[kind == 1] = (1.5 * np.sqrt(a * c) * rng.choice([-1, 1], n))[kind == 1]                  # ... indefinite ...
    b[kind == 2] = (np.sqrt(a * c) * (1 - 1e-7) * rng.choice([-1, 1], n))[kind == 2]            # ... within rounding of degenerate
    st["conic"] = np.stack([a, b, c], 1).astype(np.float32)
    st["mean2d"][:300] = rng.uniform(30, 50, (300, 2)).astype(np.float32)                     # a crowd, so that lists exceed one batch
    depth = rng.uniform(0.5, 20, n).astype(np.float32)
    got_l, ref_l, view = _lists_case(st, depth, w, h)
    assert np.array_equal(got_l["vals"], ref_l["vals"])
    assert (ref_l["ranges"][:, 1] - ref_l["ranges"][:, 0]).max() > 256
    bg = [0.1, 0.2, 0.3]
    got = view.render_fwd(bg)
    st64 = {k: np.asarray(v, dtype=np.float32).astype(np.float64) for k, v in st.items() if k != "radius"} | {"radius": st["radius"]}
    ref = oracle.render_fwd(st64, ref_l, w, h, bg)
    ok = ref["fragile"] == 0
    assert ok.mean() > 0.95
    assert np.abs(got["image"] - ref["image"])[ok].max() <= 1e-4
    assert np.array_equal(got["last_idx"][ok], ref["last_idx"][ok])
    G = rng.normal(size=(h, w, 3)).astype(np.float32)
    G[~ok] = 0.0
    G[got["last_idx"] != ref["last_idx"]] = 0.0
    g = view.render_bwd(bg, G)
    rg = oracle.render_bwd(st64, ref_l, w, h, bg, G.astype(np.float64))
    for k in ("mean2d", "conic", "opacity", "color"):
        # a pixel that sits within rounding of sigma = 0 of an indefinite splat is flagged fragile and carries no loss;
        # what is left must agree
        grad_close("indefinite conics " + k, g[k], rg[k])
