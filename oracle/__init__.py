"""CPU oracle for the splatting hot path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

A ctypes view of oracle/pbdr_oracle.c (plain C, fp64). Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this package; it imports nothing from the HIP package.

All arrays are numpy, C-contiguous; floating point is float64 unless stated. Layouts follow the
paper's "S x l" tensors (Sec. 3.1) and Table 3a: mean[n,3], log_scale[n,3], quat[n,4] (w,x,y,z),
logit[n], sh[n,K,3]; splat state mean2d[n,2], conic[n,3], opacity[n], color[n,3], radius[n] (int32),
depth[n]. Images are [H,W,3].
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

TILE = 16

_lib = None


class Camera(C.Structure):
    _fields_ = [("width", C.c_int32), ("height", C.c_int32),
                ("fx", C.c_double), ("fy", C.c_double), ("cx", C.c_double), ("cy", C.c_double),
                ("R", C.c_double * 9), ("t", C.c_double * 3),
                ("near_plane", C.c_double), ("far_plane", C.c_double), ("radius_clip", C.c_double)]


def camera(cam: dict) -> Camera:
    """cam: dict with width,height,fx,fy,cx,cy,R(3x3 world->camera),t(3),near,far,radius_clip."""
    c = Camera()
    c.width, c.height = int(cam["width"]), int(cam["height"])
    c.fx, c.fy, c.cx, c.cy = (float(cam[k]) for k in ("fx", "fy", "cx", "cy"))
    R = np.asarray(cam["R"], dtype=np.float64).reshape(9)
    t = np.asarray(cam["t"], dtype=np.float64).reshape(3)
    for i in range(9):
        c.R[i] = R[i]
    for i in range(3):
        c.t[i] = t[i]
    c.near_plane = float(cam.get("near", 0.2))
    c.far_plane = float(cam.get("far", 1e10))
    c.radius_clip = float(cam.get("radius_clip", 0.0))
    return c


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.orc_count_pairs.restype = C.c_uint64
        _lib.orc_bin_sort.restype = C.c_uint64
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def _f64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def num_threads() -> int:
    return int(lib().orc_num_threads())


def sh_basis(deg: int, direction) -> np.ndarray:
    d = _f64(direction, (3,))
    Y = np.zeros(16, dtype=np.float64)
    lib().orc_sh_basis(C.c_int(deg), _p(d, C.c_double), _p(Y, C.c_double))
    return Y


def tile_rect(mx, my, radius, width, height):
    r = np.zeros(4, dtype=np.int32)
    lib().orc_tile_rect(C.c_double(mx), C.c_double(my), C.c_int(int(radius)), C.c_int(width), C.c_int(height),
                        _p(r, C.c_int32))
    return r


def preprocess(scene: dict, cam: dict, tau: float = 2e-5) -> dict:
    """Cull + project + colour for one view. Returns the Table 3a state plus rect, cov2d, near_tie."""
    n = int(scene["mean"].shape[0])
    deg = int(scene["sh_degree"])
    K = (deg + 1) ** 2
    mean = _f64(scene["mean"], (n, 3)); ls = _f64(scene["log_scale"], (n, 3)); q = _f64(scene["quat"], (n, 4))
    lo = _f64(scene["logit"], (n,)); sh = _f64(scene["sh"], (n, K, 3))
    out = dict(mean2d=np.zeros((n, 2)), conic=np.zeros((n, 3)), opacity=np.zeros(n), color=np.zeros((n, 3)),
               radius=np.zeros(n, dtype=np.int32), depth=np.zeros(n), rect=np.zeros((n, 4), dtype=np.int32),
               cov2d=np.zeros((n, 3)), near_tie=np.zeros(n, dtype=np.uint8))
    c = camera(cam)
    lib().orc_preprocess(C.c_int(n), C.c_int(deg), _p(mean, C.c_double), _p(ls, C.c_double), _p(q, C.c_double),
                         _p(lo, C.c_double), _p(sh, C.c_double), C.byref(c), _p(out["mean2d"], C.c_double),
                         _p(out["conic"], C.c_double), _p(out["opacity"], C.c_double), _p(out["color"], C.c_double),
                         _p(out["radius"], C.c_int32), _p(out["depth"], C.c_double), _p(out["rect"], C.c_int32),
                         _p(out["cov2d"], C.c_double), _p(out["near_tie"], C.c_uint8), C.c_double(tau))
    return out


def bin_sort(mean2d, radius, depth32, width, height) -> dict:
    """Tile lists from (mean2d, radius, fp32 depth): sorted keys/vals and per-tile [start,end)."""
    n = int(radius.shape[0])
    m2 = _f64(mean2d, (n, 2))
    rad = np.ascontiguousarray(radius, dtype=np.int32)
    d32 = np.ascontiguousarray(depth32, dtype=np.float32)
    P = int(lib().orc_count_pairs(C.c_int(n), _p(m2, C.c_double), _p(rad, C.c_int32), C.c_int(width), C.c_int(height)))
    tx, ty = (width + TILE - 1) // TILE, (height + TILE - 1) // TILE
    keys = np.zeros(max(P, 1), dtype=np.uint64); vals = np.zeros(max(P, 1), dtype=np.uint32)
    ranges = np.zeros((tx * ty, 2), dtype=np.uint32)
    P2 = int(lib().orc_bin_sort(C.c_int(n), _p(m2, C.c_double), _p(rad, C.c_int32), _p(d32, C.c_float), C.c_int(width),
                                C.c_int(height), _p(keys, C.c_uint64), _p(vals, C.c_uint32), _p(ranges, C.c_uint32)))
    assert P2 == P
    return dict(P=P, keys=keys[:P], vals=vals[:P], ranges=ranges)


def render_fwd(splats: dict, lists: dict, width, height, bg) -> dict:
    n = int(splats["opacity"].shape[0])
    m2 = _f64(splats["mean2d"], (n, 2)); co = _f64(splats["conic"], (n, 3)); op = _f64(splats["opacity"], (n,))
    col = _f64(splats["color"], (n, 3)); bgv = _f64(bg, (3,))
    vals = np.ascontiguousarray(lists["vals"], dtype=np.uint32)
    if vals.size == 0:
        vals = np.zeros(1, dtype=np.uint32)
    ranges = np.ascontiguousarray(lists["ranges"], dtype=np.uint32)
    out = dict(image=np.zeros((height, width, 3)), final_T=np.zeros((height, width)),
               last_idx=np.zeros((height, width), dtype=np.uint32), fragile=np.zeros((height, width), dtype=np.uint8))
    counters = np.zeros(2, dtype=np.uint64)
    lib().orc_render_fwd(C.c_int(width), C.c_int(height), _p(m2, C.c_double), _p(co, C.c_double), _p(op, C.c_double),
                         _p(col, C.c_double), _p(vals, C.c_uint32), _p(ranges, C.c_uint32), _p(bgv, C.c_double),
                         _p(out["image"], C.c_double), _p(out["final_T"], C.c_double), _p(out["last_idx"], C.c_uint32),
                         _p(out["fragile"], C.c_uint8), _p(counters, C.c_uint64))
    out["n_eval"] = int(counters[0]); out["n_blend"] = int(counters[1])
    return out


def render_fwd_global(splats: dict, order, rect, width, height, bg) -> dict:
    n = int(splats["opacity"].shape[0])
    m2 = _f64(splats["mean2d"], (n, 2)); co = _f64(splats["conic"], (n, 3)); op = _f64(splats["opacity"], (n,))
    col = _f64(splats["color"], (n, 3)); bgv = _f64(bg, (3,))
    order = np.ascontiguousarray(order, dtype=np.uint32)
    rect = np.ascontiguousarray(rect, dtype=np.int32)
    image = np.zeros((height, width, 3)); final_T = np.zeros((height, width))
    o = order if order.size else np.zeros(1, dtype=np.uint32)
    lib().orc_render_fwd_global(C.c_int(width), C.c_int(height), C.c_int(int(order.size)), _p(o, C.c_uint32),
                                _p(rect, C.c_int32), _p(m2, C.c_double), _p(co, C.c_double), _p(op, C.c_double),
                                _p(col, C.c_double), _p(bgv, C.c_double), _p(image, C.c_double), _p(final_T, C.c_double))
    return dict(image=image, final_T=final_T)


def render_bwd(splats: dict, lists: dict, width, height, bg, dL_dimage) -> dict:
    n = int(splats["opacity"].shape[0])
    m2 = _f64(splats["mean2d"], (n, 2)); co = _f64(splats["conic"], (n, 3)); op = _f64(splats["opacity"], (n,))
    col = _f64(splats["color"], (n, 3)); bgv = _f64(bg, (3,)); g = _f64(dL_dimage, (height, width, 3))
    vals = np.ascontiguousarray(lists["vals"], dtype=np.uint32)
    if vals.size == 0:
        vals = np.zeros(1, dtype=np.uint32)
    ranges = np.ascontiguousarray(lists["ranges"], dtype=np.uint32)
    out = dict(mean2d=np.zeros((n, 2)), conic=np.zeros((n, 3)), opacity=np.zeros(n), color=np.zeros((n, 3)))
    lib().orc_render_bwd(C.c_int(width), C.c_int(height), _p(m2, C.c_double), _p(co, C.c_double), _p(op, C.c_double),
                         _p(col, C.c_double), _p(vals, C.c_uint32), _p(ranges, C.c_uint32), _p(bgv, C.c_double),
                         _p(g, C.c_double), _p(out["mean2d"], C.c_double), _p(out["conic"], C.c_double),
                         _p(out["opacity"], C.c_double), _p(out["color"], C.c_double))
    return out


def preprocess_bwd(scene: dict, cam: dict, d_splats: dict, accumulate_into: dict = None) -> dict:
    n = int(scene["mean"].shape[0])
    deg = int(scene["sh_degree"])
    K = (deg + 1) ** 2
    mean = _f64(scene["mean"], (n, 3)); ls = _f64(scene["log_scale"], (n, 3)); q = _f64(scene["quat"], (n, 4))
    lo = _f64(scene["logit"], (n,)); sh = _f64(scene["sh"], (n, K, 3))
    dm = _f64(d_splats["mean2d"], (n, 2)); dc = _f64(d_splats["conic"], (n, 3)); do = _f64(d_splats["opacity"], (n,))
    dcol = _f64(d_splats["color"], (n, 3))
    g = accumulate_into or dict(mean=np.zeros((n, 3)), log_scale=np.zeros((n, 3)), quat=np.zeros((n, 4)),
                                logit=np.zeros(n), sh=np.zeros((n, K, 3)))
    c = camera(cam)
    lib().orc_preprocess_bwd(C.c_int(n), C.c_int(deg), _p(mean, C.c_double), _p(ls, C.c_double), _p(q, C.c_double),
                             _p(lo, C.c_double), _p(sh, C.c_double), C.byref(c), _p(dm, C.c_double), _p(dc, C.c_double),
                             _p(do, C.c_double), _p(dcol, C.c_double), _p(g["mean"], C.c_double),
                             _p(g["log_scale"], C.c_double), _p(g["quat"], C.c_double), _p(g["logit"], C.c_double),
                             _p(g["sh"], C.c_double))
    return g


# --------------------------------------------------------------------------------------------
# Whole path, in the order of Alg. 1's compute lines: splat -> sort -> render -> (loss grad) ->
# render.backward -> splatting.backward. `splat_dtype` = np.float32 rounds the Table 3a state to
# fp32 before binning and blending (the state as it is stored / exchanged); np.float64 keeps it.
# --------------------------------------------------------------------------------------------
def forward(scene: dict, cam: dict, bg, splat_dtype=np.float32) -> dict:
    sp = preprocess(scene, cam)
    W, H = int(cam["width"]), int(cam["height"])
    st = {k: sp[k].astype(splat_dtype).astype(np.float64) for k in ("mean2d", "conic", "opacity", "color")}
    st["radius"] = sp["radius"]
    depth32 = sp["depth"].astype(np.float32)
    lists = bin_sort(st["mean2d"], st["radius"], depth32, W, H)
    out = render_fwd(st, lists, W, H, bg)
    out.update(splats=sp, state=st, lists=lists, depth32=depth32)
    return out


def backward(scene: dict, cam: dict, bg, fwd: dict, dL_dimage) -> dict:
    W, H = int(cam["width"]), int(cam["height"])
    d_sp = render_bwd(fwd["state"], fwd["lists"], W, H, bg, dL_dimage)
    g = preprocess_bwd(scene, cam, d_sp)
    g["d_splats"] = d_sp
    return g


# --------------------------------------------------------------------------------------------
# 2D Gaussian surfels. Scene: mean[n,3], tan_u[n,3], tan_v[n,3], log_scale[n,2], logit[n], sh[n,K,3].
# Splat state (Table 3b): mean2d[n,2], T[n,9] (ray_transforms), opacity[n], color[n,3], radius[n], depth[n], normal[n,3].
# --------------------------------------------------------------------------------------------
def ray_uv(T, x, y):
    Tm = _f64(T, (9,)); uv = np.zeros(2)
    ok = lib().orc2d_ray_uv(_p(Tm, C.c_double), C.c_double(x), C.c_double(y), _p(uv, C.c_double))
    return uv if ok else None


def _scene2d_arrays(scene):
    n = int(scene["mean"].shape[0]); deg = int(scene["sh_degree"]); K = (deg + 1) ** 2
    return (n, deg, K, _f64(scene["mean"], (n, 3)), _f64(scene["tan_u"], (n, 3)), _f64(scene["tan_v"], (n, 3)),
            _f64(scene["log_scale"], (n, 2)), _f64(scene["logit"], (n,)), _f64(scene["sh"], (n, K, 3)))


def preprocess2d(scene: dict, cam: dict, tau: float = 2e-5) -> dict:
    n, deg, K, mean, tu, tv, ls, lo, sh = _scene2d_arrays(scene)
    out = dict(mean2d=np.zeros((n, 2)), T=np.zeros((n, 9)), opacity=np.zeros(n), color=np.zeros((n, 3)),
               radius=np.zeros(n, dtype=np.int32), depth=np.zeros(n), normal=np.zeros((n, 3)), bbox=np.zeros((n, 4)),
               near_tie=np.zeros(n, dtype=np.uint8))
    c = camera(cam)
    lib().orc2d_preprocess(C.c_int(n), C.c_int(deg), _p(mean, C.c_double), _p(tu, C.c_double), _p(tv, C.c_double),
                           _p(ls, C.c_double), _p(lo, C.c_double), _p(sh, C.c_double), C.byref(c),
                           _p(out["mean2d"], C.c_double), _p(out["T"], C.c_double), _p(out["opacity"], C.c_double),
                           _p(out["color"], C.c_double), _p(out["radius"], C.c_int32), _p(out["depth"], C.c_double),
                           _p(out["normal"], C.c_double), _p(out["bbox"], C.c_double), _p(out["near_tie"], C.c_uint8),
                           C.c_double(tau))
    return out


def render_fwd2d(splats: dict, lists: dict, width, height, bg) -> dict:
    n = int(splats["opacity"].shape[0])
    m2 = _f64(splats["mean2d"], (n, 2)); T = _f64(splats["T"], (n, 9)); op = _f64(splats["opacity"], (n,))
    col = _f64(splats["color"], (n, 3)); bgv = _f64(bg, (3,))
    vals = np.ascontiguousarray(lists["vals"], dtype=np.uint32)
    if vals.size == 0:
        vals = np.zeros(1, dtype=np.uint32)
    ranges = np.ascontiguousarray(lists["ranges"], dtype=np.uint32)
    out = dict(image=np.zeros((height, width, 3)), final_T=np.zeros((height, width)),
               last_idx=np.zeros((height, width), dtype=np.uint32), fragile=np.zeros((height, width), dtype=np.uint8))
    counters = np.zeros(2, dtype=np.uint64)
    lib().orc2d_render_fwd(C.c_int(width), C.c_int(height), _p(m2, C.c_double), _p(T, C.c_double), _p(op, C.c_double),
                           _p(col, C.c_double), _p(vals, C.c_uint32), _p(ranges, C.c_uint32), _p(bgv, C.c_double),
                           _p(out["image"], C.c_double), _p(out["final_T"], C.c_double), _p(out["last_idx"], C.c_uint32),
                           _p(out["fragile"], C.c_uint8), _p(counters, C.c_uint64))
    out["n_eval"] = int(counters[0]); out["n_blend"] = int(counters[1])
    return out


def render_bwd2d(splats: dict, lists: dict, width, height, bg, dL_dimage) -> dict:
    n = int(splats["opacity"].shape[0])
    m2 = _f64(splats["mean2d"], (n, 2)); T = _f64(splats["T"], (n, 9)); op = _f64(splats["opacity"], (n,))
    col = _f64(splats["color"], (n, 3)); bgv = _f64(bg, (3,)); g = _f64(dL_dimage, (height, width, 3))
    vals = np.ascontiguousarray(lists["vals"], dtype=np.uint32)
    if vals.size == 0:
        vals = np.zeros(1, dtype=np.uint32)
    ranges = np.ascontiguousarray(lists["ranges"], dtype=np.uint32)
    out = dict(T=np.zeros((n, 9)), mean2d=np.zeros((n, 2)), opacity=np.zeros(n), color=np.zeros((n, 3)))
    lib().orc2d_render_bwd(C.c_int(width), C.c_int(height), _p(m2, C.c_double), _p(T, C.c_double), _p(op, C.c_double),
                           _p(col, C.c_double), _p(vals, C.c_uint32), _p(ranges, C.c_uint32), _p(bgv, C.c_double),
                           _p(g, C.c_double), _p(out["T"], C.c_double), _p(out["mean2d"], C.c_double),
                           _p(out["opacity"], C.c_double), _p(out["color"], C.c_double))
    return out


def preprocess_bwd2d(scene: dict, cam: dict, d_splats: dict, accumulate_into: dict = None) -> dict:
    n, deg, K, mean, tu, tv, ls, lo, sh = _scene2d_arrays(scene)
    dT = _f64(d_splats["T"], (n, 9)); dm = _f64(d_splats["mean2d"], (n, 2)); do = _f64(d_splats["opacity"], (n,))
    dc = _f64(d_splats["color"], (n, 3))
    g = accumulate_into or dict(mean=np.zeros((n, 3)), tan_u=np.zeros((n, 3)), tan_v=np.zeros((n, 3)),
                                log_scale=np.zeros((n, 2)), logit=np.zeros(n), sh=np.zeros((n, K, 3)))
    c = camera(cam)
    lib().orc2d_preprocess_bwd(C.c_int(n), C.c_int(deg), _p(mean, C.c_double), _p(tu, C.c_double), _p(tv, C.c_double),
                               _p(ls, C.c_double), _p(lo, C.c_double), _p(sh, C.c_double), C.byref(c), _p(dT, C.c_double),
                               _p(dm, C.c_double), _p(do, C.c_double), _p(dc, C.c_double), _p(g["mean"], C.c_double),
                               _p(g["tan_u"], C.c_double), _p(g["tan_v"], C.c_double), _p(g["log_scale"], C.c_double),
                               _p(g["logit"], C.c_double), _p(g["sh"], C.c_double))
    return g


def forward2d(scene: dict, cam: dict, bg, splat_dtype=np.float32) -> dict:
    sp = preprocess2d(scene, cam)
    W, H = int(cam["width"]), int(cam["height"])
    st = {k: sp[k].astype(splat_dtype).astype(np.float64) for k in ("mean2d", "T", "opacity", "color")}
    st["radius"] = sp["radius"]
    depth32 = sp["depth"].astype(np.float32)
    lists = bin_sort(st["mean2d"], st["radius"], depth32, W, H)
    out = render_fwd2d(st, lists, W, H, bg)
    out.update(splats=sp, state=st, lists=lists, depth32=depth32)
    return out


def backward2d(scene: dict, cam: dict, bg, fwd: dict, dL_dimage) -> dict:
    W, H = int(cam["width"]), int(cam["height"])
    d_sp = render_bwd2d(fwd["state"], fwd["lists"], W, H, bg, dL_dimage)
    g = preprocess_bwd2d(scene, cam, d_sp)
    g["d_splats"] = d_sp
    return g


# ---------------------------------------------------------------------------------------- point-group frustum culling
def _scene_arrays(scene):
    n = int(scene["mean"].shape[0]); deg = int(scene["sh_degree"]); K = (deg + 1) ** 2
    return (n, deg, K, _f64(scene["mean"], (n, 3)), _f64(scene["log_scale"], (n, 3)), _f64(scene["quat"], (n, 4)),
            _f64(scene["logit"], (n,)), _f64(scene["sh"], (n, K, 3)))


def group_bounds(scene: dict, group_size: int) -> np.ndarray:
    """[ceil(n/G), 7] = (min xyz, max xyz, largest scale) per group of G consecutive points."""
    n, deg, K, mean, ls, q, lo, sh = _scene_arrays(scene)
    ng = (n + group_size - 1) // group_size
    out = np.zeros((max(ng, 1), 7))
    lib().orc_group_bounds(C.c_int(n), C.c_int(group_size), _p(mean, C.c_double), _p(ls, C.c_double), _p(out, C.c_double))
    return out[:ng]


def group_cull(bounds: np.ndarray, cam: dict, tau: float = 1e-4) -> dict:
    b = np.ascontiguousarray(bounds, dtype=np.float64)
    ng = int(b.shape[0])
    out = dict(keep=np.zeros(max(ng, 1), dtype=np.uint8), near_tie=np.zeros(max(ng, 1), dtype=np.uint8))
    c = camera(cam)
    lib().orc_group_cull(C.c_int(ng), _p(b, C.c_double), C.byref(c), _p(out["keep"], C.c_uint8),
                         _p(out["near_tie"], C.c_uint8), C.c_double(tau))
    return {k: v[:ng] for k, v in out.items()}


def preprocess_grouped(scene: dict, cam: dict, group_size: int) -> dict:
    n, deg, K, mean, ls, q, lo, sh = _scene_arrays(scene)
    ng = (n + group_size - 1) // group_size
    out = dict(mean2d=np.zeros((n, 2)), conic=np.zeros((n, 3)), opacity=np.zeros(n), color=np.zeros((n, 3)),
               radius=np.zeros(n, dtype=np.int32), depth=np.zeros(n), keep=np.zeros(max(ng, 1), dtype=np.uint8))
    c = camera(cam)
    lib().orc_preprocess_grouped(C.c_int(n), C.c_int(deg), C.c_int(group_size), _p(mean, C.c_double), _p(ls, C.c_double),
                                 _p(q, C.c_double), _p(lo, C.c_double), _p(sh, C.c_double), C.byref(c),
                                 _p(out["mean2d"], C.c_double), _p(out["conic"], C.c_double), _p(out["opacity"], C.c_double),
                                 _p(out["color"], C.c_double), _p(out["radius"], C.c_int32), _p(out["depth"], C.c_double),
                                 _p(out["keep"], C.c_uint8))
    out["keep"] = out["keep"][:ng]
    return out


# ---------------------------------------------------------------------------------------- loss and optimizer step
# Alg. 1's loss_fn, loss_fn.backward and AdamUpdate steps. The paper names the steps only; the
# benchmark configurations fix the loss (mean L1 against the target image) and App. E.1 says the optimizer is the
# "selective" Adam: the textbook update (Kingma & Ba, with bias correction) applied to the points that were visible
# in the batch, every other point - parameter and both moments - left exactly as it was. Plain numpy, fp64.
def l1_loss(image, target):
    """image, target [H,W,3]. Returns (mean |image - target|, dL/dimage = sign(image - target) / (3 H W))."""
    a = np.asarray(image, dtype=np.float64); b = np.asarray(target, dtype=np.float64)
    d = a - b
    return float(np.abs(d).mean()), np.sign(d) / d.size


def adam_selective(param, grad, exp_avg, exp_avg_sq, visible, lr, beta1, beta2, eps, step):
    """One Adam step on the rows i with visible[i] != 0 of param [n, ...]; returns new (param, exp_avg, exp_avg_sq).
    step = 1 for the first update (bias corrections 1 - beta^step)."""
    p = np.array(param, dtype=np.float64); g = np.asarray(grad, dtype=np.float64)
    m = np.array(exp_avg, dtype=np.float64); v = np.array(exp_avg_sq, dtype=np.float64)
    rows = np.nonzero(np.asarray(visible) != 0)[0]
    for i in rows:
        m[i] = beta1 * m[i] + (1.0 - beta1) * g[i]
        v[i] = beta2 * v[i] + (1.0 - beta2) * g[i] * g[i]
        m_hat = m[i] / (1.0 - beta1 ** step)
        v_hat = v[i] / (1.0 - beta2 ** step)
        p[i] = p[i] - lr * m_hat / (np.sqrt(v_hat) + eps)
    return p, m, v
