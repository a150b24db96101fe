"""Thin ctypes binding over libpbdr.so (the C ABI in include/pbdr.h).

Argument marshalling only: every step of the path runs in the HIP kernels. PyTorch supplies device memory and the
current stream. There is no fallback: if the library is missing, loading raises.

Tensor layouts are the library's structure-of-arrays planes: an attribute with l components is a contiguous
[l, n] float32 tensor (the paper's S x l tensor, transposed); images are [3, H, W].
"""
import ctypes as C
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpbdr.so")

PBDR_OK = 0
PBDR_ERR_INVALID_ARG = -1
PBDR_ERR_WORKSPACE_TOO_SMALL = -2
PBDR_ERR_CAPACITY = -3
PBDR_ERR_HIP = -4
PBDR_ERR_STATIC_LIMIT = -5
PBDR_STATIC_MAX_POINTS = 16384
PBDR_STATIC_MAX_SIDE = 512
PBDR_STATIC_MAX_PAIRS = 262144
PBDR_STATIC_SCRATCH_BYTES = 24 << 20

EXPORTS = ("pbdr_workspace_bytes", "pbdr_preprocess", "pbdr_bin_sort", "pbdr_render_fwd", "pbdr_render_bwd",
           "pbdr_preprocess_bwd", "pbdr_lists_view", "pbdr_query_lists", "pbdr_status_string", "pbdr_last_hip_error",
           "pbdr_version", "pbdr_render_stats", "pbdr_profile_begin", "pbdr_profile_collect", "pbdr_profile_reset",
           "pbdr_profile_end", "pbdr_profile_kernel_name", "pbdr_profile_kernel_count",
           "pbdr2d_workspace_bytes", "pbdr2d_preprocess", "pbdr2d_render_fwd", "pbdr2d_render_bwd", "pbdr2d_preprocess_bwd",
           "pbdr2d_lists_view", "pbdr2d_render_stats", "pbdr_group_count", "pbdr_group_bounds", "pbdr_preprocess_grouped",
           "pbdr_preprocess_patch", "pbdr_render_fwd_patch", "pbdr_render_bwd_patch",
           "pbdr2d_preprocess_patch", "pbdr2d_render_fwd_patch", "pbdr2d_render_bwd_patch",
           "pbdr_l1_loss", "pbdr_mark_visible", "pbdr_adam_selective", "pbdr_preprocess_batch", "pbdr_preprocess_bwd_batch",
           "pbdr_preprocess_bwd_batch_adam", "pbdr_tile_order_view", "pbdr_render_fwd_static", "pbdr_workspace_init",
           "pbdr_status_view")

_f = C.POINTER(C.c_float)


class CScene(C.Structure):
    # also used for pbdr_scene_grads, which has the same layout plus the trailing first_view flag
    _fields_ = [("n", C.c_int32), ("sh_degree", C.c_int32), ("mean", C.c_void_p), ("log_scale", C.c_void_p),
                ("quat", C.c_void_p), ("opacity_logit", C.c_void_p), ("sh", C.c_void_p), ("first_view", C.c_int32)]


class CCamera(C.Structure):
    _fields_ = [("width", C.c_int32), ("height", C.c_int32), ("fx", C.c_float), ("fy", C.c_float), ("cx", C.c_float),
                ("cy", C.c_float), ("R", C.c_float * 9), ("t", C.c_float * 3), ("near_plane", C.c_float),
                ("far_plane", C.c_float), ("radius_clip", C.c_float)]


class CPatch(C.Structure):
    _fields_ = [("x0", C.c_int32), ("y0", C.c_int32), ("x1", C.c_int32), ("y1", C.c_int32)]


class CAdamConfig(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("step", C.c_int32),
                ("zero_grad", C.c_int32)]


class CSplats(C.Structure):
    _fields_ = [("n", C.c_int32), ("mean2d", C.c_void_p), ("conic", C.c_void_p), ("opacity", C.c_void_p),
                ("color", C.c_void_p), ("radius", C.c_void_p), ("depth", C.c_void_p)]


class CSplatGrads(C.Structure):
    _fields_ = [("n", C.c_int32), ("mean2d", C.c_void_p), ("conic", C.c_void_p), ("opacity", C.c_void_p),
                ("color", C.c_void_p)]


class CScene2D(C.Structure):
    _fields_ = [("n", C.c_int32), ("sh_degree", C.c_int32), ("mean", C.c_void_p), ("tan_u", C.c_void_p),
                ("tan_v", C.c_void_p), ("log_scale", C.c_void_p), ("opacity_logit", C.c_void_p), ("sh", C.c_void_p),
                ("first_view", C.c_int32)]


class CSplats2D(C.Structure):
    _fields_ = [("n", C.c_int32), ("mean2d", C.c_void_p), ("ray_transform", C.c_void_p), ("opacity", C.c_void_p),
                ("color", C.c_void_p), ("radius", C.c_void_p), ("depth", C.c_void_p), ("normal", C.c_void_p)]


class CSplatGrads2D(C.Structure):
    _fields_ = [("n", C.c_int32), ("mean2d", C.c_void_p), ("ray_transform", C.c_void_p), ("opacity", C.c_void_p),
                ("color", C.c_void_p)]


_lib = None


def lib():
    """Load libpbdr.so; raises if it has not been built (python -m paper_2512_20017_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with `python paper_2512_20017_amd/build.py`")
        L = C.CDLL(LIB_PATH)
        L.pbdr_status_string.restype = C.c_char_p
        L.pbdr_profile_kernel_name.restype = C.c_char_p
        for name in EXPORTS:
            getattr(L, name)
        _lib = L
    return _lib


class PbdrError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__(f"pbdr: {lib().pbdr_status_string(C.c_int(status)).decode()} ({status})")


def _check(status):
    if status != PBDR_OK:
        raise PbdrError(status)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def camera_struct(cam: dict) -> CCamera:
    c = CCamera()
    c.width, c.height = int(cam["width"]), int(cam["height"])
    c.fx, c.fy, c.cx, c.cy = (float(cam[k]) for k in ("fx", "fy", "cx", "cy"))
    R = np.asarray(cam["R"], dtype=np.float32).reshape(9)
    t = np.asarray(cam["t"], dtype=np.float32).reshape(3)
    for i in range(9):
        c.R[i] = float(R[i])
    for i in range(3):
        c.t[i] = float(t[i])
    c.near_plane = float(cam.get("near", 0.2))
    c.far_plane = float(cam.get("far", 1e10))
    c.radius_clip = float(cam.get("radius_clip", 0.0))
    return c


def _dev(t):
    return C.c_void_p(t.data_ptr()) if t is not None and t.numel() > 0 else C.c_void_p(0)


@dataclass
class Scene:
    """Point parameters on the device, SoA planes: mean[3,n], log_scale[3,n], quat[4,n], logit[n], sh[K,3,n]."""
    n: int
    sh_degree: int
    mean: torch.Tensor
    log_scale: torch.Tensor
    quat: torch.Tensor
    logit: torch.Tensor
    sh: torch.Tensor

    @staticmethod
    def from_numpy(sc: dict, device="cuda") -> "Scene":
        """From the S x l host layout (mean[n,3], ..., sh[n,K,3]) to device planes."""
        def up(a, perm):
            return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.float32).transpose(perm))).to(device)
        n = int(sc["mean"].shape[0])
        return Scene(n, int(sc["sh_degree"]), up(sc["mean"], (1, 0)), up(sc["log_scale"], (1, 0)), up(sc["quat"], (1, 0)),
                     torch.from_numpy(np.ascontiguousarray(sc["logit"], dtype=np.float32)).to(device),
                     up(sc["sh"], (1, 2, 0)))

    def zeros_like(self) -> "Scene":
        """Same shapes, zero-filled, carved out of ONE allocation (kept as `.flat`) so that a gradient buffer is cleared
        with a single fill; every attribute starts on a 16-byte boundary."""
        parts = [self.mean, self.log_scale, self.quat, self.logit, self.sh]
        sizes = [(t.numel() + 3) // 4 * 4 for t in parts]
        flat = torch.zeros(sum(sizes), dtype=torch.float32, device=self.mean.device)
        views, at = [], 0
        for t, sz in zip(parts, sizes):
            views.append(flat[at:at + t.numel()].view(t.shape))
            at += sz
        out = Scene(self.n, self.sh_degree, *views)
        out.flat = flat
        return out

    def to_numpy(self) -> dict:
        return dict(mean=self.mean.cpu().numpy().T.copy(), log_scale=self.log_scale.cpu().numpy().T.copy(),
                    quat=self.quat.cpu().numpy().T.copy(), logit=self.logit.cpu().numpy().copy(),
                    sh=self.sh.cpu().numpy().transpose(2, 0, 1).copy(), sh_degree=self.sh_degree)

    def struct(self, first_view=False) -> CScene:
        return CScene(self.n, self.sh_degree, _dev(self.mean), _dev(self.log_scale), _dev(self.quat), _dev(self.logit),
                      _dev(self.sh), int(bool(first_view)))


@dataclass
class Splats:
    """Per-view splat state (Table 3a), SoA planes."""
    n: int
    mean2d: torch.Tensor
    conic: torch.Tensor
    opacity: torch.Tensor
    color: torch.Tensor
    radius: torch.Tensor
    depth: torch.Tensor

    @staticmethod
    def empty(n, device="cuda") -> "Splats":
        f = dict(dtype=torch.float32, device=device)
        return Splats(n, torch.empty((2, n), **f), torch.empty((3, n), **f), torch.empty(n, **f), torch.empty((3, n), **f),
                      torch.empty(n, dtype=torch.int32, device=device), torch.empty(n, **f))

    @staticmethod
    def from_numpy(st: dict, device="cuda") -> "Splats":
        """From host arrays mean2d[n,2], conic[n,3], opacity[n], color[n,3], radius[n], depth[n]."""
        def up(a, dt=np.float32):
            a = np.asarray(a, dtype=dt)
            return torch.from_numpy(np.ascontiguousarray(a.T if a.ndim == 2 else a)).to(device)
        n = int(np.asarray(st["opacity"]).shape[0])
        return Splats(n, up(st["mean2d"]), up(st["conic"]), up(st["opacity"]), up(st["color"]),
                      up(st["radius"], np.int32), up(st["depth"]))

    def to_numpy(self) -> dict:
        return dict(mean2d=self.mean2d.cpu().numpy().T.copy(), conic=self.conic.cpu().numpy().T.copy(),
                    opacity=self.opacity.cpu().numpy().copy(), color=self.color.cpu().numpy().T.copy(),
                    radius=self.radius.cpu().numpy().copy(), depth=self.depth.cpu().numpy().copy())

    def struct(self) -> CSplats:
        return CSplats(self.n, _dev(self.mean2d), _dev(self.conic), _dev(self.opacity), _dev(self.color),
                       _dev(self.radius), _dev(self.depth))


@dataclass
class SplatGrads:
    n: int
    mean2d: torch.Tensor
    conic: torch.Tensor
    opacity: torch.Tensor
    color: torch.Tensor

    @staticmethod
    def empty(n, device="cuda") -> "SplatGrads":
        f = dict(dtype=torch.float32, device=device)
        return SplatGrads(n, torch.empty((2, n), **f), torch.empty((3, n), **f), torch.empty(n, **f), torch.empty((3, n), **f))

    @staticmethod
    def from_numpy(d: dict, device="cuda") -> "SplatGrads":
        def up(a):
            a = np.asarray(a, dtype=np.float32)
            return torch.from_numpy(np.ascontiguousarray(a.T if a.ndim == 2 else a)).to(device)
        n = int(np.asarray(d["opacity"]).shape[0])
        return SplatGrads(n, up(d["mean2d"]), up(d["conic"]), up(d["opacity"]), up(d["color"]))

    def to_numpy(self) -> dict:
        return dict(mean2d=self.mean2d.cpu().numpy().T.copy(), conic=self.conic.cpu().numpy().T.copy(),
                    opacity=self.opacity.cpu().numpy().copy(), color=self.color.cpu().numpy().T.copy())

    def struct(self) -> CSplatGrads:
        return CSplatGrads(self.n, _dev(self.mean2d), _dev(self.conic), _dev(self.opacity), _dev(self.color))


def pbdr_version() -> int:
    return int(lib().pbdr_version())


def pbdr_workspace_bytes(n, width, height, dup_capacity) -> int:
    out = C.c_size_t(0)
    _check(lib().pbdr_workspace_bytes(C.c_int32(n), C.c_int32(width), C.c_int32(height), C.c_uint64(dup_capacity),
                                      C.byref(out)))
    return int(out.value)


def _alloc_ws(nbytes, device):
    """256-byte aligned and zero-filled once (pbdr_workspace_init), as the library asks of a workspace."""
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + nbytes]
    _check(lib().pbdr_workspace_init(C.c_void_p(ws.data_ptr()), C.c_size_t(nbytes), _stream(None)))
    return ws


def alloc_workspace(n, width, height, dup_capacity, device="cuda") -> torch.Tensor:
    return _alloc_ws(pbdr_workspace_bytes(n, width, height, dup_capacity), device)


def pbdr_status_view(ws, n, width, height, dup_capacity) -> torch.Tensor:
    """The three status words {pairs found, overflow flag, listed points} as a device tensor (a view into ws)."""
    p = C.POINTER(C.c_uint32)()
    _check(lib().pbdr_status_view(C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), C.c_int32(n), C.c_int32(width),
                                  C.c_int32(height), C.c_uint64(dup_capacity), C.byref(p)))
    off = C.cast(p, C.c_void_p).value - ws.data_ptr()
    return ws[off:off + 12].view(torch.int32)


def pbdr_preprocess(scene: Scene, cam: dict, out: Splats, stream=None) -> None:
    s, c, o = scene.struct(), camera_struct(cam), out.struct()
    _check(lib().pbdr_preprocess(C.byref(s), C.byref(c), C.byref(o), _stream(stream)))


def pbdr_group_count(n: int, group_size: int) -> int:
    ng = int(lib().pbdr_group_count(C.c_int32(n), C.c_int32(group_size)))
    if ng < 0:
        raise PbdrError(ng)
    return ng


def pbdr_group_bounds(scene: Scene, group_size: int, bounds: torch.Tensor, stream=None) -> None:
    """bounds: float32 [7, n_groups] on the device."""
    s = scene.struct()
    _check(lib().pbdr_group_bounds(C.byref(s), C.c_int32(group_size), _dev(bounds), _stream(stream)))


def pbdr_preprocess_grouped(scene: Scene, cam: dict, group_size: int, bounds: torch.Tensor, keep: torch.Tensor,
                            out: Splats, stream=None) -> None:
    """keep: uint8 [n_groups] on the device, written."""
    s, c, o = scene.struct(), camera_struct(cam), out.struct()
    _check(lib().pbdr_preprocess_grouped(C.byref(s), C.byref(c), C.c_int32(group_size), _dev(bounds), _dev(keep),
                                         C.byref(o), _stream(stream)))


def pbdr_preprocess_batch(scene: Scene, cams, outs, group_size: int = 0, bounds=None, keep=None, stream=None) -> None:
    """cams: list of camera dicts; outs: list of Splats, one per view. With group_size != 0: bounds float32 [7, n_groups]
    and keep uint8 [len(cams), n_groups] on the device (keep is written)."""
    s = scene.struct()
    cs = (CCamera * len(cams))(*[camera_struct(c) for c in cams])
    structs = [o.struct() for o in outs]
    os_ = (type(structs[0]) * len(outs))(*structs)
    _check(lib().pbdr_preprocess_batch(C.byref(s), C.c_int32(len(cams)), cs, os_, C.c_int32(group_size),
                                       _dev(bounds) if bounds is not None else None,
                                       _dev(keep) if keep is not None else None, _stream(stream)))


def pbdr_preprocess_bwd_batch(scene: Scene, cams, splats, g_splats, grads: Scene, stream=None, first_view=False) -> None:
    """cams / splats / g_splats: lists with one entry per view."""
    sc, g = scene.struct(), grads.struct(first_view)
    cs = (CCamera * len(cams))(*[camera_struct(c) for c in cams])
    sps = [x.struct() for x in splats]
    g2s = [x.struct() for x in g_splats]
    sp_arr = (type(sps[0]) * len(sps))(*sps)
    g2_arr = (type(g2s[0]) * len(g2s))(*g2s)
    _check(lib().pbdr_preprocess_bwd_batch(C.byref(sc), C.c_int32(len(cams)), cs, sp_arr, g2_arr, C.byref(g), _stream(stream)))


def pbdr_preprocess_bwd_batch_adam(scene: Scene, cams, splats, g_splats, exp_avg: Scene, exp_avg_sq: Scene, lrs, beta1, beta2, eps,
                                   step: int, stream=None) -> None:
    """lrs: learning rates of (mean, log_scale, quat, logit, sh). Updates the scene's tensors and both moments in place."""
    sc, m, v = scene.struct(), exp_avg.struct(), exp_avg_sq.struct()
    cs = (CCamera * len(cams))(*[camera_struct(c) for c in cams])
    sps = [x.struct() for x in splats]
    g2s = [x.struct() for x in g_splats]
    sp_arr = (type(sps[0]) * len(sps))(*sps)
    g2_arr = (type(g2s[0]) * len(g2s))(*g2s)
    lr = (C.c_float * 5)(*[float(x) for x in lrs])
    cfg = CAdamConfig(0.0, float(beta1), float(beta2), float(eps), int(step), 0)
    _check(lib().pbdr_preprocess_bwd_batch_adam(C.byref(sc), C.c_int32(len(cams)), cs, sp_arr, g2_arr, C.byref(m), C.byref(v), lr,
                                                C.byref(cfg), _stream(stream)))


def pbdr_bin_sort(splats: Splats, cam: dict, dup_capacity: int, ws: torch.Tensor, stream=None) -> None:
    s, c = splats.struct(), camera_struct(cam)
    _check(lib().pbdr_bin_sort(C.byref(s), C.byref(c), C.c_uint64(dup_capacity), C.c_void_p(ws.data_ptr()),
                               C.c_size_t(ws.numel()), _stream(stream)))


def pbdr_render_fwd(splats: Splats, cam: dict, bg, dup_capacity: int, image, final_T, last_idx, ws, stream=None) -> None:
    s, c = splats.struct(), camera_struct(cam)
    bgv = (C.c_float * 3)(*[float(x) for x in bg])
    _check(lib().pbdr_render_fwd(C.byref(s), C.byref(c), bgv, C.c_uint64(dup_capacity), _dev(image), _dev(final_T),
                                 _dev(last_idx), C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), _stream(stream)))


def pbdr_render_fwd_static(splats: Splats, cam: dict, bg, image, final_T, last_idx, pair_count=None, stream=None) -> None:
    """pbdr_render_fwd on the library's own fixed scratch array (no workspace argument); pair_count: uint32 tensor [1] or None."""
    s, c = splats.struct(), camera_struct(cam)
    bgv = (C.c_float * 3)(*[float(x) for x in bg])
    _check(lib().pbdr_render_fwd_static(C.byref(s), C.byref(c), bgv, _dev(image), _dev(final_T), _dev(last_idx),
                                        _dev(pair_count), _stream(stream)))


def pbdr_render_bwd(scene, splats: Splats, cam: dict, bg, dup_capacity: int, final_T, last_idx, dL_dimage,
                    g_splats: SplatGrads, grads, ws, stream=None, first_view=False) -> None:
    """scene/grads: both Scene (gradient accumulated into grads) or both None (stop at g_splats). first_view: write
    instead of accumulating, zeros for points the view does not use (the first view of a batch, buffer not cleared)."""
    sp, c = splats.struct(), camera_struct(cam)
    g2 = g_splats.struct() if g_splats is not None else None      # None (with scene/grads given): no splat-state gradient output
    bgv = (C.c_float * 3)(*[float(x) for x in bg])
    if scene is not None:
        sc, g = scene.struct(), grads.struct(first_view)
        psc, pg = C.byref(sc), C.byref(g)
    else:
        psc, pg = None, None
    _check(lib().pbdr_render_bwd(psc, C.byref(sp), C.byref(c), bgv, C.c_uint64(dup_capacity), _dev(final_T), _dev(last_idx),
                                 _dev(dL_dimage), C.byref(g2) if g2 is not None else None, pg, C.c_void_p(ws.data_ptr()),
                                 C.c_size_t(ws.numel()), _stream(stream)))


def pbdr_l1_loss(image: torch.Tensor, target: torch.Tensor, loss: torch.Tensor, dL_dimage: torch.Tensor, stream=None) -> None:
    """image, target, dL_dimage [3, H, W]; loss: float32 device scalar, accumulated."""
    _, H, W = image.shape
    _check(lib().pbdr_l1_loss(C.c_int32(W), C.c_int32(H), _dev(image), _dev(target), _dev(loss), _dev(dL_dimage), _stream(stream)))


def pbdr_mark_visible(radius: torch.Tensor, visible: torch.Tensor, stream=None) -> None:
    _check(lib().pbdr_mark_visible(C.c_int32(radius.numel()), _dev(radius), _dev(visible), _stream(stream)))


def pbdr_adam_selective(param, grad, exp_avg, exp_avg_sq, visible, lr, beta1, beta2, eps, step, zero_grad=False,
                        stream=None) -> None:
    """One attribute tensor [planes, n] (or [n]); visible uint8 [n]."""
    n = int(param.shape[-1])
    planes = int(param.numel() // n) if n else 0
    cfg = CAdamConfig(float(lr), float(beta1), float(beta2), float(eps), int(step), int(bool(zero_grad)))
    _check(lib().pbdr_adam_selective(C.c_int32(n), C.c_int32(planes), _dev(param), _dev(grad), _dev(exp_avg), _dev(exp_avg_sq),
                                     _dev(visible), C.byref(cfg), _stream(stream)))


def _patch(patch) -> CPatch:
    x0, y0, x1, y1 = (int(v) for v in patch)
    return CPatch(x0, y0, x1, y1)


def pbdr_preprocess_patch(scene: Scene, cam: dict, patch, out: Splats, stream=None) -> None:
    """patch = (x0, y0, x1, y1): the pixel rectangle [x0, x1) x [y0, y1) of the camera's image."""
    s, c, p, o = scene.struct(), camera_struct(cam), _patch(patch), out.struct()
    _check(lib().pbdr_preprocess_patch(C.byref(s), C.byref(c), C.byref(p), C.byref(o), _stream(stream)))


def pbdr_render_fwd_patch(splats: Splats, cam: dict, patch, bg, dup_capacity: int, image, final_T, last_idx, ws,
                          stream=None) -> None:
    s, c, p = splats.struct(), camera_struct(cam), _patch(patch)
    bgv = (C.c_float * 3)(*[float(x) for x in bg])
    _check(lib().pbdr_render_fwd_patch(C.byref(s), C.byref(c), C.byref(p), bgv, C.c_uint64(dup_capacity), _dev(image),
                                       _dev(final_T), _dev(last_idx), C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()),
                                       _stream(stream)))


def pbdr_render_bwd_patch(scene, splats: Splats, cam: dict, patch, bg, dup_capacity: int, final_T, last_idx, dL_dimage,
                          g_splats: SplatGrads, grads, ws, stream=None, first_view=False) -> None:
    sp, c, p = splats.struct(), camera_struct(cam), _patch(patch)
    g2 = g_splats.struct() if g_splats is not None else None
    bgv = (C.c_float * 3)(*[float(x) for x in bg])
    if scene is not None:
        sc, g = scene.struct(), grads.struct(first_view)
        psc, pg = C.byref(sc), C.byref(g)
    else:
        psc, pg = None, None
    _check(lib().pbdr_render_bwd_patch(psc, C.byref(sp), C.byref(c), C.byref(p), bgv, C.c_uint64(dup_capacity),
                                       _dev(final_T), _dev(last_idx), _dev(dL_dimage), C.byref(g2) if g2 is not None else None, pg,
                                       C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), _stream(stream)))


def pbdr_preprocess_bwd(scene: Scene, cam: dict, splats: Splats, g_splats: SplatGrads, grads: Scene, stream=None, first_view=False) -> None:
    sc, c, sp, g2, g = scene.struct(), camera_struct(cam), splats.struct(), g_splats.struct(), grads.struct(first_view)
    _check(lib().pbdr_preprocess_bwd(C.byref(sc), C.byref(c), C.byref(sp), C.byref(g2), C.byref(g), _stream(stream)))


def pbdr_query_lists(ws, n, width, height, dup_capacity, stream=None):
    """Synchronises. Returns (num_dup, overflowed)."""
    out = C.c_uint64(0)
    st = lib().pbdr_query_lists(C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), C.c_int32(n), C.c_int32(width),
                                C.c_int32(height), C.c_uint64(dup_capacity), _stream(stream), C.byref(out))
    if st not in (PBDR_OK, PBDR_ERR_CAPACITY):
        raise PbdrError(st)
    return int(out.value), st == PBDR_ERR_CAPACITY


def pbdr_lists_view(ws, n, width, height, dup_capacity, _entry="pbdr_lists_view"):
    """Copies the sorted lists out of the workspace (synchronises): dict(P, keys, vals, ranges) as numpy."""
    keys, vals, ranges, nd = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_void_p()
    _check(getattr(lib(), _entry)(C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), C.c_int32(n), C.c_int32(width),
                                  C.c_int32(height), C.c_uint64(dup_capacity), _stream(None), C.byref(keys), C.byref(vals),
                                  C.byref(ranges), C.byref(nd)))
    torch.cuda.synchronize()
    base = ws.data_ptr()
    host = ws.cpu().numpy()

    def view(ptr, count, dt):
        off = ptr.value - base
        return host[off:off + count * np.dtype(dt).itemsize].view(dt).copy()
    tiles = ((width + 15) // 16) * ((height + 15) // 16)
    P_raw = int(view(nd, 1, np.uint32)[0])
    P = min(P_raw, max(int(dup_capacity), 1))
    return dict(P=P, P_raw=P_raw, keys=view(keys, P, np.uint64), vals=view(vals, P, np.uint32),
                ranges=view(ranges, 2 * tiles, np.uint32).reshape(tiles, 2))


def pbdr_tile_order_view(ws, n, width, height, dup_capacity, tiles, surfels=False):
    """Copies out (synchronises) the order in which the compositing kernels take the `tiles` tiles of the last call's grid."""
    ptr = C.c_void_p()
    _check(lib().pbdr_tile_order_view(C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), C.c_int32(n), C.c_int32(width),
                                      C.c_int32(height), C.c_uint64(dup_capacity), C.c_int32(int(bool(surfels))), C.byref(ptr)))
    torch.cuda.synchronize()
    off = ptr.value - ws.data_ptr()
    return ws[off:off + 4 * tiles].cpu().numpy().view(np.uint32).copy()


def pbdr_render_stats(cam: dict, n, dup_capacity, ws, stream=None, _entry="pbdr_render_stats"):
    """(examined, blended) pair counts of a forward pass over the lists now in the workspace. Synchronises."""
    c = camera_struct(cam)
    counters = torch.zeros(2, dtype=torch.int64, device=ws.device)
    _check(getattr(lib(), _entry)(C.byref(c), C.c_int32(n), C.c_uint64(dup_capacity), _dev(counters),
                                   C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), _stream(stream)))
    torch.cuda.synchronize()
    out = counters.cpu().numpy()
    return int(out[0]), int(out[1])


def profile_kernel_names():
    L = lib()
    return [L.pbdr_profile_kernel_name(C.c_int32(i)).decode() for i in range(int(L.pbdr_profile_kernel_count()))]


def pbdr_profile_begin(kernel_mask: int, max_records: int) -> None:
    _check(lib().pbdr_profile_begin(C.c_uint32(kernel_mask), C.c_int32(max_records)))


def pbdr_profile_reset() -> None:
    _check(lib().pbdr_profile_reset())


def pbdr_profile_collect(kernel_id: int):
    """(total_ms, records) for one kernel id; waits for the recorded events."""
    ms, cnt = C.c_double(0.0), C.c_int32(0)
    _check(lib().pbdr_profile_collect(C.c_int32(kernel_id), C.byref(ms), C.byref(cnt)))
    return float(ms.value), int(cnt.value)


def pbdr_profile_end() -> None:
    _check(lib().pbdr_profile_end())


# ---------------------------------------------------------------------------------------------- 2D Gaussian surfels
@dataclass
class Scene2D:
    """Surfel parameters on the device: mean[3,n], tan_u[3,n], tan_v[3,n], log_scale[2,n], logit[n], sh[K,3,n]."""
    n: int
    sh_degree: int
    mean: torch.Tensor
    tan_u: torch.Tensor
    tan_v: torch.Tensor
    log_scale: torch.Tensor
    logit: torch.Tensor
    sh: torch.Tensor

    @staticmethod
    def from_numpy(sc: dict, device="cuda") -> "Scene2D":
        def up(a, perm):
            return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.float32).transpose(perm))).to(device)
        n = int(sc["mean"].shape[0])
        return Scene2D(n, int(sc["sh_degree"]), up(sc["mean"], (1, 0)), up(sc["tan_u"], (1, 0)), up(sc["tan_v"], (1, 0)),
                       up(sc["log_scale"], (1, 0)),
                       torch.from_numpy(np.ascontiguousarray(sc["logit"], dtype=np.float32)).to(device), up(sc["sh"], (1, 2, 0)))

    def zeros_like(self) -> "Scene2D":
        return Scene2D(self.n, self.sh_degree, torch.zeros_like(self.mean), torch.zeros_like(self.tan_u),
                       torch.zeros_like(self.tan_v), torch.zeros_like(self.log_scale), torch.zeros_like(self.logit),
                       torch.zeros_like(self.sh))

    def to_numpy(self) -> dict:
        return dict(mean=self.mean.cpu().numpy().T.copy(), tan_u=self.tan_u.cpu().numpy().T.copy(),
                    tan_v=self.tan_v.cpu().numpy().T.copy(), log_scale=self.log_scale.cpu().numpy().T.copy(),
                    logit=self.logit.cpu().numpy().copy(), sh=self.sh.cpu().numpy().transpose(2, 0, 1).copy(),
                    sh_degree=self.sh_degree)

    def struct(self, first_view=False) -> CScene2D:
        return CScene2D(self.n, self.sh_degree, _dev(self.mean), _dev(self.tan_u), _dev(self.tan_v), _dev(self.log_scale),
                        _dev(self.logit), _dev(self.sh), int(bool(first_view)))


@dataclass
class Splats2D:
    """Per-view surfel state (Table 3b), SoA planes; T is the 3x3 ray transform, row-major over its 9 planes."""
    n: int
    mean2d: torch.Tensor
    T: torch.Tensor
    opacity: torch.Tensor
    color: torch.Tensor
    radius: torch.Tensor
    depth: torch.Tensor
    normal: torch.Tensor

    @staticmethod
    def empty(n, device="cuda") -> "Splats2D":
        f = dict(dtype=torch.float32, device=device)
        return Splats2D(n, torch.empty((2, n), **f), torch.empty((9, n), **f), torch.empty(n, **f), torch.empty((3, n), **f),
                        torch.empty(n, dtype=torch.int32, device=device), torch.empty(n, **f), torch.empty((3, n), **f))

    @staticmethod
    def from_numpy(st: dict, device="cuda") -> "Splats2D":
        def up(a, dt=np.float32):
            a = np.asarray(a, dtype=dt)
            return torch.from_numpy(np.ascontiguousarray(a.T if a.ndim == 2 else a)).to(device)
        n = int(np.asarray(st["opacity"]).shape[0])
        normal = st["normal"] if "normal" in st else np.zeros((n, 3))
        return Splats2D(n, up(st["mean2d"]), up(st["T"]), up(st["opacity"]), up(st["color"]), up(st["radius"], np.int32),
                        up(st["depth"]), up(normal))

    def to_numpy(self) -> dict:
        return dict(mean2d=self.mean2d.cpu().numpy().T.copy(), T=self.T.cpu().numpy().T.copy(),
                    opacity=self.opacity.cpu().numpy().copy(), color=self.color.cpu().numpy().T.copy(),
                    radius=self.radius.cpu().numpy().copy(), depth=self.depth.cpu().numpy().copy(),
                    normal=self.normal.cpu().numpy().T.copy())

    def struct(self) -> CSplats2D:
        return CSplats2D(self.n, _dev(self.mean2d), _dev(self.T), _dev(self.opacity), _dev(self.color), _dev(self.radius),
                         _dev(self.depth), _dev(self.normal))


@dataclass
class SplatGrads2D:
    n: int
    mean2d: torch.Tensor
    T: torch.Tensor
    opacity: torch.Tensor
    color: torch.Tensor

    @staticmethod
    def empty(n, device="cuda") -> "SplatGrads2D":
        f = dict(dtype=torch.float32, device=device)
        return SplatGrads2D(n, torch.empty((2, n), **f), torch.empty((9, n), **f), torch.empty(n, **f), torch.empty((3, n), **f))

    @staticmethod
    def from_numpy(d: dict, device="cuda") -> "SplatGrads2D":
        def up(a):
            a = np.asarray(a, dtype=np.float32)
            return torch.from_numpy(np.ascontiguousarray(a.T if a.ndim == 2 else a)).to(device)
        n = int(np.asarray(d["opacity"]).shape[0])
        return SplatGrads2D(n, up(d["mean2d"]), up(d["T"]), up(d["opacity"]), up(d["color"]))

    def to_numpy(self) -> dict:
        return dict(mean2d=self.mean2d.cpu().numpy().T.copy(), T=self.T.cpu().numpy().T.copy(),
                    opacity=self.opacity.cpu().numpy().copy(), color=self.color.cpu().numpy().T.copy())

    def struct(self) -> CSplatGrads2D:
        return CSplatGrads2D(self.n, _dev(self.mean2d), _dev(self.T), _dev(self.opacity), _dev(self.color))


def pbdr2d_workspace_bytes(n, width, height, dup_capacity) -> int:
    out = C.c_size_t(0)
    _check(lib().pbdr2d_workspace_bytes(C.c_int32(n), C.c_int32(width), C.c_int32(height), C.c_uint64(dup_capacity),
                                        C.byref(out)))
    return int(out.value)


def alloc_workspace2d(n, width, height, dup_capacity, device="cuda") -> torch.Tensor:
    return _alloc_ws(pbdr2d_workspace_bytes(n, width, height, dup_capacity), device)


def pbdr2d_preprocess(scene: Scene2D, cam: dict, out: Splats2D, stream=None) -> None:
    s, c, o = scene.struct(), camera_struct(cam), out.struct()
    _check(lib().pbdr2d_preprocess(C.byref(s), C.byref(c), C.byref(o), _stream(stream)))


def pbdr2d_render_fwd(splats: Splats2D, cam: dict, bg, dup_capacity: int, image, final_T, last_idx, ws, stream=None) -> None:
    s, c = splats.struct(), camera_struct(cam)
    bgv = (C.c_float * 3)(*[float(x) for x in bg])
    _check(lib().pbdr2d_render_fwd(C.byref(s), C.byref(c), bgv, C.c_uint64(dup_capacity), _dev(image), _dev(final_T),
                                   _dev(last_idx), C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), _stream(stream)))


def pbdr2d_render_bwd(scene, splats: Splats2D, cam: dict, bg, dup_capacity: int, final_T, last_idx, dL_dimage,
                      g_splats: SplatGrads2D, grads, ws, stream=None, first_view=False) -> None:
    sp, c = splats.struct(), camera_struct(cam)
    g2 = g_splats.struct() if g_splats is not None else None      # None (with scene/grads given): no splat-state gradient output
    bgv = (C.c_float * 3)(*[float(x) for x in bg])
    if scene is not None:
        sc, g = scene.struct(), grads.struct(first_view)
        psc, pg = C.byref(sc), C.byref(g)
    else:
        psc, pg = None, None
    _check(lib().pbdr2d_render_bwd(psc, C.byref(sp), C.byref(c), bgv, C.c_uint64(dup_capacity), _dev(final_T), _dev(last_idx),
                                   _dev(dL_dimage), C.byref(g2) if g2 is not None else None, pg, C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()),
                                   _stream(stream)))


def pbdr2d_preprocess_patch(scene: Scene2D, cam: dict, patch, out: Splats2D, stream=None) -> None:
    s, c, p, o = scene.struct(), camera_struct(cam), _patch(patch), out.struct()
    _check(lib().pbdr2d_preprocess_patch(C.byref(s), C.byref(c), C.byref(p), C.byref(o), _stream(stream)))


def pbdr2d_render_fwd_patch(splats: Splats2D, cam: dict, patch, bg, dup_capacity: int, image, final_T, last_idx, ws,
                            stream=None) -> None:
    s, c, p = splats.struct(), camera_struct(cam), _patch(patch)
    bgv = (C.c_float * 3)(*[float(x) for x in bg])
    _check(lib().pbdr2d_render_fwd_patch(C.byref(s), C.byref(c), C.byref(p), bgv, C.c_uint64(dup_capacity), _dev(image),
                                         _dev(final_T), _dev(last_idx), C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()),
                                         _stream(stream)))


def pbdr2d_render_bwd_patch(scene, splats: Splats2D, cam: dict, patch, bg, dup_capacity: int, final_T, last_idx, dL_dimage,
                            g_splats: SplatGrads2D, grads, ws, stream=None, first_view=False) -> None:
    sp, c, p = splats.struct(), camera_struct(cam), _patch(patch)
    g2 = g_splats.struct() if g_splats is not None else None
    bgv = (C.c_float * 3)(*[float(x) for x in bg])
    if scene is not None:
        sc, g = scene.struct(), grads.struct(first_view)
        psc, pg = C.byref(sc), C.byref(g)
    else:
        psc, pg = None, None
    _check(lib().pbdr2d_render_bwd_patch(psc, C.byref(sp), C.byref(c), C.byref(p), bgv, C.c_uint64(dup_capacity),
                                         _dev(final_T), _dev(last_idx), _dev(dL_dimage), C.byref(g2) if g2 is not None else None, pg,
                                         C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), _stream(stream)))


def pbdr2d_preprocess_bwd(scene: Scene2D, cam: dict, splats: Splats2D, g_splats: SplatGrads2D, grads: Scene2D, stream=None, first_view=False) -> None:
    sc, c, sp, g2, g = scene.struct(), camera_struct(cam), splats.struct(), g_splats.struct(), grads.struct(first_view)
    _check(lib().pbdr2d_preprocess_bwd(C.byref(sc), C.byref(c), C.byref(sp), C.byref(g2), C.byref(g), _stream(stream)))


def pbdr2d_lists_view(ws, n, width, height, dup_capacity):
    return pbdr_lists_view(ws, n, width, height, dup_capacity, _entry="pbdr2d_lists_view")


def pbdr2d_render_stats(cam: dict, n, dup_capacity, ws, stream=None):
    return pbdr_render_stats(cam, n, dup_capacity, ws, stream, _entry="pbdr2d_render_stats")
