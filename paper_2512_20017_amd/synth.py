"""Seeded synthetic scenes, cameras and loss targets.

These stand in for the paper's datasets (Table 1: Rubble, Ithaca365, Campus, BigCity, Sci-Art), which are
not available: same shapes, sizes and value distributions as the benchmark configurations. This module holds
no arithmetic of the rendering method; it serves both the HIP path and the CPU oracle, and imports neither.

Scene arrays are float32 in the paper's "S x l" layout (Sec. 3.1): mean[n,3], log_scale[n,3], quat[n,4]
(w,x,y,z, not normalised), logit[n], sh[n,K,3], K = (sh_degree+1)^2 -- 59 floats per point at degree 3.
A camera is a dict: width, height, fx, fy, cx, cy, R (3x3 world->camera, +x right, +y down, +z forward),
t (3), near, far, radius_clip.
"""
import math

import numpy as np

SH_C0 = 0.28209479177387814  # Y_0^0, used only to turn a target RGB into a DC coefficient (config 1)


def _rng(seed, stream):
    return np.random.Generator(np.random.PCG64([int(seed), int(stream)]))


def pinhole(width, height, fov_deg, R, t, near=0.2, far=1e10, radius_clip=0.0):
    """Horizontal field of view; square pixels; principal point at the image centre."""
    f = 0.5 * width / math.tan(math.radians(fov_deg) * 0.5)
    return dict(width=int(width), height=int(height), fx=f, fy=f, cx=0.5 * width, cy=0.5 * height,
                R=np.asarray(R, dtype=np.float64).reshape(3, 3), t=np.asarray(t, dtype=np.float64).reshape(3),
                near=float(near), far=float(far), radius_clip=float(radius_clip))


def look_at(eye, target, up):
    """World->camera rotation and translation for a camera at `eye` looking at `target`."""
    eye = np.asarray(eye, dtype=np.float64); target = np.asarray(target, dtype=np.float64)
    up = np.asarray(up, dtype=np.float64)
    z = target - eye; z /= np.linalg.norm(z)
    x = np.cross(z, up)
    if np.linalg.norm(x) < 1e-9:
        x = np.cross(z, np.array([1.0, 0.0, 0.0]))
    x /= np.linalg.norm(x)
    y = np.cross(z, x)
    R = np.stack([x, y, z])
    return R, -R @ eye


def _attributes(rng, n, sh_degree, ls_mu, ls_sigma, logit_sigma, dc_mode):
    K = (sh_degree + 1) ** 2
    log_scale = rng.normal(ls_mu, ls_sigma, size=(n, 3)).astype(np.float32)
    quat = rng.normal(0.0, 1.0, size=(n, 4)).astype(np.float32)
    logit = rng.normal(0.0, logit_sigma, size=n).astype(np.float32)
    sh = np.zeros((n, K, 3), dtype=np.float32)
    u = rng.uniform(0.0, 1.0, size=(n, 3))
    if dc_mode == "rgb":      # rendered colour at degree 0 equals the drawn RGB
        sh[:, 0, :] = ((u - 0.5) / SH_C0).astype(np.float32)
    else:                     # the DC coefficient itself is U[0,1]
        sh[:, 0, :] = u.astype(np.float32)
    if K > 1:
        sh[:, 1:, :] = rng.normal(0.0, 0.05, size=(n, K - 1, 3)).astype(np.float32)
    return log_scale, quat, logit, sh


def _gmm_means(rng, n, n_comp, lo, hi, sig_lo, sig_hi, z_squash=1.0):
    lo = np.asarray(lo, dtype=np.float64); hi = np.asarray(hi, dtype=np.float64)
    centres = rng.uniform(lo, hi, size=(n_comp, 3))
    sig = np.exp(rng.uniform(math.log(sig_lo), math.log(sig_hi), size=n_comp))
    wts = rng.uniform(0.5, 1.5, size=n_comp); wts /= wts.sum()
    comp = rng.choice(n_comp, size=n, p=wts)
    noise = rng.normal(0.0, 1.0, size=(n, 3))
    noise[:, 2] *= z_squash
    return (centres[comp] + noise * sig[comp][:, None]).astype(np.float32)


def _part1by2(v):
    """Spread the low 21 bits of v so that two zero bits separate consecutive bits."""
    v = v.astype(np.uint64) & np.uint64(0x1FFFFF)
    v = (v | (v << np.uint64(32))) & np.uint64(0x1F00000000FFFF)
    v = (v | (v << np.uint64(16))) & np.uint64(0x1F0000FF0000FF)
    v = (v | (v << np.uint64(8))) & np.uint64(0x100F00F00F00F00F)
    v = (v | (v << np.uint64(4))) & np.uint64(0x10C30C30C30C30C3)
    v = (v | (v << np.uint64(2))) & np.uint64(0x1249249249249249)
    return v


def zorder_permutation(mean):
    """Permutation that puts points in Z-order (Morton order) of their positions, 21 bits per axis.
    The paper keeps its point cloud in this order so that contiguous blocks of points are spatially local
    (Sec. 4.2.1 point groups; App. D.1 "Z-order linearization")."""
    lo = mean.min(axis=0).astype(np.float64); hi = mean.max(axis=0).astype(np.float64)
    q = ((mean.astype(np.float64) - lo) / np.maximum(hi - lo, 1e-30) * (2 ** 21 - 1)).astype(np.uint64)
    code = _part1by2(q[:, 0]) | (_part1by2(q[:, 1]) << np.uint64(1)) | (_part1by2(q[:, 2]) << np.uint64(2))
    return np.argsort(code, kind="stable")


def _reorder(scene, perm):
    return {k: (v[perm] if isinstance(v, np.ndarray) else v) for k, v in scene.items()}


def scene_tiny(seed=0, n=4096, sh_degree=0):
    """Config 1: means U[-1,1]^3, log-scales N(-3.5,0.3), opacity sigmoid(N(0,1)), degree-0 RGB ~ U[0,1]."""
    rng = _rng(seed, 1)
    mean = rng.uniform(-1.0, 1.0, size=(n, 3)).astype(np.float32)
    log_scale, quat, logit, sh = _attributes(rng, n, sh_degree, -3.5, 0.3, 1.0, "rgb")
    return dict(mean=mean, log_scale=log_scale, quat=quat, logit=logit, sh=sh, sh_degree=sh_degree)


def camera_tiny(width=128, height=128):
    """Config 1: eye (0,0,-3) looking down +z at the origin, 60 degree FoV."""
    return pinhole(width, height, 60.0, np.eye(3), [0.0, 0.0, 3.0])


def scene_mid(seed=0, n=1_000_000, sh_degree=3, n_comp=64, zorder=True):
    """Config 2/3: 64-component mixture in a 20^3 box, log-scales N(-4,0.5), opacity sigmoid(N(0,1.5)), SH3.
    Points are stored in Z-order of their positions, as the paper's system stores its point cloud."""
    rng = _rng(seed, 2)
    mean = _gmm_means(rng, n, n_comp, [-10, -10, -10], [10, 10, 10], 0.3, 2.0)
    log_scale, quat, logit, sh = _attributes(rng, n, sh_degree, -4.0, 0.5, 1.5, "dc")
    sc = dict(mean=mean, log_scale=log_scale, quat=quat, logit=logit, sh=sh, sh_degree=sh_degree)
    return _reorder(sc, zorder_permutation(mean)) if zorder else sc


def cameras_sphere(count=16, radius=15.0, width=1920, height=1080, fov_deg=60.0):
    """Config 3: Fibonacci lattice on a sphere, looking at the centre, world up +y. Config 2 uses camera 0."""
    cams = []
    golden = math.pi * (3.0 - math.sqrt(5.0))
    for k in range(count):
        yy = 1.0 - 2.0 * (k + 0.5) / count
        rr = math.sqrt(max(0.0, 1.0 - yy * yy))
        th = golden * k
        eye = radius * np.array([rr * math.cos(th), yy, rr * math.sin(th)])
        R, t = look_at(eye, [0.0, 0.0, 0.0], [0.0, 1.0, 0.0])
        cams.append(pinhole(width, height, fov_deg, R, t))
    return cams


def scene_large(seed=0, n=8_000_000, sh_degree=3, n_comp=512, zorder=True):
    """Config 4: one GPU's share of a city-scale scene: 512-component mixture over 200 x 200 x 30 m, z up."""
    rng = _rng(seed, 4)
    mean = _gmm_means(rng, n, n_comp, [-100, -100, 0], [100, 100, 30], 1.0, 8.0, z_squash=0.3)
    log_scale, quat, logit, sh = _attributes(rng, n, sh_degree, -4.0, 0.5, 1.5, "dc")
    sc = dict(mean=mean, log_scale=log_scale, quat=quat, logit=logit, sh=sh, sh_degree=sh_degree)
    return _reorder(sc, zorder_permutation(mean)) if zorder else sc


def cameras_street(seed=0, count=8, width=3840, height=2160, fov_deg=70.0):
    """Config 4: street-level cameras 2 m above the ground plane, random position and yaw, world up +z."""
    rng = _rng(seed, 5)
    cams = []
    for _ in range(count):
        pos = np.array([rng.uniform(-100, 100), rng.uniform(-100, 100), 2.0])
        yaw = rng.uniform(0.0, 2.0 * math.pi)
        fwd = np.array([math.cos(yaw), math.sin(yaw), 0.0])
        R, t = look_at(pos, pos + fwd, [0.0, 0.0, 1.0])
        cams.append(pinhole(width, height, fov_deg, R, t))
    return cams


def scene_surfels(seed=0, n=1_000_000, sh_degree=3, n_comp=64, zorder=True):
    """Config 5: 2D Gaussian disks. Means as the mid scene; two raw tangent vectors ~ N(0,1)^3 (orthonormalised by the
    renderer, normal = their cross product); two log-scales N(-4,0.5); opacity sigmoid(N(0,1)); SH degree 3."""
    rng = _rng(seed, 6)
    mean = _gmm_means(rng, n, n_comp, [-10, -10, -10], [10, 10, 10], 0.3, 2.0)
    log_scale3, _, logit, sh = _attributes(rng, n, sh_degree, -4.0, 0.5, 1.0, "dc")
    tan_u = rng.normal(0.0, 1.0, size=(n, 3)).astype(np.float32)
    tan_v = rng.normal(0.0, 1.0, size=(n, 3)).astype(np.float32)
    sc = dict(mean=mean, tan_u=tan_u, tan_v=tan_v, log_scale=np.ascontiguousarray(log_scale3[:, :2]), logit=logit, sh=sh,
              sh_degree=sh_degree)
    return _reorder(sc, zorder_permutation(mean)) if zorder else sc


def random_small_surfels(seed, n, sh_degree, spread=0.6, ls_mu=-2.0, ls_sigma=0.4):
    """Small random surfel scene for parity sweeps and finite differences."""
    rng = _rng(seed, 10)
    mean = rng.uniform(-spread, spread, size=(n, 3)).astype(np.float32)
    log_scale3, _, logit, sh = _attributes(rng, n, sh_degree, ls_mu, ls_sigma, 1.0, "rgb")
    if sh_degree > 0:
        sh[:, 1:, :] *= 4.0
    tan_u = rng.normal(0.0, 1.0, size=(n, 3)).astype(np.float32)
    tan_v = rng.normal(0.0, 1.0, size=(n, 3)).astype(np.float32)
    return dict(mean=mean, tan_u=tan_u, tan_v=tan_v, log_scale=np.ascontiguousarray(log_scale3[:, :2]), logit=logit, sh=sh,
                sh_degree=sh_degree)


def target_image(seed, width, height):
    """Seeded U[0,1] ground-truth stand-in, [H,W,3] float32."""
    return _rng(seed, 7).uniform(0.0, 1.0, size=(height, width, 3)).astype(np.float32)


def random_small_scene(seed, n, sh_degree, spread=0.6, ls_mu=-2.2, ls_sigma=0.4):
    """Small random scene for parity sweeps and finite differences (few, fairly large splats)."""
    rng = _rng(seed, 9)
    mean = rng.uniform(-spread, spread, size=(n, 3)).astype(np.float32)
    log_scale, quat, logit, sh = _attributes(rng, n, sh_degree, ls_mu, ls_sigma, 1.0, "rgb")
    if sh_degree > 0:
        sh[:, 1:, :] *= 4.0  # make the view-dependent part matter
    return dict(mean=mean, log_scale=log_scale, quat=quat, logit=logit, sh=sh, sh_degree=sh_degree)
