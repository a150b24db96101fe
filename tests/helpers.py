"""Shared test helpers (no method arithmetic beyond what a test states as its own independent check)."""
import numpy as np

TILE = 16


def simple_camera(width, height, f, z_cam, near=0.2, far=1e10, radius_clip=0.0):
    """Camera at (0,0,-z_cam) looking down +z: R = I, t = (0,0,z_cam)."""
    return dict(width=width, height=height, fx=float(f), fy=float(f), cx=0.5 * width, cy=0.5 * height,
                R=np.eye(3), t=np.array([0.0, 0.0, float(z_cam)]), near=near, far=far, radius_clip=radius_clip)


def one_point_scene(mean, log_scale, quat, logit, rgb=None, sh=None, sh_degree=0):
    K = (sh_degree + 1) ** 2
    if sh is None:
        sh = np.zeros((1, K, 3))
        sh[0, 0, :] = (np.asarray(rgb, dtype=np.float64) - 0.5) / 0.28209479177387814
    return dict(mean=np.asarray(mean, dtype=np.float64).reshape(1, 3),
                log_scale=np.asarray(log_scale, dtype=np.float64).reshape(1, 3),
                quat=np.asarray(quat, dtype=np.float64).reshape(1, 4),
                logit=np.asarray([logit], dtype=np.float64), sh=np.asarray(sh, dtype=np.float64).reshape(1, K, 3),
                sh_degree=sh_degree)


def to_f64(scene):
    out = dict(scene)
    for k in ("mean", "log_scale", "quat", "tan_u", "tan_v", "logit", "sh"):
        if k in scene:
            out[k] = np.asarray(scene[k], dtype=np.float64).copy()
    return out


def splat_state(mean2d, conic, opacity, color, radius):
    n = len(opacity)
    return dict(mean2d=np.asarray(mean2d, dtype=np.float64).reshape(n, 2),
                conic=np.asarray(conic, dtype=np.float64).reshape(n, 3),
                opacity=np.asarray(opacity, dtype=np.float64).reshape(n),
                color=np.asarray(color, dtype=np.float64).reshape(n, 3),
                radius=np.asarray(radius, dtype=np.int32).reshape(n))


def tiles_xy(width, height):
    return (width + TILE - 1) // TILE, (height + TILE - 1) // TILE


GRAD_RTOL = 1e-3      # gradients: 1e-3 relative ...
GRAD_FLOOR = 1e-5     # ... + 1e-5 of the largest reference magnitude of the attribute
IMG_ATOL = 1e-4       # image and final_T: absolute


def grad_close(name, got, ref, report=True):
    """Every element: |got - ref| <= 1e-3 |ref| + 1e-5 max|ref| (max over the compared elements of the attribute).
    No element is exempt here: a caller may leave elements out only on the strength of a flag the oracle raised.
    Prints the worst error over its tolerance, so that the headroom is on record."""
    ref = np.asarray(ref, dtype=np.float64); got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    err = np.abs(got - ref)
    tol = GRAD_RTOL * np.abs(ref) + GRAD_FLOOR * max(float(np.abs(ref).max()), 1e-30)
    worst = float((err / tol).max())
    if report:
        print(f"[parity] {name}: worst |err|/tol = {worst:.3f} over {ref.size} elements (max|ref| = {float(np.abs(ref).max()):.3e})")
    bad = err > tol
    assert not bad.any(), (name, int(bad.sum()), ref.size, worst, float(err.max()), float(np.abs(ref).max()))
    return worst
