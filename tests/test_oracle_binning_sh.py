"""Pins for the oracle's tile lists (brute force) and spherical-harmonic basis (quadrature, library)."""
import numpy as np
import pytest
from scipy import special

import oracle
from helpers import TILE, tiles_xy


def _random_splats(seed, n, width, height, rmax=40):
    rng = np.random.default_rng(seed)
    mean2d = np.stack([rng.uniform(-30, width + 30, n), rng.uniform(-30, height + 30, n)], 1)
    mean2d = mean2d.astype(np.float32).astype(np.float64)
    radius = rng.integers(0, rmax, n).astype(np.int32)          # some zeros = culled
    depth = rng.uniform(0.5, 9.0, n).astype(np.float32)
    depth[rng.integers(0, n, n // 4)] = depth[0]                 # plenty of exact depth ties
    return mean2d, radius, depth


@pytest.mark.parametrize("seed,width,height", [(0, 64, 48), (1, 100, 70), (2, 16, 16), (3, 33, 17)])
def test_tile_lists_brute_force(seed, width, height):
    n = 200
    mean2d, radius, depth = _random_splats(seed, n, width, height)
    lists = oracle.bin_sort(mean2d, radius, depth, width, height)
    TX, TY = tiles_xy(width, height)
    bits = depth.view(np.uint32)
    total = 0
    for ty in range(TY):
        for tx in range(TX):
            # a tile belongs to the splat's square [m-r, m+r] (rounded out to the tile grid) iff, per axis,
            # 16*t + 16 > m - r  and  16*t + 1 <= m + r
            members = [i for i in range(n) if radius[i] > 0
                       and TILE * tx + TILE > mean2d[i, 0] - radius[i] and TILE * tx + 1 <= mean2d[i, 0] + radius[i]
                       and TILE * ty + TILE > mean2d[i, 1] - radius[i] and TILE * ty + 1 <= mean2d[i, 1] + radius[i]]
            members.sort(key=lambda i: (int(bits[i]), i))
            s, e = lists["ranges"][ty * TX + tx]
            assert lists["vals"][s:e].tolist() == members, (tx, ty)
            if members:
                keys = [((ty * TX + tx) << 32) | int(bits[i]) for i in members]
                assert lists["keys"][s:e].tolist() == keys
            else:
                assert (s, e) == (0, 0)
            total += len(members)
    assert total == lists["P"]
    assert (np.diff(lists["keys"].astype(np.uint64)) >= 0).all() if lists["P"] > 1 else True


def test_tile_lists_degenerate():
    # nothing visible
    lists = oracle.bin_sort(np.zeros((3, 2)), np.zeros(3, dtype=np.int32), np.ones(3, dtype=np.float32), 32, 32)
    assert lists["P"] == 0 and (lists["ranges"] == 0).all()
    # one splat covering everything
    lists = oracle.bin_sort(np.array([[16.0, 16.0]]), np.array([100], dtype=np.int32), np.ones(1, dtype=np.float32), 32, 32)
    assert lists["P"] == 4 and lists["ranges"].tolist() == [[0, 1], [1, 2], [2, 3], [3, 4]]
    # exactly on a tile border: centre 16.0, radius 1 -> reaches pixels 15..17 -> both tiles
    r = oracle.tile_rect(16.0, 8.0, 1, 32, 16)
    assert r.tolist() == [0, 0, 2, 1]
    r = oracle.tile_rect(24.9, 8.0, 3, 32, 16)      # stays inside tile 1: 21.9 .. 27.9
    assert r.tolist() == [1, 0, 2, 1]
    r = oracle.tile_rect(-500.0, 8.0, 3, 32, 16)    # off-screen: empty
    assert (r[2] - r[0]) * (r[3] - r[1]) == 0


# ------------------------------------------------------------------ spherical harmonics
def _dirs(n, seed=0):
    v = np.random.default_rng(seed).normal(size=(n, 3))
    return v / np.linalg.norm(v, axis=1, keepdims=True)


def test_sh_matches_library_real_harmonics():
    """Y_k = (-1)^m x the real harmonic built from scipy's complex Y_l^m (Condon-Shortley phase kept)."""
    for d in _dirs(50):
        Y = oracle.sh_basis(3, d)
        theta = np.arccos(d[2]); phi = np.arctan2(d[1], d[0])
        for l in range(4):
            for m in range(-l, l + 1):
                y = special.sph_harm_y(l, abs(m), theta, phi)
                if m == 0:
                    ref = y.real
                elif m > 0:
                    ref = np.sqrt(2) * (-1) ** m * y.real
                else:
                    ref = np.sqrt(2) * (-1) ** m * y.imag
                ref *= (-1) ** m
                assert abs(Y[l * l + l + m] - ref) < 1e-13, (l, m)


def test_sh_orthonormal_by_quadrature():
    nt, nphi = 64, 128
    x, w = np.polynomial.legendre.leggauss(nt)      # cos(theta) nodes
    phi = (np.arange(nphi) + 0.5) * 2 * np.pi / nphi
    G = np.zeros((16, 16))
    for ct, wt in zip(x, w):
        st = np.sqrt(1 - ct * ct)
        for p in phi:
            Y = oracle.sh_basis(3, np.array([st * np.cos(p), st * np.sin(p), ct]))
            G += wt * (2 * np.pi / nphi) * np.outer(Y, Y)
    np.testing.assert_allclose(G, np.eye(16), atol=1e-12)


def test_sh_degree_truncation_and_dc():
    d = _dirs(1)[0]
    for deg, K in [(0, 1), (1, 4), (2, 9), (3, 16)]:
        Y = oracle.sh_basis(deg, d)
        assert (Y[K:] == 0).all() and (Y[:K] != 0).all()
    assert abs(oracle.sh_basis(0, d)[0] - 0.28209479177387814) < 1e-15
