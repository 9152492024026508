"""Shared test helpers: node coordinates and small trees (no method arithmetic)."""
import numpy as np


def coords(leaves):
    """x, y, z arrays (n,8,8,8) [k][j][i] of owned-node coordinates."""
    lv = np.asarray(leaves, dtype=np.int64)
    h = 2.0 ** -(lv[:, 0] + 3.0)
    i = np.arange(8.0)
    n = lv.shape[0]
    x = ((8.0 * lv[:, 1])[:, None, None, None] + i[None, None, None, :]) * h[:, None, None, None]
    y = ((8.0 * lv[:, 2])[:, None, None, None] + i[None, None, :, None]) * h[:, None, None, None]
    z = ((8.0 * lv[:, 3])[:, None, None, None] + i[None, :, None, None]) * h[:, None, None, None]
    s = (n, 8, 8, 8)
    return np.broadcast_to(x, s), np.broadcast_to(y, s), np.broadcast_to(z, s)


def padded_coords(leaves):
    """unwrapped coordinates of all 14^3 padded points (may lie outside [0,1))."""
    lv = np.asarray(leaves, dtype=np.int64)
    h = 2.0 ** -(lv[:, 0] + 3.0)
    i = np.arange(14.0) - 3.0
    n = lv.shape[0]
    x = ((8.0 * lv[:, 1])[:, None, None, None] + i[None, None, None, :]) * h[:, None, None, None]
    y = ((8.0 * lv[:, 2])[:, None, None, None] + i[None, None, :, None]) * h[:, None, None, None]
    z = ((8.0 * lv[:, 3])[:, None, None, None] + i[None, :, None, None]) * h[:, None, None, None]
    s = (n, 14, 14, 14)
    return np.broadcast_to(x, s), np.broadcast_to(y, s), np.broadcast_to(z, s)


def away_from_wrap(leaves):
    """mask of blocks whose padded box stays strictly inside the unit cube"""
    lv = np.asarray(leaves, dtype=np.int64)
    n = 1 << lv[:, 0]
    ok = np.ones(lv.shape[0], dtype=bool)
    for c in (1, 2, 3):
        ok &= (lv[:, c] >= 1) & (lv[:, c] <= n - 2)
    return ok


def uniform_to_grid(leaves, zipped):
    """uniform-level tree: zipped (n,8,8,8) -> global array [Z][Y][X]"""
    lv = np.asarray(leaves, dtype=np.int64)
    l = int(lv[0, 0])
    assert (lv[:, 0] == l).all()
    N = 8 << l
    g = np.empty((N, N, N))
    for b in range(lv.shape[0]):
        ix, iy, iz = lv[b, 1:]
        g[8 * iz:8 * iz + 8, 8 * iy:8 * iy + 8, 8 * ix:8 * ix + 8] = zipped[b]
    return g


def grid_to_uniform(leaves, g):
    lv = np.asarray(leaves, dtype=np.int64)
    out = np.empty((lv.shape[0], 8, 8, 8))
    for b in range(lv.shape[0]):
        ix, iy, iz = lv[b, 1:]
        out[b] = g[8 * iz:8 * iz + 8, 8 * iy:8 * iy + 8, 8 * ix:8 * ix + 8]
    return out
