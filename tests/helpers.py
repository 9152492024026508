"""Shared test helpers: node coordinates, small trees and the comparison against the oracle (no method arithmetic)."""
import numpy as np

KIND = {"DERIVS": 0, "WAVE": 1, "BURGERS": 2, "SYN24": 3}
# fp64 values: pass iff |gpu - oracle| <= RTOL |oracle| + ATOL
RTOL, ATOL = 1e-12, 1e-13


def assert_close(got, want, what):
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape
    assert np.isfinite(want).all() and np.isfinite(got).all(), what
    err = np.abs(got - want)
    bound = RTOL * np.abs(want) + ATOL
    nz = int((got != want).sum())
    print("%s: %d of %d values differ, worst |diff|/bound = %.3g" % (what, nz, got.size, (err / bound).max()), flush=True)
    assert (err <= bound).all(), what


def dev_empty(shape, dev):
    """NaN-filled device array, so that a point the kernel failed to write cannot pass by accident"""
    import torch
    return torch.full(shape, float("nan"), dtype=torch.float64, device=dev)


def trees(orc, name, seed=1):
    """the oracle's and the library's tree of a named workload"""
    import paper_2007_12792_amd as octfd
    import synthdata as sd
    p = sd.tree_params(name, seed)
    return orc.Tree.build(**p), octfd.Tree.build(**p)


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
