"""Pins of the oracle's centred-stencil ghost rule (no GPU): uniform trees, an independent global
formulation on a two-level tree (exact in integers), polynomial reproduction through three levels,
bit-equality with the clamped rule wherever the two stencils coincide, and the smaller error
constant that motivates the variant."""
import numpy as np
import pytest

import synthdata as sd
from helpers import coords, padded_coords, uniform_to_grid

W = np.array([3.0, -25.0, 150.0, 150.0, -25.0, 3.0]) / 256.0


def uniform_tree(orc, level):
    return orc.Tree.build(level, level, np.zeros((1, 3), np.uint32), np.zeros(1, np.uint32))


def two_level_tree(orc):
    return orc.Tree.build(3, 4, np.array([[1 << 19] * 3], np.uint32), np.array([90000], np.uint32))


def ghost_source_level(t):
    """(n,14,14,14) level of the leaf that contains each padded point, by brute force on a cell map"""
    lv = t.leaves.astype(np.int64)
    lmax = int(lv[:, 0].max())
    n = 1 << lmax
    cell = np.empty((n, n, n), dtype=np.int64)            # level of the leaf covering each finest octant [z][y][x]
    for l, ix, iy, iz in lv:
        s = 1 << (lmax - l)
        cell[iz * s:(iz + 1) * s, iy * s:(iy + 1) * s, ix * s:(ix + 1) * s] = l
    out = np.empty((t.n, 14, 14, 14), dtype=np.int64)
    g = np.arange(14) - 3
    for b, (l, ix, iy, iz) in enumerate(lv):
        N = 8 << l
        sh = lmax - l
        px = (((8 * ix + g) % N) >> 3) << sh
        py = (((8 * iy + g) % N) >> 3) << sh
        pz = (((8 * iz + g) % N) >> 3) << sh
        out[b] = cell[np.ix_(pz, py, px)]
    return out


def test_uniform_tree_is_periodic_padding(orc):
    t = uniform_tree(orc, 3)
    u = np.random.default_rng(1).standard_normal((2, t.n, 8, 8, 8))
    assert (t.unzip_centred(u) == t.unzip(u)).all()


def test_interior_and_non_coarse_ghosts_equal_the_clamped_rule(orc):
    t = orc.Tree.build(**sd.tree_params("T4", 1))
    u = np.random.default_rng(2).standard_normal((1, t.n, 8, 8, 8))
    a, b = t.unzip(u)[0], t.unzip_centred(u)[0]
    src = ghost_source_level(t)
    own = t.leaves[:, 0].astype(np.int64)[:, None, None, None]
    assert (a[src >= own] == b[src >= own]).all()
    assert (orc.Tree.zip(b[None])[0] == u[0]).all()
    # coarser source: the two rules use the same nodes when every odd fine coordinate has its
    # centred stencil inside the source leaf (c0 = 2, 3 or 4), and then agree to the last bit
    lv = t.leaves.astype(np.int64)
    g = np.arange(14) - 3
    same = np.zeros(a.shape, dtype=bool)
    for blk in range(t.n):
        l = lv[blk, 0]
        ok = []
        for ax in (1, 2, 3):
            f = (8 * lv[blk, ax] + g) % 16               # fine coordinate inside an aligned coarse octant
            c0 = (f - 1) // 2
            ok.append((f % 2 == 0) | ((c0 >= 2) & (c0 <= 4)))
        same[blk] = ok[2][:, None, None] & ok[1][None, :, None] & ok[0][None, None, :]
    coarse = src < own
    assert coarse.sum() > 1000
    assert (a[coarse & same] == b[coarse & same]).all()
    assert (a[coarse & ~same] != b[coarse & ~same]).mean() > 0.9


def test_two_level_tree_equals_global_coarse_lattice_interpolation(orc):
    t = two_level_tree(orc)
    lv = t.leaves.astype(np.int64)
    assert set(lv[:, 0]) == {3, 4}
    rng = np.random.default_rng(3)
    u = rng.integers(-1000, 1000, size=(1, t.n, 8, 8, 8)).astype(np.float64)   # dyadic weights: all sums exact
    # the level-3 lattice function on the whole cube: level-3 leaves as stored, level-4 leaves injected
    G = np.empty((64, 64, 64))
    for b, (l, ix, iy, iz) in enumerate(lv):
        if l == 3:
            G[8 * iz:8 * iz + 8, 8 * iy:8 * iy + 8, 8 * ix:8 * ix + 8] = u[0, b]
        else:
            G[4 * iz:4 * iz + 4, 4 * iy:4 * iy + 4, 4 * ix:4 * ix + 4] = u[0, b][::2, ::2, ::2]

    def refine(A, axis):                                   # coarse periodic lattice -> fine lattice along one axis
        odd = sum(W[m] * np.roll(A, -(m - 2), axis) for m in range(6))
        out = np.empty([2 * s if d == axis else s for d, s in enumerate(A.shape)])
        sl_e = [slice(None)] * 3; sl_o = [slice(None)] * 3
        sl_e[axis] = slice(0, None, 2); sl_o[axis] = slice(1, None, 2)
        out[tuple(sl_e)] = A; out[tuple(sl_o)] = odd
        return out

    F = refine(refine(refine(G, 2), 1), 0)                 # x, then y, then z
    p = t.unzip_centred(u)[0]
    src = ghost_source_level(t)
    g = np.arange(14) - 3
    n = 0
    for b, (l, ix, iy, iz) in enumerate(lv):
        if l != 4:
            continue
        m = src[b] == 3
        if not m.any():
            continue
        want = F[np.ix_((8 * iz + g) % 128, (8 * iy + g) % 128, (8 * ix + g) % 128)]
        assert (p[b][m] == want[m]).all()
        n += int(m.sum())
    assert n > 10000


def poly5(x, y, z):
    return (1.0 + x - 2.0 * x ** 3 + 0.5 * x ** 5) * (2.0 - y ** 2 + y ** 5) * (1.0 + 3.0 * z ** 4 - z ** 5) + x * y * z


def test_polynomials_are_reproduced_through_three_levels(orc):
    t = orc.Tree.build(3, 5, np.array([[500000, 520000, 540000]], np.uint32), np.array([60000, 40000], np.uint32))
    assert set(t.leaves[:, 0]) == {3, 4, 5}
    from helpers import away_from_wrap
    x, y, z = coords(t.leaves)
    p = t.unzip_centred(poly5(x, y, z)[None])[0]
    X, Y, Z = padded_coords(t.leaves)
    ok = away_from_wrap(t.leaves)                          # a polynomial is not periodic
    # a coarse block's ghost layer may still reach across the wrap through the recursion: keep blocks two cells in
    lv = t.leaves.astype(np.int64)
    for c in (1, 2, 3):
        ok &= (lv[:, c] >= 2 * (1 << (lv[:, 0] - 3))) & (lv[:, c] < (1 << lv[:, 0]) - 2 * (1 << (lv[:, 0] - 3)))
    assert ok.sum() > 100 and (lv[ok, 0] == 5).any() and (lv[ok, 0] == 4).any()
    err = np.abs(p[ok] - poly5(X[ok], Y[ok], Z[ok]))
    assert err.max() < 5e-14 * 30


def test_error_constant_is_smaller_than_with_clamped_stencils(orc):
    t = two_level_tree(orc)
    x, y, z = coords(t.leaves)
    f = lambda x, y, z: np.sin(2 * np.pi * x) * np.cos(2 * np.pi * y) * np.sin(2 * np.pi * z + 0.3)
    X, Y, Z = padded_coords(t.leaves)
    src = ghost_source_level(t)
    coarse = src < t.leaves[:, 0].astype(np.int64)[:, None, None, None]
    e_clamped = np.abs(t.unzip(f(x, y, z)[None])[0] - f(X, Y, Z))[coarse].max()
    e_centred = np.abs(t.unzip_centred(f(x, y, z)[None])[0] - f(X, Y, Z))[coarse].max()
    assert e_centred < e_clamped / 10.0


def test_centred_step_equals_the_clamped_step_without_level_jumps_and_tracks_a_plane_wave(orc):
    t = uniform_tree(orc, 3)
    x, y, z = coords(t.leaves)
    om = 2 * np.pi * np.sqrt(2.0)
    ph = 2 * np.pi * (x + y)
    u = np.stack([np.sin(ph), -om * np.cos(ph)])
    dt = sd.time_step(3)
    a = t.rk4_step(1, u, dt, 0.1)
    b = t.rk4_step_centred(1, u, dt, 0.1)
    assert (a == b).all()                              # no coarser leaf anywhere: the same arithmetic
    # on a tree with level jumps the step stays close to the exact solution
    t2 = two_level_tree(orc)
    x, y, z = coords(t2.leaves)
    ph = 2 * np.pi * (x + y)
    v = np.stack([np.sin(ph), -om * np.cos(ph)])
    dt = sd.time_step(4)
    for _ in range(4):
        v = t2.rk4_step_centred(1, v, dt, 0.4)
    exact = np.sin(ph - om * 4 * dt)
    assert np.abs(v[0] - exact).max() < 2e-6


def test_F_centred_differentiates_a_polynomial_exactly_across_level_jumps(orc):
    """F_centred itself against a closed form: the centred rule reproduces polynomials of degree <= 5 in every
    ghost point, and the sixth-order stencils are exact on them, so on a three-level tree the derivatives of such
    a polynomial come out exact (to rounding, amplified by 1/h^2) at every point, next to level jumps too."""
    t = orc.Tree.build(3, 5, np.array([[500000, 520000, 540000]], np.uint32), np.array([60000, 40000], np.uint32))
    from helpers import away_from_wrap
    x, y, z = coords(t.leaves)
    f = poly5(x, y, z)
    got = t.F_centred(0, f[None])                          # DERIVS: (Dx, Dy, Dz, Laplacian)
    lv = t.leaves.astype(np.int64)
    ok = away_from_wrap(t.leaves)
    for c in (1, 2, 3):
        ok &= (lv[:, c] >= 2 * (1 << (lv[:, 0] - 3))) & (lv[:, c] < (1 << lv[:, 0]) - 2 * (1 << (lv[:, 0] - 3)))
    # the same derivatives by central differences of the closed form in much higher precision would need its
    # symbols; instead differentiate the polynomial numerically with a tiny complex step, which is exact to rounding
    hstep = 1e-30
    dx = np.imag(poly5(x + 1j * hstep, y, z)) / hstep
    dy = np.imag(poly5(x, y + 1j * hstep, z)) / hstep
    dz = np.imag(poly5(x, y, z + 1j * hstep)) / hstep
    scale = np.abs(f).max()
    ih = (8.0 * 2.0 ** lv[:, 0])[:, None, None, None]
    for name, g, want in (("Dx", got[0], dx), ("Dy", got[1], dy), ("Dz", got[2], dz)):
        err = np.abs(g - want)[ok]
        assert err.max() < 1e-13 * scale * ih[ok].max(), name
    # Laplacian: second complex-step differences lose precision; use the exactness of D2 on degree <= 5 through the
    # clamped rule's F on a uniform tree of the finest level as the independent reference at the same points
    fine = lv[:, 0] == 5
    tu = uniform_tree(orc, 5)
    xu, yu, zu = coords(tu.leaves)
    lap_u = tu.F(0, poly5(xu, yu, zu)[None])[3]
    key = {tuple(r[1:]): i for i, r in enumerate(tu.leaves.astype(np.int64))}
    sel = np.flatnonzero(ok & fine)
    assert sel.size > 50
    idx = np.array([key[tuple(lv[b, 1:])] for b in sel])
    # (blocks of the uniform tree next to the wrap see a discontinuous periodic extension, but those are excluded)
    assert np.abs(got[3][sel] - lap_u[idx]).max() < 1e-12 * scale * (8.0 * 32) ** 2
