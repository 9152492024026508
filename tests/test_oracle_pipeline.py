"""Pins of the oracle's unzip / rhs / zip / rk4 against independent evaluations (no GPU):
a uniform tree must reproduce a direct periodic uniform-grid computation, polynomials must be
reproduced at every ghost point of an adaptive tree, errors must fall at sixth order, the
24-field system must equal an analytic evaluation on polynomial data, and the Burgers and wave
steps must track their exact solutions."""
import numpy as np
import pytest

import synthdata as sd
from helpers import away_from_wrap, coords, grid_to_uniform, padded_coords, uniform_to_grid

TP = 2.0 * np.pi


# ---------------------------------------------------------------- independent uniform-grid operators
C1 = {1: 3.0 / 4.0, 2: -3.0 / 20.0, 3: 1.0 / 60.0}
C2 = {0: -49.0 / 18.0, 1: 3.0 / 2.0, 2: -3.0 / 20.0, 3: 1.0 / 90.0}
AX = {"x": 2, "y": 1, "z": 0}


def gd1(g, ax, h):
    a = AX[ax]
    return sum(C1[k] * (np.roll(g, -k, a) - np.roll(g, k, a)) for k in (1, 2, 3)) / h


def gd2(g, ax, h):
    a = AX[ax]
    return (C2[0] * g + sum(C2[k] * (np.roll(g, -k, a) + np.roll(g, k, a)) for k in (1, 2, 3))) / h ** 2


def gko(g, sigma, h):
    w = {0: -20.0, 1: 15.0, 2: -6.0, 3: 1.0}
    tot = 0.0
    for a in (2, 1, 0):
        tot = tot + w[0] * g + sum(w[k] * (np.roll(g, -k, a) + np.roll(g, k, a)) for k in (1, 2, 3))
    return sigma * tot / (64.0 * h)


def uniform_tree(orc, level):
    return orc.Tree.build(level, level, np.zeros((1, 3), np.uint32), np.zeros(1, np.uint32))


def close(a, b, rel, abs_):
    return np.all(np.abs(a - b) <= rel * np.abs(b) + abs_)


# ---------------------------------------------------------------- uniform tree == uniform grid
def test_uniform_unzip_is_periodic_padding(orc):
    t = uniform_tree(orc, 3)
    rng = np.random.default_rng(3)
    g = rng.standard_normal((64, 64, 64))
    z = grid_to_uniform(t.leaves, g)[None]
    p = t.unzip(z)[0]
    gp = np.pad(g, 3, mode="wrap")
    for b in range(t.n):
        _, ix, iy, iz = t.leaves[b].astype(int)
        assert (p[b] == gp[8 * iz:8 * iz + 14, 8 * iy:8 * iy + 14, 8 * ix:8 * ix + 14]).all()
    assert (orc.Tree.zip(p[None])[0] == z[0]).all()          # zip(unzip(u)) == u


def test_uniform_rhs_equals_direct_grid_evaluation(orc):
    t = uniform_tree(orc, 3)
    h = 1.0 / 64
    x, y, zc = coords(t.leaves)
    rng = np.random.default_rng(4)
    u = np.sin(TP * x) * np.sin(TP * y) * np.sin(TP * zc) + 1e-3 * rng.standard_normal(x.shape)
    pi = np.cos(TP * x) + 1e-3 * rng.standard_normal(x.shape)
    g, gp = uniform_to_grid(t.leaves, u), uniform_to_grid(t.leaves, pi)
    lap = gd2(g, "x", h) + gd2(g, "y", h) + gd2(g, "z", h)
    scale = np.abs(lap).max()

    out = t.F(orc.DERIVS, u[None])
    for w, ref in enumerate([gd1(g, "x", h), gd1(g, "y", h), gd1(g, "z", h), lap]):
        assert close(uniform_to_grid(t.leaves, out[w]), ref, 0, 1e-13 * scale)

    sig = 0.4
    out = t.F(orc.WAVE, np.stack([u, pi]), sigma=sig)
    assert close(uniform_to_grid(t.leaves, out[0]), gp + gko(g, sig, h), 0, 1e-13 * scale)
    assert close(uniform_to_grid(t.leaves, out[1]), lap + gko(gp, sig, h), 0, 1e-13 * scale)

    out = t.F(orc.BURGERS, u[None], sigma=sig)
    assert close(uniform_to_grid(t.leaves, out[0]), -g * gd1(g, "x", h) + gko(g, sig, h), 0, 1e-13 * scale)


def test_sixth_order_convergence_on_sine(orc):
    errs = []
    for level in (3, 4):
        t = uniform_tree(orc, level)
        x, y, z = coords(t.leaves)
        u = np.sin(TP * x) * np.sin(TP * y) * np.sin(TP * z)
        out = t.F(orc.DERIVS, u[None])
        ex = TP * np.cos(TP * x) * np.sin(TP * y) * np.sin(TP * z)
        ey = TP * np.sin(TP * x) * np.cos(TP * y) * np.sin(TP * z)
        ez = TP * np.sin(TP * x) * np.sin(TP * y) * np.cos(TP * z)
        el = -3 * TP ** 2 * u
        errs.append([np.abs(out[w] - e).max() for w, e in enumerate([ex, ey, ez, el])])
    order = np.log2(np.array(errs[0]) / np.array(errs[1]))
    assert (order > 5.8).all() and (order < 6.2).all(), order


# ---------------------------------------------------------------- adaptive unzip
def poly5(rng):
    c = rng.integers(-4, 5, size=(6, 6, 6)).astype(float)
    c[(np.add.outer(np.add.outer(np.arange(6), np.arange(6)), np.arange(6))) > 7] = 0.0

    def p(x, y, z):
        out = np.zeros_like(x)
        for a in range(6):
            for b in range(6):
                for d in range(6):
                    if c[a, b, d]:
                        out = out + c[a, b, d] * x ** a * y ** b * z ** d
        return out
    return p


def test_adaptive_unzip_reproduces_polynomial_at_every_ghost(orc):
    t = orc.Tree.build(**sd.tree_params("T4"))
    p = poly5(np.random.default_rng(5))
    x, y, z = coords(t.leaves)
    pad = t.unzip(p(x, y, z)[None])[0]
    ok = away_from_wrap(t.leaves)
    X, Y, Z = padded_coords(t.leaves)
    want = p(X, Y, Z)
    err = np.abs(pad - want)[ok]
    assert err.max() < 1e-12 * np.abs(want).max()
    # the selection covered all three ghost kinds including the half-cell extrapolation row
    g = t.ghost_table()[ok]
    assert {0, 1, 2} <= set(np.unique(g[:, :, 0]).tolist())
    assert (g[:, 12, 0] == orc.G_COARSER).any()              # -x face coarser -> f = 15 occurs


def test_adaptive_unzip_periodic_smooth_field_and_order(orc):
    # ghost values of a periodic smooth field equal the field to interpolation accuracy, also across
    # the periodic wrap; refining every leaf once cuts the worst error by about 2^6
    p = sd.tree_params("T2")

    def worst(tree):
        x, y, z = coords(tree.leaves)
        f = lambda a, b, c: np.sin(TP * a) * np.cos(TP * b) + np.sin(2 * TP * c)
        pad = tree.unzip(f(x, y, z)[None])[0]
        X, Y, Z = padded_coords(tree.leaves)
        return np.abs(pad - f(X, Y, Z)).max()

    t0 = orc.Tree.build(**p)
    lv = t0.leaves.astype(np.int64)
    kids = [(l + 1, 2 * x + (c & 1), 2 * y + ((c >> 1) & 1), 2 * z + ((c >> 2) & 1)) for l, x, y, z in lv.tolist() for c in range(8)]
    t1 = orc.Tree.from_leaves(np.array(kids, dtype=np.uint32))
    e0, e1 = worst(t0), worst(t1)
    assert e0 < 5e-4
    assert 40 < e0 / e1 < 90, (e0, e1)


def test_unzip_copies_and_injections_are_exact(orc):
    t = orc.Tree.build(**sd.tree_params("T4"))
    rng = np.random.default_rng(6)
    u = rng.standard_normal((1, t.n, 8, 8, 8))
    pad = t.unzip(u)[0]
    assert (orc.Tree.zip(pad[None])[0] == u[0]).all()
    g = t.ghost_table()
    lv = t.leaves.astype(np.int64)
    # +x face, same level: ghost columns 11..13 equal neighbour's owned columns 0..2
    hits = 0
    for b in range(t.n):
        if g[b, 14, 0] == orc.G_SAME:
            nb = g[b, 14, 1]
            assert (pad[b, 3:11, 3:11, 11:14] == u[0, nb, :, :, 0:3]).all()
            hits += 1
        if g[b, 14, 0] == orc.G_FINER:
            ids = g[b, 14, 1:5]                               # ascending = (y,z) child order 00,10,01,11
            for q, nb in enumerate(ids):
                cy, cz = q & 1, q >> 1
                want = u[0, nb, ::2, ::2, 0:6:2]
                got = pad[b, 3 + 4 * cz:7 + 4 * cz, 3 + 4 * cy:7 + 4 * cy, 11:14]
                assert (got == want).all()
            hits += 1
    assert hits > 100
    # constant field: every ghost equals the constant exactly (dyadic constant)
    c = np.full((1, t.n, 8, 8, 8), 0.75)
    assert (t.unzip(c) == 0.75).all()


def test_unzip_translation_invariance(orc):
    p = sd.tree_params("T2")
    t0 = orc.Tree.build(**p)
    Q = 1 << 20
    shift = np.array([2, 7, 5], dtype=np.int64)
    pts = (p["pts_q20"].astype(np.int64) + shift * (Q >> 3)) % Q
    t1 = orc.Tree.build(p["lmin"], p["lmax"], pts.astype(np.uint32), p["radius_q20"])
    a = t0.leaves.astype(np.int64)
    moved = a.copy()
    for d in range(3):
        moved[:, 1 + d] = (a[:, 1 + d] + (shift[d] << (a[:, 0] - 3))) % (1 << a[:, 0])
    index1 = {tuple(r): i for i, r in enumerate(t1.leaves.astype(np.int64).tolist())}
    perm = np.array([index1[tuple(r)] for r in moved.tolist()])
    rng = np.random.default_rng(7)
    u0 = rng.standard_normal((1, t0.n, 8, 8, 8))
    u1 = np.empty_like(u0)
    u1[0, perm] = u0[0]
    assert (t1.unzip(u1)[0, perm] == t0.unzip(u0)[0]).all()
    assert (t1.F(orc.DERIVS, u1)[:, perm] == t0.F(orc.DERIVS, u0)).all()


# ---------------------------------------------------------------- linearity, sigma = 0
def test_linearity_and_zero_sigma(orc):
    t = orc.Tree.build(**sd.tree_params("T3"))
    rng = np.random.default_rng(8)
    u = rng.standard_normal((2, t.n, 8, 8, 8))
    f1 = t.F(orc.WAVE, u, sigma=0.5)
    assert (t.F(orc.WAVE, 2.0 * u, sigma=0.5) == 2.0 * f1).all()
    f0 = t.F(orc.WAVE, u, sigma=0.0)
    assert (f0[0] == u[1]).all()                              # KO contributes exactly zero
    d = t.F(orc.DERIVS, u[:1])
    assert (f0[1] == d[3]).all()


# ---------------------------------------------------------------- the 24-field system
def syn24_analytic(coef, x, y, z, h, sigma):
    """Fields u_a = sum_m coef[a][m] * monomial_m; RHS from analytic derivatives.

    monomials: 1, x, y, z, x^2, y^2, z^2, xy, xz, yz, x^2 y, y^2 z, z^2 x, x^6 (the last one only to
    excite the dissipation term: its sixth difference is 720 h^6).
    """
    one, zero = np.ones_like(x), np.zeros_like(x)
    mon = [one, x, y, z, x * x, y * y, z * z, x * y, x * z, y * z, x * x * y, y * y * z, z * z * x, x ** 6]
    dx = [zero, one, zero, zero, 2 * x, zero, zero, y, z, zero, 2 * x * y, zero, z * z, 6 * x ** 5]
    dy = [zero, zero, one, zero, zero, 2 * y, zero, x, zero, z, x * x, 2 * y * z, zero, zero]
    dz = [zero, zero, zero, one, zero, zero, 2 * z, zero, x, y, zero, y * y, 2 * z * x, zero]
    dxx = [zero] * 4 + [2 * one, zero, zero, zero, zero, zero, 2 * y, zero, zero, 30 * x ** 4]
    dyy = [zero] * 4 + [zero, 2 * one, zero, zero, zero, zero, zero, 2 * z, zero, zero]
    dzz = [zero] * 4 + [zero, zero, 2 * one, zero, zero, zero, zero, zero, 2 * x, zero]
    dxy = [zero] * 7 + [one, zero, zero, 2 * x, zero, zero, zero]
    dxz = [zero] * 7 + [zero, one, zero, zero, zero, 2 * z, zero]
    dyz = [zero] * 7 + [zero, zero, one, zero, 2 * y, zero, zero]

    def comb(tab, a):
        return sum(coef[a][m] * tab[m] for m in range(14))

    U = [comb(mon, a) for a in range(24)]
    D = [[comb(dx, a), comb(dy, a), comb(dz, a)] for a in range(24)]
    alpha, beta = U[0], U[1:4]
    gxx, gxy, gxz, gyy, gyz, gzz = U[4:10]
    Gxx, Gyy, Gzz = 1 - gxx / 8, 1 - gyy / 8, 1 - gzz / 8
    Gxy, Gxz, Gyz = -gxy / 8, -gxz / 8, -gyz / 8
    lap = []
    for s in range(10):
        lap.append(Gxx * comb(dxx, s) + Gyy * comb(dyy, s) + Gzz * comb(dzz, s)
                   + 2 * (Gxy * comb(dxy, s) + Gxz * comb(dxz, s) + Gyz * comb(dyz, s)))
    rhs = []
    for a in range(24):
        adv = sum(beta[d] * D[a][d] for d in range(3))
        cross = sum(D[a][d] * D[(a + 1) % 24][d] for d in range(3))
        ko = sigma * coef[a][13] * 720.0 * h ** 6 / (64.0 * h)
        rhs.append(adv + 2.0 ** -(a % 4) * lap[a % 10] + 0.25 * cross - 0.5 * alpha * U[(a + 11) % 24] + ko)
    return np.stack(U), np.stack(rhs)


def test_syn24_equals_analytic_evaluation_on_polynomials(orc):
    t = uniform_tree(orc, 3)
    h = 1.0 / 64
    rng = np.random.default_rng(9)
    coef = rng.integers(-3, 4, size=(24, 14)).astype(float)
    x, y, z = coords(t.leaves)
    U, want = syn24_analytic(coef, x, y, z, h, 0.4)
    got = t.F(orc.SYN24, U, sigma=0.4)
    ok = away_from_wrap(t.leaves)
    assert ok.sum() == 216
    scale = np.abs(want[:, ok]).max()
    assert np.abs(got[:, ok] - want[:, ok]).max() < 1e-9 * scale
    # every term matters at this tolerance: a perturbed coefficient table must fail
    coef2 = coef.copy()
    coef2[11, 2] += 1.0
    _, other = syn24_analytic(coef2, x, y, z, h, 0.4)
    assert np.abs(got[:, ok] - other[:, ok]).max() > 1e-3 * scale


def test_syn24_on_adaptive_tree_matches_analytic_polynomials(orc):
    t = orc.Tree.build(**sd.tree_params("T4"))
    rng = np.random.default_rng(10)
    coef = rng.integers(-3, 4, size=(24, 14)).astype(float)
    coef[:, 13] = 0.0                                         # degree <= 3: interpolation is exact too
    x, y, z = coords(t.leaves)
    U, want = syn24_analytic(coef, x, y, z, 1.0, 0.4)
    ok = np.flatnonzero(away_from_wrap(t.leaves))
    got = t.F(orc.SYN24, U, sigma=0.4, blocks=ok)
    scale = np.abs(want[:, ok]).max()
    assert np.abs(got - want[:, ok]).max() < 1e-8 * scale


def test_syn24_reduces_to_scalar_operators(orc):
    # g = 0, beta = 0, alpha = 0 and all other fields equal to zero except one field s < 10:
    # RHS_a = kappa_a * Laplacian(u_s) + KO(u_a) for a = s, s+10, s+20
    t = orc.Tree.build(**sd.tree_params("T4"))
    rng = np.random.default_rng(11)
    blocks = np.arange(0, t.n, 7)
    for s in (0, 3):
        U = np.zeros((24, t.n, 8, 8, 8))
        U[s + 10] = rng.standard_normal((t.n, 8, 8, 8))       # field s+10 has a<10 false: no coupling to G
        f = t.F(orc.SYN24, U, sigma=0.4, blocks=blocks)
        w = t.F(orc.WAVE, np.stack([U[s + 10], U[s + 10]]), sigma=0.4, blocks=blocks)
        ko = w[0] - U[s + 10][blocks]                          # pi + KO(u) - pi: KO up to one rounding
        assert np.abs(f[s + 10] - ko).max() <= 1e-12 * np.abs(ko).max()
        others = [a for a in range(24) if a != s + 10]
        assert (f[others] == 0.0).all()
    # a field with second derivatives: u_2 only (beta^y). alpha = 0, g = 0 -> G = identity
    U = np.zeros((24, t.n, 8, 8, 8))
    U[0] = rng.standard_normal((t.n, 8, 8, 8))                # alpha only
    f = t.F(orc.SYN24, U, sigma=0.0, blocks=blocks)
    lap = t.F(orc.DERIVS, U[:1], blocks=blocks)[3]
    # RHS_0 = lap(alpha) - 0.5*alpha*u_11 (=0) ; RHS_10 = kappa_10 * lap = 2^-2 lap ; RHS_20 = lap
    tol = 1e-12 * np.abs(lap).max()
    assert np.abs(f[0] - lap).max() <= tol
    assert np.abs(f[10] - 0.25 * lap).max() <= tol
    assert np.abs(f[20] - lap).max() <= tol
    # RHS_13 = -0.5 * alpha * u_0 = -0.5 alpha^2   (a + 11 = 24 -> field 0)
    assert np.abs(f[13] + 0.5 * U[0][blocks] ** 2).max() <= 1e-15 * 10


# ---------------------------------------------------------------- time stepping
def burgers_exact(x, t, c):
    """u = u0(x - u t) by Newton iteration, valid before the shock time 1/(pi c)."""
    u0 = lambda s: 0.5 * (1 - np.cos(TP * c * s))
    du0 = lambda s: 0.5 * TP * c * np.sin(TP * c * s)
    u = u0(x)
    for _ in range(60):
        r = u - u0(x - u * t)
        u = u - r / (1 + t * du0(x - u * t))
    return u


def test_burgers_step_tracks_characteristics(orc):
    # the paper's equation and initial data (its introduction), c = 1 so that 64 points resolve it
    t = uniform_tree(orc, 3)
    x, _, _ = coords(t.leaves)
    u0 = 0.5 * (1 - np.cos(TP * x))
    dt = 2.0 ** -8
    u1 = t.rk4_step(orc.BURGERS, u0[None], dt, sigma=0.0)[0]
    err = np.abs(u1 - burgers_exact(x, dt, 1.0)).max()
    assert err < 2e-8                                        # O(dt h^6) + O(dt^5)
    assert np.abs(u1 - u0).max() > 1e-3                      # and the step did move the solution
    # a flux of the wrong sign would follow the time-reversed solution instead
    assert np.abs(u1 - burgers_exact(x, -dt, 1.0)).max() > 1e4 * err


def test_rk4_is_fourth_order(orc):
    # step-doubling differences of the semi-discrete Burgers system shrink by 2^5 per halving
    t = uniform_tree(orc, 3)
    x, _, _ = coords(t.leaves)
    u0 = 0.5 * (1 - np.cos(TP * x))[None]
    diffs = []
    for dt in (2.0 ** -5, 2.0 ** -6, 2.0 ** -7):
        one = t.rk4_step(orc.BURGERS, u0, dt)
        two = t.rk4_step(orc.BURGERS, t.rk4_step(orc.BURGERS, u0, dt / 2), dt / 2)
        diffs.append(np.abs(one - two).max())
    r = np.log2(np.array(diffs[:-1]) / np.array(diffs[1:]))
    assert (r > 4.7).all() and (r < 5.3).all(), (diffs, r)


def test_wave_step_tracks_plane_wave(orc):
    t = uniform_tree(orc, 3)
    x, _, _ = coords(t.leaves)
    u = lambda s: np.sin(TP * (x - s))
    pi = lambda s: -TP * np.cos(TP * (x - s))
    dt = 2.0 ** -8
    out = t.rk4_step(orc.WAVE, np.stack([u(0.0), pi(0.0)]), dt, sigma=0.0)
    assert np.abs(out[0] - u(dt)).max() < 1e-9
    assert np.abs(out[1] - pi(dt)).max() < 1e-8
    assert np.abs(out[0] - u(0.0)).max() > 1e-3


def test_rk4_leaves_a_stationary_state_alone(orc):
    t = orc.Tree.build(**sd.tree_params("T3"))
    u = np.stack([np.full((t.n, 8, 8, 8), 0.625), np.zeros((t.n, 8, 8, 8))])
    assert (t.rk4_step(orc.WAVE, u, 2.0 ** -10, sigma=0.4) == u).all()


def test_rk4_equals_stage_by_stage_composition(orc):
    # classical tableau written out with F as a black box
    t = orc.Tree.build(**sd.tree_params("T3"))
    u = sd.make_fields("T3", t.leaves).numpy()
    u[1] = 0.1 * np.random.default_rng(12).standard_normal(u[1].shape)
    dt, sg = sd.time_step(5), 0.4
    F = lambda v: t.F(orc.WAVE, v, sigma=sg)
    k1 = F(u)
    k2 = F(u + dt / 2 * k1)
    k3 = F(u + dt / 2 * k2)
    k4 = F(u + dt * k3)
    want = u + dt / 6 * (k1 + 2 * k2 + 2 * k3 + k4)
    got = t.rk4_step(orc.WAVE, u, dt, sigma=sg)
    assert np.abs(got - want).max() <= 4e-16 * np.abs(want).max()
