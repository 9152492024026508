"""Pins of the oracle's inter-grid transfer (no GPU): identity, samples of one function on two trees
(bit-exact where the new point is an old node, to rounding where a polynomial of degree 5 is
interpolated), exact rational Lagrange interpolation written out independently, sixth-order
convergence on a smooth function, and the refusal of a two-level refinement."""
from fractions import Fraction

import numpy as np
import pytest

import synthdata as sd
from helpers import coords


def orbit_pair(orc, name, phase):
    a = orc.Tree.build(**sd.tree_params(name, 1))
    b = orc.Tree.build(**sd.tree_params(name, 1, phase=phase))
    return a, b


def uniform_tree(orc, level):
    return orc.Tree.build(level, level, np.zeros((1, 3), np.uint32), np.zeros(1, np.uint32))


def relation(src, dst):
    """per target leaf: level of the source leaf that contains its first point, minus its own level;
    brute force over all source leaves (independent of the oracle's point location)."""
    s = src.leaves.astype(np.int64)
    out = np.empty(dst.n, dtype=np.int64)
    for b, (l, ix, iy, iz) in enumerate(dst.leaves.astype(np.int64)):
        down = np.maximum(l - s[:, 0], 0)        # source coarser: express the target anchor at its level
        up = np.maximum(s[:, 0] - l, 0)          # source finer: it must sit exactly at the anchor corner
        hit = (((ix >> down) << up) == s[:, 1]) & (((iy >> down) << up) == s[:, 2]) & (((iz >> down) << up) == s[:, 3])
        cand = np.nonzero(hit)[0]
        assert cand.size == 1                    # the leaves tile the cube
        out[b] = s[cand[0], 0] - l
    return out


def poly5(x, y, z):
    return (1.0 + x - 2.0 * x ** 3 + 0.5 * x ** 5) * (2.0 - y ** 2 + y ** 5) * (1.0 + 3.0 * z ** 4 - z ** 5) + x * y * z


def test_identity_is_bit_exact(orc):
    a, _ = orbit_pair(orc, "T4", 0.0)
    u = np.random.default_rng(0).standard_normal((3, a.n, 8, 8, 8))
    assert (orc.transfer(a, a, u) == u).all()


def test_moved_tree_has_all_three_cases_and_samples_a_polynomial(orc):
    a, b = orbit_pair(orc, "T4", 0.35)
    rel = relation(a, b)
    assert (rel == 0).any() and (rel == -1).any() and (rel >= 1).any() and rel.min() == -1
    xa, ya, za = coords(a.leaves)
    xb, yb, zb = coords(b.leaves)
    got = orc.transfer(a, b, poly5(xa, ya, za)[None])[0]
    want = poly5(xb, yb, zb)
    same = rel >= 0                                  # every point of these leaves is a source node
    assert (got[same] == want[same]).all()
    # degree <= 5 per axis is reproduced by the six-point interpolant up to rounding; the weights'
    # absolute sums are at most 18.25 per axis
    err = np.abs(got[~same] - want[~same])
    assert err.max() < 2e-11 and err.max() > 0.0
    # in an interpolated leaf the points with three even fine coordinates are source nodes again
    lv = b.leaves.astype(np.int64)
    for blk in np.nonzero(~same)[0][:50]:
        o = (8 * lv[blk, 1:4]) % 16                   # fine coordinate of the leaf's first point: 0 or 8
        assert (o % 8 == 0).all()
        assert (got[blk][::2, ::2, ::2] == want[blk][::2, ::2, ::2]).all()


def lagrange_exact(nodes, values, x):
    tot = Fraction(0)
    for m, xm in enumerate(nodes):
        w = Fraction(1)
        for n, xn in enumerate(nodes):
            if n != m:
                w *= Fraction(x - xn) / Fraction(xm - xn)
        tot += w * values[m]
    return tot


def test_interpolated_points_equal_exact_rational_lagrange(orc):
    a = uniform_tree(orc, 3)
    b = orc.Tree.build(3, 4, np.array([[1 << 19] * 3], np.uint32), np.array([40000], np.uint32))
    assert b.n > a.n
    rng = np.random.default_rng(5)
    u = rng.integers(-1000, 1000, size=(1, a.n, 8, 8, 8)).astype(np.float64)
    got = orc.transfer(a, b, u)[0]
    la = {tuple(r[1:]): i for i, r in enumerate(a.leaves.astype(int))}
    fine = np.nonzero(b.leaves[:, 0] == 4)[0]
    checked = 0
    for blk in fine[:: max(1, fine.size // 12)]:
        _, ix, iy, iz = b.leaves[blk].astype(int)
        src = u[0, la[(ix // 2, iy // 2, iz // 2)]]
        for (k, j, i) in [(0, 0, 0), (1, 0, 0), (0, 1, 0), (0, 0, 1), (7, 7, 7), (1, 1, 1), (3, 5, 7), (7, 2, 1), (5, 5, 5)]:
            f = [8 * (ix % 2) + i, 8 * (iy % 2) + j, 8 * (iz % 2) + k]   # fine coordinate inside the coarse leaf

            def line(vals, fa):
                if fa % 2 == 0:
                    return vals[fa // 2]
                s = min(max((fa - 1) // 2 - 2, 0), 2)
                return lagrange_exact(list(range(s, s + 6)), vals[s:s + 6], Fraction(fa, 2))

            plane = [[line([Fraction(int(src[cz, cy, cx])) for cx in range(8)], f[0]) for cy in range(8)] for cz in range(8)]
            col = [line(plane[cz], f[1]) for cz in range(8)]
            exact = line(col, f[2])
            assert abs(got[blk, k, j, i] - float(exact)) <= 1e-12 * max(1.0, abs(float(exact))) * 50
            checked += 1
    assert checked >= 100


def test_injection_takes_the_coinciding_node(orc):
    # coarsening by one, two and four levels: every new point is an old node
    fine = orc.Tree.build(3, 7, np.array([[300000, 500000, 700000]], np.uint32), np.array([30000] * 4, np.uint32))
    assert fine.leaves[:, 0].max() == 7
    coarse = uniform_tree(orc, 3)
    xf, yf, zf = coords(fine.leaves)
    xc, yc, zc = coords(coarse.leaves)
    f = lambda x, y, z: np.sin(3.0 * x) + np.cos(5.0 * y) * z + x * y
    got = orc.transfer(fine, coarse, f(xf, yf, zf)[None])[0]
    assert (got == f(xc, yc, zc)).all()
    with pytest.raises(ValueError):
        orc.transfer(coarse, fine, f(xc, yc, zc)[None])      # four levels finer: refused


def test_refinement_by_exactly_two_levels_is_refused_and_by_one_is_not(orc):
    # the boundary of the rule: level 3 -> level 5 somewhere is refused, level 3 -> level 4 is served
    coarse = uniform_tree(orc, 3)
    u = np.zeros((1, coarse.n, 8, 8, 8))
    with pytest.raises(ValueError):
        orc.transfer(coarse, uniform_tree(orc, 5), u)
    two = orc.Tree.build(3, 5, np.array([[300000, 500000, 700000]], np.uint32), np.array([30000, 30000], np.uint32))
    assert two.leaves[:, 0].max() == 5 and two.leaves[:, 0].min() == 3
    with pytest.raises(ValueError):
        orc.transfer(coarse, two, u)
    assert orc.transfer(coarse, uniform_tree(orc, 4), u).shape == (1, 4096, 8, 8, 8)


def test_prolongation_converges_at_sixth_order(orc):
    errs = []
    for l in (3, 4):
        a = uniform_tree(orc, l)
        b = uniform_tree(orc, l + 1)
        xa, ya, za = coords(a.leaves)
        xb, yb, zb = coords(b.leaves)
        f = lambda x, y, z: np.sin(2 * np.pi * x) * np.cos(2 * np.pi * y) + np.sin(4 * np.pi * z)
        got = orc.transfer(a, b, f(xa, ya, za)[None])[0]
        errs.append(np.abs(got - f(xb, yb, zb)).max())
    assert 40.0 < errs[0] / errs[1] < 90.0            # 2^6 = 64
