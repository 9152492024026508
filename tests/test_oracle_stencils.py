"""Pins of the oracle's 1-D operators against mathematics (no GPU).

The source paper gives no stencil coefficients (its forward model uses 3x3 Sobel/Laplacian kernels
and only suggests higher-order stencils), so these are pinned by what defines them: exactness on
polynomials, the leading error term, and exact rational recomputation of the Lagrange weights.
"""
from fractions import Fraction
from math import factorial

import numpy as np
import pytest


def line(f, x0, h):
    return np.array([f(x0 + k * h) for k in range(-3, 4)])


def test_scale_constants_are_correctly_rounded():
    assert float.fromhex("0x1.1111111111111p-6") == 1.0 / 60.0
    assert float.fromhex("0x1.6c16c16c16c17p-8") == 1.0 / 180.0


@pytest.mark.parametrize("n", range(0, 8))
def test_d1_d2_exact_on_monomials(orc, n):
    # small integer abscissae so that the monomials are exact in fp64
    h, x0 = 0.5, 1.5
    u = line(lambda x: x ** n, x0, h)
    d1 = orc.d1_line(u, 1.0 / h)
    d2 = orc.d2_line(u, 1.0 / h ** 2)
    if n <= 6:
        assert d1 == pytest.approx(n * x0 ** (n - 1) if n else 0.0, rel=1e-13, abs=1e-12)
    assert d2 == pytest.approx(n * (n - 1) * x0 ** (n - 2) if n > 1 else 0.0, rel=1e-13, abs=1e-11)


def test_d1_leading_error_term(orc):
    # centred D1 errors alternate in sign with the order (+h^2/6 f''', -h^4/30 f^(5), +h^6/140 f^(7));
    # for x^7 at 0 the 6th-order operator therefore returns +36 h^6
    h, x0 = 0.5, 0.0
    u = line(lambda x: x ** 7, x0, h)
    assert orc.d1_line(u, 1.0 / h) == pytest.approx(factorial(7) / 140.0 * h ** 6, rel=1e-12)


def test_d2_leading_error_term(orc):
    # centred D2 errors: +h^2/12 f^(4), -h^4/90 f^(6), +h^6/560 f^(8); for x^8 at 0: +72 h^6
    h = 0.5
    u = line(lambda x: x ** 8, 0.0, h)
    assert orc.d2_line(u, 1.0 / h ** 2) == pytest.approx(factorial(8) / 560.0 * h ** 6, rel=1e-12)


@pytest.mark.parametrize("n", range(0, 7))
def test_ko_is_sixth_difference(orc, n):
    h, x0 = 0.5, 1.0
    q = orc.ko_line(line(lambda x: x ** n, x0, h))
    want = 0.0 if n <= 5 else 720.0 * h ** 6
    assert q == pytest.approx(want, abs=1e-9)


def test_ko_sign_is_dissipative(orc):
    # on the highest grid mode (+1,-1,...) the operator must have the sign opposite to u
    u = np.array([1.0, -1, 1, -1, 1, -1, 1])  # centre value -1
    assert orc.ko_line(u) == 64.0  # -> +64 at a point where u = -1: damps the mode


def lagrange_row(r):
    """exact weights of the 6-point interpolant on nodes 0..5 at abscissa r"""
    w = []
    for j in range(6):
        num, den = Fraction(1), Fraction(1)
        for m in range(6):
            if m != j:
                num *= (r - m)
                den *= (j - m)
        w.append(num / den)
    return w


def expected_row(f):
    """odd fine coordinate f -> (first node, exact weights) under the clamped-stencil rule"""
    c0 = (f - 1) // 2
    s = min(max(c0 - 2, 0), 2)
    return s, lagrange_row(Fraction(f, 2) - s)


@pytest.mark.parametrize("f", range(1, 16, 2))
def test_interp_weights_match_exact_rationals(orc, f):
    s, w = expected_row(f)
    assert sum(w) == 1
    assert all((x * 256).denominator == 1 for x in w)  # dyadic with denominator 256
    # probe the oracle with unit impulses along x, y and z separately
    for axis in range(3):
        for node in range(8):
            src = np.zeros((8, 8, 8))
            idx = [2, 4, 6]            # even fine coords 4, 8, 12 on the other axes -> pass through
            idx[axis] = node
            src[idx[2], idx[1], idx[0]] = 1.0
            fc = [4, 8, 12]
            fc[axis] = f
            got = orc.interp(src, *fc)
            want = float(w[node - s]) if s <= node < s + 6 else 0.0
            assert got == want, (axis, node, f)


def test_interp_rows_are_mirror_images():
    for k in range(5):
        a = lagrange_row(Fraction(2 * k + 1, 2))
        b = lagrange_row(Fraction(2 * (4 - k) + 1, 2))
        assert a == b[::-1]


def test_interp_even_coordinates_pass_through(orc):
    rng = np.random.default_rng(0)
    src = rng.standard_normal((8, 8, 8))
    for fx, fy, fz in [(0, 2, 4), (14, 0, 6), (8, 8, 8)]:
        assert orc.interp(src, fx, fy, fz) == src[fz // 2, fy // 2, fx // 2]


def test_interp_reproduces_tensor_polynomials_degree5(orc):
    rng = np.random.default_rng(1)
    c = rng.integers(-3, 4, size=(6, 6, 6)).astype(float)
    X = np.arange(8.0)

    def p(x, y, z):
        return sum(c[a, b, d] * x ** a * y ** b * z ** d for a in range(6) for b in range(6) for d in range(6))

    src = np.array([[[p(x / 8, y / 8, z / 8) for x in X] for y in X] for z in X])
    scale = np.abs(src).max()
    for fx in range(16):
        for fy in (1, 6, 15):
            for fz in (0, 7, 13):
                got = orc.interp(src, fx, fy, fz)
                assert abs(got - p(fx / 16, fy / 16, fz / 16)) < 2e-12 * scale


def test_interp_remainder_on_x6(orc):
    # textbook remainder: f(r) - p(r) = prod(r - j)/720 * f^(6) for nodes j = 0..5 (node spacing 1)
    X = np.arange(8.0)
    src = np.broadcast_to(X ** 6, (8, 8, 8)).copy()
    for f in range(1, 16, 2):
        s, _ = expected_row(f)
        r = f / 2.0 - s
        rem = np.prod([r - j for j in range(6)])  # * 720/720
        got = orc.interp(src, f, 0, 0)
        assert (f / 2.0) ** 6 - got == pytest.approx(rem, rel=1e-9)


def test_interp_order_is_x_then_y_then_z(orc):
    # the three 1-D passes do not commute in floating point; pin the order by emulating it
    rng = np.random.default_rng(2)
    src = rng.standard_normal((8, 8, 8))

    def row(f):
        s, w = expected_row(f)
        return s, [float(x) for x in w]

    import math

    def chain(w, v):
        acc = w[0] * v[0]
        for m in range(1, 6):
            acc = math.fma(w[m], v[m], acc) if hasattr(math, "fma") else None
        return acc

    if not hasattr(math, "fma"):
        # emulate fma exactly with rationals
        def chain(w, v):  # noqa: F811
            acc = w[0] * v[0]
            for m in range(1, 6):
                acc = float(Fraction(w[m]) * Fraction(v[m]) + Fraction(acc))
            return acc

    fx, fy, fz = 5, 15, 1
    sx, wx = row(fx)
    sy, wy = row(fy)
    sz, wz = row(fz)
    vx = np.array([[chain(wx, src[cz, cy, sx:sx + 6]) for cy in range(8)] for cz in range(8)])
    vy = np.array([chain(wy, vx[cz, sy:sy + 6]) for cz in range(8)])
    want = chain(wz, vy[sz:sz + 6])
    assert orc.interp(src, fx, fy, fz) == want
