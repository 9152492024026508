"""Mutation check of the oracle's pins (CPU only; run as `python tests/oracle_mutants.py [name ...]`).

One plausible mistake at a time (a wrong sign, index, coefficient, transposed operand, dropped
periodic image ...) is planted in a COPY of oracle/octfd_oracle.c inside a temporary copy of the
oracle, its pin tests and the input generators; the copy's pin tests must then fail.  The tree
itself is never modified and nothing here touches a GPU.  A mistake that only changes the order of
floating-point rounding is not on the list: no closed form can see it, the element-by-element
comparison of the two independent implementations does.

Last full run: every mutant below was killed; the test named in the log is the first that failed.
tests/test_oracle_mutants.py runs a few quick ones with every CPU test run.
"""
import os
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_TESTS = ["tests/test_oracle_tree.py", "tests/test_oracle_stencils.py", "tests/test_oracle_pipeline.py",
             "tests/test_oracle_transfer.py", "tests/test_oracle_centred.py"]

# (name, text in oracle/octfd_oracle.c, replacement, which occurrence)
MUTANTS = [
 ("refine strict<", "if (d2 < R * R) return 1;", "if (d2 <= R * R) return 1;", 1),
 ("no periodic images", "for (int im = -1; im <= 1; im++) {", "for (int im = 0; im <= 0; im++) {", 1),
 ("open box", "axis_gap(pts[3 * p + d], a[d] * s, (a[d] + 1) * s)", "axis_gap(pts[3 * p + d], a[d] * s, (a[d] + 1) * s - 1)", 1),
 ("balance skips corners", "if (!dx && !dy && !dz) continue;", "if (!dx && !dy && !dz) continue; if (dx && dy && dz) continue;", 1),
 ("balance skips edges+corners", "if (!dx && !dy && !dz) continue;", "if (!dx && !dy && !dz) continue; if ((dx != 0) + (dy != 0) + (dz != 0) > 1) continue;", 1),
 ("balance allows 2 levels", "t->leaves[c].level + 1 >= o.level", "t->leaves[c].level + 2 >= o.level", 1),
 ("balance not periodic", "uint32_t nx = (o.ix + (uint32_t)dx) & m, ny = (o.iy + (uint32_t)dy) & m, nz = (o.iz + (uint32_t)dz) & m;",
  "uint32_t nx = (o.ix + (uint32_t)dx) & m, ny = (o.iy + (uint32_t)dy) & m, nz = (o.iz + (uint32_t)dz) & m; if (nx != o.ix + (uint32_t)dx || ny != o.iy + (uint32_t)dy || nz != o.iz + (uint32_t)dz) continue;", 1),
 ("morton y/z swapped", "((y >> b) & 1) << (3 * b + 1) | ((z >> b) & 1) << (3 * b + 2)", "((y >> b) & 1) << (3 * b + 2) | ((z >> b) & 1) << (3 * b + 1)", 1),
 ("lagrange sign", "{   3.0,  -25.0,  150.0,  150.0,   -25.0,   3.0 },", "{   3.0,  -25.0,  150.0,  150.0,   -25.0,  -3.0 },", 1),
 ("lagrange row0 entry", "{  63.0,  315.0, -210.0,  126.0,   -45.0,   7.0 },", "{  63.0,  315.0, -210.0,  126.0,   -45.0,   5.0 },", 1),
 ("lagrange last row", "{ -63.0,  385.0, -990.0, 1386.0, -1155.0, 693.0 },", "{ -63.0,  385.0, -990.0, 1386.0, -1155.0, 695.0 },", 1),
 ("stencil clamp", "if (st > 2) st = 2;", "if (st > 1) st = 1;", 1),
 ("stencil not clamped low", "if (st < 0) st = 0;", "if (st < 1) st = 1;", 1),
 ("interp y/z transposed", "return src[(cz * NPT + cy) * NPT + fx / 2];", "return src[(cy * NPT + cz) * NPT + fx / 2];", 1),
 ("injection offset", "q[d] = (int)(2 * P[d] - NPT * sa[d]);\n                    val = src", "q[d] = (int)(2 * P[d] - NPT * sa[d]) ^ 1;\n                    val = src", 1),
 ("unzip shifted", "P[d] = ((NPT * a[d] + pp[d] - PAD) % N + N) % N;\n            int64_t L = locate(t, l, P);\n            orc_leaf S", "P[d] = ((NPT * a[d] + pp[d] - PAD + 1) % N + N) % N;\n            int64_t L = locate(t, l, P);\n            orc_leaf S", 1),
 ("coarse f offset", "f[d] = (int)(P[d] - 2 * NPT * sa[d]);\n                    val = interp_xyz(src, f[0], f[1], f[2]);\n                } else {\n                    val = NAN;  /*", "f[d] = (int)(P[d] - 2 * NPT * sa[d]) ^ 1;\n                    val = interp_xyz(src, f[0], f[1], f[2]);\n                } else {\n                    val = NAN;  /*", 1),
 ("d1 sign", "double t = fma(-9.0, d2, d3);", "double t = fma(9.0, d2, d3);", 1),
 ("d1 coeff", "t = fma(45.0, d1, t);", "t = fma(46.0, d1, t);", 1),
 ("d1 reversed", "double d1 = p1 - m1, d2 = p2 - m2, d3 = p3 - m3;", "double d1 = m1 - p1, d2 = m2 - p2, d3 = m3 - p3;", 1),
 ("d2 centre", "t = fma(-490.0, u0, t);", "t = fma(-489.0, u0, t);", 1),
 ("d2 outer", "double t = 2.0 * s3;", "double t = 3.0 * s3;", 1),
 ("d2 scale", "return (t * C180) * ih2;", "return (t * C60) * ih2;", 1),
 ("ko sign", "double q = fma(-6.0, s2, s3);", "double q = fma(6.0, s2, s3);", 1),
 ("ko centre", "q = fma(-20.0, u0, q);", "q = fma(-19.0, u0, q);", 1),
 ("ko scale", "(ih * 0.015625)", "(ih * 0.03125)", 1),
 ("ko overall sign", "return sigma * (((q[0] + q[1]) + q[2])", "return -sigma * (((q[0] + q[1]) + q[2])", 1),
 ("lap misses z", "return (D2(U, c, 0, ih2) + D2(U, c, 1, ih2)) + D2(U, c, 2, ih2);", "return (D2(U, c, 0, ih2) + D2(U, c, 1, ih2)) + D2(U, c, 1, ih2);", 1),
 ("stride y/z swapped", "static const int STRIDE[3] = { 1, NP, NP * NP };", "static const int STRIDE[3] = { 1, NP * NP, NP };", 1),
 ("dmix inner = outer", "return d1_taps(D1(U, c - 3 * s, b, ih), D1(U, c - 2 * s, b, ih), D1(U, c - s, b, ih),\n                   D1(U, c + s, b, ih), D1(U, c + 2 * s, b, ih), D1(U, c + 3 * s, b, ih), ih);",
  "return d1_taps(D1(U, c - 3 * s, a, ih), D1(U, c - 2 * s, a, ih), D1(U, c - s, a, ih),\n                   D1(U, c + s, a, ih), D1(U, c + 2 * s, a, ih), D1(U, c + 3 * s, a, ih), ih);", 1),
 ("wave ko sign", "O[0][c] = I[1][c] + KO(I[0], c, sigma, ih);", "O[0][c] = I[1][c] - KO(I[0], c, sigma, ih);", 1),
 ("wave lap of pi", "O[1][c] = LAP(I[0], c, ih2) + KO(I[1], c, sigma, ih);", "O[1][c] = LAP(I[1], c, ih2) + KO(I[1], c, sigma, ih);", 1),
 ("burgers flux sign", "O[0][c] = KO(I[0], c, sigma, ih) - flux;", "O[0][c] = KO(I[0], c, sigma, ih) + flux;", 1),
 ("burgers axis", "double flux = I[0][c] * D1(I[0], c, 0, ih);", "double flux = I[0][c] * D1(I[0], c, 1, ih);", 1),
 ("derivs order", "O[0][c] = D1(I[0], c, 0, ih); O[1][c] = D1(I[0], c, 1, ih);", "O[0][c] = D1(I[0], c, 1, ih); O[1][c] = D1(I[0], c, 0, ih);", 1),
 ("syn successor", "int n = (a + 1) % 24, m = (a + 11) % 24;", "int n = (a + 2) % 24, m = (a + 11) % 24;", 1),
 ("syn a+11", "int n = (a + 1) % 24, m = (a + 11) % 24;", "int n = (a + 1) % 24, m = (a + 12) % 24;", 1),
 ("syn kappa", "double kappa = ldexp(1.0, -(a % 4));", "double kappa = ldexp(1.0, -(a % 3));", 1),
 ("syn lap index", "double t2 = kappa * lap[a % 10];", "double t2 = kappa * lap[a % 9];", 1),
 ("syn off factor", "lap[s] = fma(2.0, off, diag);", "lap[s] = fma(1.0, off, diag);", 1),
 ("syn Gxy sign", "Gxy = -(eps * in[5][c])", "Gxy = (eps * in[5][c])", 1),
 ("syn Gyy field", "double Gyy = 1.0 - eps * in[7][c]", "double Gyy = 1.0 - eps * in[8][c]", 1),
 ("syn t3 factor", "t3 = 0.25 * t3;", "t3 = 0.5 * t3;", 1),
 ("syn t4 sign", "out[a][c] = (((t1 + t2) + t3) - t4) + ko[a];", "out[a][c] = (((t1 + t2) + t3) + t4) + ko[a];", 1),
 ("syn eps", "const double eps = 0.125;", "const double eps = 0.25;", 1),
 ("syn dxz axes", "dxz = DMIX(U, c, 0, 2, ih)", "dxz = DMIX(U, c, 0, 1, ih)", 1),
 ("syn beta order", "double t1 = bx * d[a][0]; t1 = fma(by, d[a][1], t1); t1 = fma(bz, d[a][2], t1);", "double t1 = bx * d[a][0]; t1 = fma(bz, d[a][1], t1); t1 = fma(by, d[a][2], t1);", 1),
 ("syn half alpha", "double t4 = (0.5 * alpha) * in[m][c];", "double t4 = (1.0 * alpha) * in[m][c];", 1),
 ("rk4 weight k2", "acc[i] = acc[i] + 2.0 * k[i]; st[i] = fma(half, k[i], u[i]); }", "acc[i] = acc[i] + 1.0 * k[i]; st[i] = fma(half, k[i], u[i]); }", 1),
 ("rk4 stage 4 step", "st[i] = fma(dt, k[i], u[i]); }", "st[i] = fma(half, k[i], u[i]); }", 1),
 ("rk4 sixth", "const double half = 0.5 * dt, sixth = dt / 6.0;", "const double half = 0.5 * dt, sixth = dt / 8.0;", 1),
 ("rk4 stage from stage", "acc[i] = acc[i] + 2.0 * k[i]; st[i] = fma(half, k[i], u[i]); }", "acc[i] = acc[i] + 2.0 * k[i]; st[i] = fma(half, k[i], st[i]); }", 1),
 ("transfer injection offset", "q[d] = (int)((P[d] << dl) - NPT * sa[d]);", "q[d] = (int)((P[d] << dl) - NPT * sa[d]) ^ (dl > 0);", 1),
 ("transfer axes swapped", "val = interp_xyz(src, f[0], f[1], f[2]);\n                }\n                zipped_dst", "val = interp_xyz(src, f[1], f[0], f[2]);\n                }\n                zipped_dst", 1),
 ("transfer refusal", "(int)S->leaves[L].level < (int)B.level - 1) return -8;", "(int)S->leaves[L].level < (int)B.level - 2) return -8;", 1),
 ("centred window", "for (int m = 0; m < 6; m++) v[m] = row[c0 - 2 + m];", "for (int m = 0; m < 6; m++) v[m] = row[c0 - 1 + m];", 1),
 ("centred weights row", "double acc = (LAG256[2][0] / 256.0) * v[0];\n    for (int m = 1; m < 6; m++) acc = fma(LAG256[2][m] / 256.0, v[m], acc);", "double acc = (LAG256[1][0] / 256.0) * v[0];\n    for (int m = 1; m < 6; m++) acc = fma(LAG256[1][m] / 256.0, v[m], acc);", 1),
 ("centred = clamped", "val = cen_xyz(padded + ((size_t)v * t->n + L) * PBLK, f[0], f[1], f[2]);", "val = interp_xyz(src, f[0], f[1], f[2]);", 1),
 ("centred y window", "for (int m = 0; m < 6; m++) v[m] = cen_x(pad, fx, c0 - 2 + m, cz);", "for (int m = 0; m < 6; m++) v[m] = cen_x(pad, fx, c0 - 3 + m, cz);", 1),
 ("ghost dir decode", "int dlt[3] = { dir % 3 - 1, (dir / 3) % 3 - 1, dir / 9 - 1 };", "int dlt[3] = { dir / 9 - 1, (dir / 3) % 3 - 1, dir % 3 - 1 };", 1),
 ("zip offset", "padded[q * PBLK + ((size_t)(k + PAD) * NP + (j + PAD)) * NP + (i + PAD)];", "padded[q * PBLK + ((size_t)(k + PAD) * NP + (j + PAD)) * NP + (i + PAD - 1)];", 1),
]

def sandbox():
    """temporary copy of what the pin tests need: oracle source, pin tests, input generators"""
    tmp = tempfile.mkdtemp(prefix="octfd_mutants_")
    os.makedirs(os.path.join(tmp, "oracle"))
    for f in ("__init__.py", "octfd_oracle.c"):
        shutil.copy(os.path.join(ROOT, "oracle", f), os.path.join(tmp, "oracle", f))
    shutil.copytree(os.path.join(ROOT, "synthdata"), os.path.join(tmp, "synthdata"), ignore=shutil.ignore_patterns("__pycache__"))
    os.makedirs(os.path.join(tmp, "tests"))
    for f in ["conftest.py", "helpers.py"] + [os.path.basename(t) for t in PIN_TESTS]:
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(tmp, "tests", f))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(tmp, "tests", "golden"))
    return tmp


def run_mutant(tmp, original, name, old, new, nth, tests=None):
    """plants the mistake in the sandbox, runs its pin tests; returns (killed, first failing test)"""
    if original.count(old) < nth:
        raise ValueError("mutant %r: its text no longer occurs in the oracle source" % name)
    idx = -1
    for _ in range(nth):
        idx = original.index(old, idx + 1)
    with open(os.path.join(tmp, "oracle", "octfd_oracle.c"), "w") as f:
        f.write(original[:idx] + new + original[idx + len(old):])
    lib = os.path.join(tmp, "oracle", "liboctfd_oracle.so")
    if os.path.exists(lib):
        os.remove(lib)                       # the copy's loader compiles what it finds
    env = dict(os.environ, PYTHONPATH=tmp, PYTHONDONTWRITEBYTECODE="1")
    r = subprocess.run([sys.executable, "-m", "pytest"] + (tests or PIN_TESTS) + ["-x", "-q", "-p", "no:cacheprovider"],
                       cwd=tmp, env=env, capture_output=True, text=True, timeout=1800)
    failed = [l.split(" ")[1] for l in r.stdout.splitlines() if l.startswith(("FAILED", "ERROR"))]
    return r.returncode != 0, (failed[0] if failed else None)


def main(names):
    original = open(os.path.join(ROOT, "oracle", "octfd_oracle.c")).read()
    tmp = sandbox()
    survivors = []
    try:
        for name, old, new, nth in MUTANTS:
            if names and name not in names:
                continue
            killed, by = run_mutant(tmp, original, name, old, new, nth)
            print("%-30s %s" % (name, "killed by " + str(by) if killed else "SURVIVED"), flush=True)
            if not killed:
                survivors.append(name)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    print("survivors:", survivors)
    return 1 if survivors else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
