"""ctypes loader for the plain CPU oracle (oracle/octfd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's cpu-baseline
leg.  The product package never imports this module.  All arithmetic lives in the C file; this
module only marshals numpy arrays.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "octfd_oracle.c")
_LIB = os.path.join(_HERE, "liboctfd_oracle.so")

DERIVS, WAVE, BURGERS, SYN24 = 0, 1, 2, 3
NVAR_IN = {DERIVS: 1, WAVE: 2, BURGERS: 1, SYN24: 24}
NVAR_OUT = {DERIVS: 4, WAVE: 2, BURGERS: 1, SYN24: 24}
G_SAME, G_FINER, G_COARSER = 0, 1, 2


def build(force=False):
    """Compile the oracle with gcc: -O2, no contraction (fma only where the source says fma)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-mfma", "-fopenmp", "-fPIC", "-shared",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.check_call(cmd)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, i64, i32, dbl = C.c_void_p, C.c_int64, C.c_int, C.c_double
        L.orc_tree_build.restype = i64
        L.orc_tree_build.argtypes = [i32, i32, i32, vp, vp, C.POINTER(vp)]
        L.orc_tree_from_leaves.restype = i64
        L.orc_tree_from_leaves.argtypes = [vp, i64, C.POINTER(vp)]
        L.orc_tree_size.restype = i64
        L.orc_tree_size.argtypes = [vp]
        L.orc_tree_leaves.restype = None
        L.orc_tree_leaves.argtypes = [vp, vp]
        L.orc_tree_free.restype = None
        L.orc_tree_free.argtypes = [vp]
        L.orc_unzip.restype = None
        L.orc_unzip.argtypes = [vp, i32, vp, vp, vp, i64]
        L.orc_zip.restype = None
        L.orc_zip.argtypes = [i32, i64, vp, vp]
        L.orc_ghost_table.restype = i32
        L.orc_ghost_table.argtypes = [vp, vp]
        L.orc_rhs.restype = None
        L.orc_rhs.argtypes = [i32, dbl, i64, vp, vp, vp]
        L.orc_F.restype = None
        L.orc_F.argtypes = [vp, i32, dbl, vp, vp, i64, vp]
        L.orc_rk4_step.restype = i32
        L.orc_rk4_step.argtypes = [vp, i32, dbl, dbl, vp]
        for name in ("orc_d1_line", "orc_d2_line"):
            f = getattr(L, name)
            f.restype = dbl
            f.argtypes = [vp, dbl]
        L.orc_unzip_centred.restype = None
        L.orc_unzip_centred.argtypes = [vp, i32, vp, vp]
        L.orc_F_centred.restype = None
        L.orc_F_centred.argtypes = [vp, i32, dbl, vp, vp]
        L.orc_rk4_step_centred.restype = i32
        L.orc_rk4_step_centred.argtypes = [vp, i32, dbl, dbl, vp]
        L.orc_transfer.restype = i32
        L.orc_transfer.argtypes = [vp, vp, i32, vp, vp]
        L.orc_ko_line.restype = dbl
        L.orc_ko_line.argtypes = [vp]
        L.orc_interp.restype = dbl
        L.orc_interp.argtypes = [vp, i32, i32, i32]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


class Tree:
    """Oracle octree: leaves in Morton order, (n,4) uint32 rows (level, ix, iy, iz)."""

    def __init__(self, handle, n):
        self._h = handle
        self.n = int(n)
        self.leaves = np.empty((self.n, 4), dtype=np.uint32)
        lib().orc_tree_leaves(self._h, _p(self.leaves))

    @classmethod
    def build(cls, lmin, lmax, pts_q20, radius_q20):
        pts = np.ascontiguousarray(pts_q20, dtype=np.uint32).reshape(-1, 3)
        rad = np.ascontiguousarray(radius_q20, dtype=np.uint32).reshape(-1)
        assert rad.size >= lmax - lmin
        if rad.size == 0:
            rad = np.zeros(1, dtype=np.uint32)
        h = C.c_void_p()
        n = lib().orc_tree_build(lmin, lmax, pts.shape[0], _p(pts), _p(rad), C.byref(h))
        if n < 0:
            raise ValueError("orc_tree_build failed: %d" % n)
        return cls(h, n)

    @classmethod
    def from_leaves(cls, leaves):
        lv = np.ascontiguousarray(leaves, dtype=np.uint32).reshape(-1, 4)
        h = C.c_void_p()
        n = lib().orc_tree_from_leaves(_p(lv), lv.shape[0], C.byref(h))
        if n < 0:
            lib().orc_tree_free(h)
            raise ValueError({-3: "unbalanced", -4: "incomplete"}.get(n, "bad leaf list"))
        return cls(h, n)

    def __del__(self):
        try:
            if self._h:
                lib().orc_tree_free(self._h)
                self._h = None
        except Exception:
            pass

    # -- tables ---------------------------------------------------------------
    def ghost_table(self):
        out = np.empty((self.n, 27, 5), dtype=np.int32)
        bad = lib().orc_ghost_table(self._h, _p(out))
        if bad:
            raise ValueError("tree is not 26-balanced (%d inconsistent ghost regions)" % bad)
        return out

    # -- pipeline -------------------------------------------------------------
    def _sel(self, blocks):
        if blocks is None:
            return None, self.n, None
        b = np.ascontiguousarray(blocks, dtype=np.int64)
        return b, b.size, _p(b)

    def unzip(self, zipped, blocks=None):
        z = _f64(zipped)
        nvar = z.shape[0]
        assert z.shape == (nvar, self.n, 8, 8, 8)
        b, nsel, bp = self._sel(blocks)
        out = np.empty((nvar, nsel, 14, 14, 14), dtype=np.float64)
        lib().orc_unzip(self._h, nvar, _p(z), _p(out), bp, nsel)
        return out

    def unzip_centred(self, zipped):
        """ghost rule with centred coarse-lattice stencils (coarsest level first); all blocks"""
        z = _f64(zipped)
        nvar = z.shape[0]
        assert z.shape == (nvar, self.n, 8, 8, 8)
        out = np.full((nvar, self.n, 14, 14, 14), np.nan, dtype=np.float64)
        lib().orc_unzip_centred(self._h, nvar, _p(z), _p(out))
        return out

    def levels(self, blocks=None):
        lv = self.leaves[:, 0] if blocks is None else self.leaves[np.asarray(blocks), 0]
        return np.ascontiguousarray(lv, dtype=np.uint32)

    def rhs(self, kind, padded, sigma=0.0, blocks=None):
        p = _f64(padded)
        nsel = p.shape[1]
        assert p.shape == (NVAR_IN[kind], nsel, 14, 14, 14)
        lev = self.levels(blocks)
        assert lev.size == nsel
        out = np.zeros((NVAR_OUT[kind], nsel, 14, 14, 14), dtype=np.float64)
        lib().orc_rhs(kind, float(sigma), nsel, _p(lev), _p(p), _p(out))
        return out

    @staticmethod
    def zip(padded):
        p = _f64(padded)
        nvar, nsel = p.shape[:2]
        out = np.empty((nvar, nsel, 8, 8, 8), dtype=np.float64)
        lib().orc_zip(nvar, nsel, _p(p), _p(out))
        return out

    def F(self, kind, zipped, sigma=0.0, blocks=None):
        z = _f64(zipped)
        assert z.shape == (NVAR_IN[kind], self.n, 8, 8, 8)
        b, nsel, bp = self._sel(blocks)
        out = np.empty((NVAR_OUT[kind], nsel, 8, 8, 8), dtype=np.float64)
        lib().orc_F(self._h, kind, float(sigma), _p(z), bp, nsel, _p(out))
        return out

    def F_centred(self, kind, zipped, sigma=0.0):
        z = _f64(zipped)
        assert z.shape == (NVAR_IN[kind], self.n, 8, 8, 8)
        out = np.empty((NVAR_OUT[kind], self.n, 8, 8, 8), dtype=np.float64)
        lib().orc_F_centred(self._h, kind, float(sigma), _p(z), _p(out))
        return out

    def rk4_step_centred(self, kind, u, dt, sigma=0.0):
        z = _f64(u).copy()
        assert z.shape == (NVAR_IN[kind], self.n, 8, 8, 8)
        rc = lib().orc_rk4_step_centred(self._h, kind, float(sigma), float(dt), _p(z))
        if rc:
            raise ValueError("rk4 needs nvar_in == nvar_out")
        return z

    def rk4_step(self, kind, u, dt, sigma=0.0):
        z = _f64(u).copy()
        assert z.shape == (NVAR_IN[kind], self.n, 8, 8, 8)
        rc = lib().orc_rk4_step(self._h, kind, float(sigma), float(dt), _p(z))
        if rc:
            raise ValueError("rk4 needs nvar_in == nvar_out")
        return z


def transfer(src_tree, dst_tree, zipped):
    """Zipped data on src_tree -> zipped data on dst_tree (copy / injection / interpolation from a
    leaf one level coarser).  Raises ValueError when dst_tree is somewhere two or more levels finer."""
    z = _f64(zipped)
    nvar = z.shape[0]
    assert z.shape == (nvar, src_tree.n, 8, 8, 8)
    out = np.empty((nvar, dst_tree.n, 8, 8, 8), dtype=np.float64)
    rc = lib().orc_transfer(src_tree._h, dst_tree._h, nvar, _p(z), _p(out))
    if rc:
        raise ValueError("target tree is two or more levels finer than the source tree somewhere (%d)" % rc)
    return out


def d1_line(u7, ih):
    return lib().orc_d1_line(_p(_f64(u7)), float(ih))


def d2_line(u7, ih2):
    return lib().orc_d2_line(_p(_f64(u7)), float(ih2))


def ko_line(u7):
    return lib().orc_ko_line(_p(_f64(u7)))


def interp(src8, fx, fy, fz):
    s = _f64(src8)
    assert s.shape == (8, 8, 8)
    return lib().orc_interp(_p(s), int(fx), int(fy), int(fz))
