"""Python binding of liboctfd (C ABI in include/octfd.h): argument marshalling only.

Every step of the pipeline runs inside the library's HIP kernels.  PyTorch is used by callers for
device memory and streams; this module only takes `.data_ptr()` of the tensors it is given.  There
is no CPU fallback: a missing library or a failing call raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liboctfd.so")

DERIVS, WAVE, BURGERS, SYN24 = 0, 1, 2, 3
KINDS = {"DERIVS": DERIVS, "WAVE": WAVE, "BURGERS": BURGERS, "SYN24": SYN24}
OT_OK, OT_E_BADARG, OT_E_NOMEM, OT_E_UNBALANCED, OT_E_INCOMPLETE = 0, -1, -2, -3, -4
OT_E_WORKSPACE, OT_E_HIP, OT_E_NODEVICE, OT_E_UNSUPPORTED = -5, -6, -7, -8
STATIC_WORKSPACE_BYTES = 160 << 20   # OT_STATIC_WORKSPACE_BYTES

EXPORTS = ["octree_build", "octree_from_leaves", "octree_num_blocks", "octree_get_leaves",
           "octree_get_ghost_table", "octree_upload", "octree_free", "ot_rhs_nvar_in", "ot_rhs_nvar_out",
           "unzip", "rhs_eval", "zip", "rhs_eval_zipped", "rk_workspace_bytes", "rk_step", "rk_step_static",
           "unzip_centred", "rk_centred_workspace_bytes", "rk_step_centred",
           "regrid_plan", "regrid_table", "regrid_transfer", "regrid_free",
           "ot_strerror", "ot_last_hip_error"]


class OctfdError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (status %d, hip error %d)" % (what, strerror(status), status, last_hip_error()))


class BuildParams(C.Structure):
    _fields_ = [("lmin", C.c_uint32), ("lmax", C.c_uint32), ("npts", C.c_uint32),
                ("pts_q20", C.c_void_p), ("radius_q20", C.c_void_p),
                ("points_per_dim", C.c_uint32), ("pad", C.c_uint32), ("periodic", C.c_uint32)]


class RhsParams(C.Structure):
    _fields_ = [("ko_sigma", C.c_double), ("reserved", C.c_double * 7)]


_lib = None


def lib():
    """Loads liboctfd.so; raises if it has not been built (python -m paper_2007_12792_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("liboctfd.so is not built: run `python -m paper_2007_12792_amd.build` "
                           "(there is no fallback implementation)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz, dbl = C.c_void_p, C.c_int, C.c_int64, C.c_size_t, C.c_double
    sig = {
        "octree_build": [C.POINTER(BuildParams), C.POINTER(vp)],
        "octree_from_leaves": [vp, sz, C.c_uint32, C.POINTER(vp)],
        "octree_num_blocks": [vp, C.POINTER(i64)],
        "octree_get_leaves": [vp, vp, sz],
        "octree_get_ghost_table": [vp, vp, sz],
        "octree_upload": [vp],
        "octree_free": [vp],
        "ot_rhs_nvar_in": [i32],
        "ot_rhs_nvar_out": [i32],
        "unzip": [vp, i32, vp, vp, vp],
        "rhs_eval": [vp, i32, C.POINTER(RhsParams), vp, vp, vp],
        "zip": [vp, i32, vp, vp, vp],
        "rhs_eval_zipped": [vp, i32, C.POINTER(RhsParams), vp, vp, vp],
        "rk_workspace_bytes": [vp, i32, C.POINTER(sz)],
        "rk_step": [vp, i32, C.POINTER(RhsParams), dbl, vp, vp, sz, vp],
        "rk_step_static": [vp, i32, C.POINTER(RhsParams), dbl, vp, vp],
        "unzip_centred": [vp, i32, vp, vp, vp],
        "rk_centred_workspace_bytes": [vp, i32, C.POINTER(sz)],
        "rk_step_centred": [vp, i32, C.POINTER(RhsParams), dbl, vp, vp, sz, vp],
        "regrid_plan": [vp, vp, C.POINTER(vp)],
        "regrid_table": [vp, vp, sz],
        "regrid_transfer": [vp, i32, vp, vp, vp],
        "regrid_free": [vp],
        "ot_last_hip_error": [],
    }
    for name, args in sig.items():
        f = getattr(L, name)
        f.argtypes = args
        f.restype = i32
    L.ot_strerror.argtypes = [i32]
    L.ot_strerror.restype = C.c_char_p
    _lib = L
    return L


def strerror(status):
    return lib().ot_strerror(int(status)).decode()


def last_hip_error():
    return lib().ot_last_hip_error()


def _check(status, what):
    if status != OT_OK:
        raise OctfdError(status, what)


def nvar_in(kind):
    return lib().ot_rhs_nvar_in(kind)


def nvar_out(kind):
    return lib().ot_rhs_nvar_out(kind)


def _ptr(t):
    """device pointer of a torch tensor (must be contiguous float64 on the GPU)"""
    if not (t.is_cuda and t.is_contiguous() and t.dtype.is_floating_point and t.element_size() == 8):
        raise ValueError("expected a contiguous float64 CUDA tensor")
    return C.c_void_p(t.data_ptr())


def _shape(t, want, name):
    if tuple(t.shape) != tuple(want):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(want)))


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


class Tree:
    """Handle on an ot_tree.  Leaves and the ghost table are host numpy arrays."""

    def __init__(self, handle):
        self._h = handle
        n = C.c_int64()
        _check(lib().octree_num_blocks(self._h, C.byref(n)), "octree_num_blocks")
        self.n = n.value

    @classmethod
    def build(cls, lmin, lmax, pts_q20, radius_q20):
        pts = np.ascontiguousarray(pts_q20, dtype=np.uint32).reshape(-1, 3)
        rad = np.ascontiguousarray(radius_q20, dtype=np.uint32).reshape(-1)
        if rad.size < lmax - lmin:
            raise ValueError("need lmax-lmin radii")
        p = BuildParams(lmin, lmax, pts.shape[0], pts.ctypes.data_as(C.c_void_p),
                        rad.ctypes.data_as(C.c_void_p) if rad.size else None, 8, 3, 1)
        h = C.c_void_p()
        _check(lib().octree_build(C.byref(p), C.byref(h)), "octree_build")
        return cls(h)

    @classmethod
    def from_leaves(cls, leaves, pad=3):
        lv = np.ascontiguousarray(leaves, dtype=np.uint32).reshape(-1, 4)
        h = C.c_void_p()
        _check(lib().octree_from_leaves(lv.ctypes.data_as(C.c_void_p), lv.shape[0], pad, C.byref(h)),
               "octree_from_leaves")
        return cls(h)

    def __del__(self):
        try:
            if self._h:
                lib().octree_free(self._h)
                self._h = None
        except Exception:
            pass

    @property
    def leaves(self):
        out = np.empty((self.n, 4), dtype=np.uint32)
        _check(lib().octree_get_leaves(self._h, out.ctypes.data_as(C.c_void_p), self.n), "octree_get_leaves")
        return out

    def ghost_table(self):
        out = np.empty((self.n, 27, 5), dtype=np.int32)
        _check(lib().octree_get_ghost_table(self._h, out.ctypes.data_as(C.c_void_p), out.size), "octree_get_ghost_table")
        return out

    def upload(self):
        _check(lib().octree_upload(self._h), "octree_upload")

    # ---- device calls: tensors in, tensors out (outputs allocated by the caller) -------------
    def unzip(self, zipped, padded, stream=None):
        nvar = zipped.shape[0]
        _shape(zipped, (nvar, self.n, 8, 8, 8), "zipped")
        _shape(padded, (nvar, self.n, 14, 14, 14), "padded")
        _check(lib().unzip(self._h, nvar, _ptr(zipped), _ptr(padded), _stream(stream)), "unzip")

    def unzip_centred(self, zipped, padded, stream=None):
        nvar = zipped.shape[0]
        _shape(zipped, (nvar, self.n, 8, 8, 8), "zipped")
        _shape(padded, (nvar, self.n, 14, 14, 14), "padded")
        _check(lib().unzip_centred(self._h, nvar, _ptr(zipped), _ptr(padded), _stream(stream)), "unzip_centred")

    def zip(self, padded, zipped, stream=None):
        nvar = padded.shape[0]
        _shape(zipped, (nvar, self.n, 8, 8, 8), "zipped")
        _shape(padded, (nvar, self.n, 14, 14, 14), "padded")
        _check(lib().zip(self._h, nvar, _ptr(padded), _ptr(zipped), _stream(stream)), "zip")

    def rhs_eval(self, kind, padded, rhs_padded, sigma=0.0, stream=None):
        _shape(padded, (nvar_in(kind), self.n, 14, 14, 14), "padded")
        _shape(rhs_padded, (nvar_out(kind), self.n, 14, 14, 14), "rhs_padded")
        p = RhsParams(float(sigma))
        _check(lib().rhs_eval(self._h, kind, C.byref(p), _ptr(padded), _ptr(rhs_padded), _stream(stream)), "rhs_eval")

    def rhs_eval_zipped(self, kind, zipped, rhs_zipped, sigma=0.0, stream=None):
        _shape(zipped, (nvar_in(kind), self.n, 8, 8, 8), "zipped")
        _shape(rhs_zipped, (nvar_out(kind), self.n, 8, 8, 8), "rhs_zipped")
        p = RhsParams(float(sigma))
        _check(lib().rhs_eval_zipped(self._h, kind, C.byref(p), _ptr(zipped), _ptr(rhs_zipped), _stream(stream)),
               "rhs_eval_zipped")

    def rk_workspace_bytes(self, kind):
        n = C.c_size_t()
        _check(lib().rk_workspace_bytes(self._h, kind, C.byref(n)), "rk_workspace_bytes")
        return n.value

    def rk_step(self, kind, u, dt, workspace, sigma=0.0, stream=None):
        _shape(u, (nvar_in(kind), self.n, 8, 8, 8), "u")
        p = RhsParams(float(sigma))
        nbytes = workspace.numel() * workspace.element_size()
        _check(lib().rk_step(self._h, kind, C.byref(p), float(dt), _ptr(u), _ptr(workspace), nbytes, _stream(stream)),
               "rk_step")

    def rk_step_static(self, kind, u, dt, sigma=0.0, stream=None):
        """rk_step with the library's static device workspace (allocates nothing; needs upload() first)"""
        _shape(u, (nvar_in(kind), self.n, 8, 8, 8), "u")
        p = RhsParams(float(sigma))
        _check(lib().rk_step_static(self._h, kind, C.byref(p), float(dt), _ptr(u), _stream(stream)), "rk_step_static")

    def rk_centred_workspace_bytes(self, kind):
        n = C.c_size_t()
        _check(lib().rk_centred_workspace_bytes(self._h, kind, C.byref(n)), "rk_centred_workspace_bytes")
        return n.value

    def rk_step_centred(self, kind, u, dt, workspace, sigma=0.0, stream=None):
        _shape(u, (nvar_in(kind), self.n, 8, 8, 8), "u")
        p = RhsParams(float(sigma))
        nbytes = workspace.numel() * workspace.element_size()
        _check(lib().rk_step_centred(self._h, kind, C.byref(p), float(dt), _ptr(u), _ptr(workspace), nbytes,
                                     _stream(stream)), "rk_step_centred")


class Transfer:
    """Handle on an ot_transfer: carries zipped data from `src` (old tree) to `dst` (regridded tree)."""

    def __init__(self, src, dst):
        h = C.c_void_p()
        _check(lib().regrid_plan(src._h, dst._h, C.byref(h)), "regrid_plan")
        self._h = h
        self.n_from, self.n_to = src.n, dst.n

    def __del__(self):
        try:
            if self._h:
                lib().regrid_free(self._h)
                self._h = None
        except Exception:
            pass

    @property
    def table(self):
        """(n_to, 4) int32 rows {kind, first source leaf, number of source leaves, child octant}"""
        out = np.empty((self.n_to, 4), dtype=np.int32)
        _check(lib().regrid_table(self._h, out.ctypes.data_as(C.c_void_p), out.size), "regrid_table")
        return out

    def apply(self, zipped_from, zipped_to, stream=None):
        nvar = zipped_from.shape[0]
        _shape(zipped_from, (nvar, self.n_from, 8, 8, 8), "zipped_from")
        _shape(zipped_to, (nvar, self.n_to, 8, 8, 8), "zipped_to")
        _check(lib().regrid_transfer(self._h, nvar, _ptr(zipped_from), _ptr(zipped_to), _stream(stream)),
               "regrid_transfer")
