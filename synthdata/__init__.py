"""Seeded synthetic inputs for the octree block finite-difference pipeline.

This module serves both the GPU library's callers and the CPU oracle's callers.  It holds
none of the method's arithmetic (no stencils, no interpolation, no tree construction): it only
draws seed points, refinement radii and initial field values.  Everything is a pure function of
an integer seed.  Field generators are written with torch ops so that the large workloads can be
generated on the GPU; the array that comes out is then handed, unchanged, to whichever side
consumes it (values are never regenerated independently on the two sides).

The source paper has no dataset for this path; these workloads stand in for adaptive runs with
two refinement centres and >= 80 % of the blocks on the finest level.
"""
import math

import numpy as np
import torch

MASK64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15
Q = 1 << 20  # seed points and radii live on the 2^20 lattice


# ------------------------------------------------------------------ splitmix64
class SplitMix64:
    """Scalar splitmix64 stream (python ints)."""

    def __init__(self, seed):
        self.s = seed & MASK64

    def next(self):
        self.s = (self.s + GAMMA) & MASK64
        z = self.s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)

    def uniform(self, lo=0.0, hi=1.0):
        return lo + (hi - lo) * ((self.next() >> 11) * 2.0 ** -53)


def _lshr(z, k):
    return (z >> k) & ((1 << (64 - k)) - 1)


def _as_i64(v):
    v &= MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


def splitmix_at(seed, counter):
    """n-th output (counter = n, int64 tensor) of the splitmix64 stream started at `seed`,
    computed element-wise with wrapping int64 arithmetic."""
    z = counter * _as_i64(GAMMA) + _as_i64(seed + GAMMA)
    z = (z ^ _lshr(z, 30)) * _as_i64(0xBF58476D1CE4E5B9)
    z = (z ^ _lshr(z, 27)) * _as_i64(0x94D049BB133111EB)
    return z ^ _lshr(z, 31)


def normal_noise(seed, numel, device="cpu", chunk=1 << 24):
    """numel standard normals, element e from outputs 2e and 2e+1 of the stream (Box-Muller)."""
    out = torch.empty(numel, dtype=torch.float64, device=device)
    for s in range(0, numel, chunk):
        e = torch.arange(s, min(numel, s + chunk), dtype=torch.int64, device=device)
        a = _lshr(splitmix_at(seed, 2 * e), 11).to(torch.float64)
        b = _lshr(splitmix_at(seed, 2 * e + 1), 11).to(torch.float64)
        u1 = (a + 1.0) * 2.0 ** -53
        u2 = b * 2.0 ** -53
        out[s:s + e.numel()] = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
    return out


# ------------------------------------------------------------------ seed points, radii
def seed_points(style, seed, phase=0.0):
    """Two refinement centres on the 2^20 lattice, (2,3) uint32.  `phase` (radians) advances the
    "orbit" pair along its circle: the moved centres of a later regrid."""
    r = SplitMix64(seed)
    if style == "rand":      # each coordinate in [1/4, 3/4)
        pts = [[(1 << 18) + (r.next() % (1 << 19)) for _ in range(3)] for _ in range(2)]
    elif style == "orbit":   # two points opposite each other on a circle of radius 0.15
        phi = 2.0 * math.pi * (r.next() / 2.0 ** 64) + phase
        pts = []
        for sgn in (+1.0, -1.0):
            p = (0.5 + sgn * 0.15 * math.cos(phi), 0.5 + sgn * 0.15 * math.sin(phi), 0.5 + 2.0 ** -20)
            pts.append([int(math.floor(c * Q)) for c in p])
    else:
        raise ValueError(style)
    return np.asarray(pts, dtype=np.uint32)


# name -> tree recipe and right-hand side.  radius_q20 has one entry per level lmin..lmax-1.
CONFIGS = {
    "C1": dict(lmin=3, lmax=3, style="rand", radius_q20=[], kind="DERIVS", field="sine"),
    "C2": dict(lmin=3, lmax=6, style="rand", radius_q20=[125829] * 3, kind="DERIVS", field="sine"),
    "C3": dict(lmin=3, lmax=7, style="rand", radius_q20=[125829] * 4, kind="WAVE", field="pulse"),
    "C3B": dict(lmin=3, lmax=7, style="rand", radius_q20=[125829] * 4, kind="BURGERS", field="burgers"),
    "C4": dict(lmin=3, lmax=7, style="rand", radius_q20=[89128] * 4, kind="SYN24", field="gauss24"),
    "C5": dict(lmin=3, lmax=9, style="orbit",
               radius_q20=[104857, 87031, 72236, 59956, 49763, 41303], kind="SYN24", field="gauss24"),
    # uniform tree of 32,768 blocks: no level jumps at all (isolates the cost of ghost interpolation)
    "U5": dict(lmin=5, lmax=5, style="rand", radius_q20=[], kind="SYN24", field="gauss24"),
    "U4": dict(lmin=4, lmax=4, style="rand", radius_q20=[], kind="SYN24", field="gauss24"),
    "U6": dict(lmin=6, lmax=6, style="rand", radius_q20=[], kind="SYN24", field="gauss24"),
    # small trees of the same shape, for element-by-element parity in seconds
    "T2": dict(lmin=3, lmax=5, style="rand", radius_q20=[60000, 40000], kind="DERIVS", field="sine"),
    "T3": dict(lmin=3, lmax=5, style="rand", radius_q20=[60000, 40000], kind="WAVE", field="pulse"),
    "T3B": dict(lmin=3, lmax=5, style="rand", radius_q20=[60000, 40000], kind="BURGERS", field="burgers"),
    "T4": dict(lmin=3, lmax=5, style="orbit", radius_q20=[70000, 45000], kind="SYN24", field="gauss24"),
}
KO_SIGMA = 0.4
CFL = 0.25


def tree_params(name, seed=1, phase=0.0):
    c = CONFIGS[name]
    return dict(lmin=c["lmin"], lmax=c["lmax"], pts_q20=seed_points(c["style"], seed, phase),
                radius_q20=np.asarray(c["radius_q20"], dtype=np.uint32))


def time_step(lmax):
    """dt = CFL * h at the finest level; a power of two."""
    return CFL * 2.0 ** -(lmax + 3)


# ------------------------------------------------------------------ node coordinates, fields
def node_coords(leaves, device="cpu"):
    """leaves (n,4) [level,ix,iy,iz] -> x, y, z float64 tensors (n,8,8,8) of owned-node coordinates."""
    lv = torch.as_tensor(np.asarray(leaves).astype(np.int64), device=device)
    h = torch.pow(2.0, -(lv[:, 0].to(torch.float64) + 3.0))
    i = torch.arange(8, dtype=torch.float64, device=device)
    n = lv.shape[0]

    def ax(col, shape):
        base = (8.0 * lv[:, col].to(torch.float64)).view(n, 1, 1, 1) + i.view(shape)
        return (base * h.view(n, 1, 1, 1)).expand(n, 8, 8, 8)

    return ax(1, (1, 1, 1, 8)), ax(2, (1, 1, 8, 1)), ax(3, (1, 8, 1, 1))


def _min_image(d):
    return d - torch.round(d)


def _gauss(x, y, z, centre, width):
    r2 = _min_image(x - centre[0]) ** 2 + _min_image(y - centre[1]) ** 2 + _min_image(z - centre[2]) ** 2
    return torch.exp(-r2 / (2.0 * width * width))


def make_fields(name, leaves, seed=1, device="cpu"):
    """Initial zipped state [nvar][n][8][8][8] (float64 tensor on `device`) for a named workload."""
    c = CONFIGS[name]
    x, y, z = node_coords(leaves, device)
    n = x.shape[0]
    kind = c["field"]
    tp = 2.0 * math.pi
    if kind == "sine":
        u = torch.sin(tp * x) * torch.sin(tp * y) * torch.sin(tp * z)
        u = u + 1e-3 * normal_noise(seed + 101, n * 512, device).view(n, 8, 8, 8)
        return u.unsqueeze(0).contiguous()
    if kind == "pulse":
        pts = seed_points(c["style"], seed).astype(np.float64) / Q
        u = _gauss(x, y, z, pts[0], 0.05) + _gauss(x, y, z, pts[1], 0.05)
        return torch.stack([u, torch.zeros_like(u)]).contiguous()
    if kind == "burgers":   # the paper's one-parameter initial condition with c = 3, constant in y and z
        u = 0.5 * (1.0 - torch.cos(tp * 3.0 * x))
        return u.unsqueeze(0).contiguous()
    if kind == "gauss24":
        r = SplitMix64(seed + 202)
        out = torch.empty((24, n, 8, 8, 8), dtype=torch.float64, device=device)
        for a in range(24):
            f = torch.zeros((n, 8, 8, 8), dtype=torch.float64, device=device)
            for _ in range(4):
                ctr = [r.uniform(0.25, 0.75) for _ in range(3)]
                amp = r.uniform(0.1, 1.0)
                wid = r.uniform(0.05, 0.2)
                f += amp * _gauss(x, y, z, ctr, wid)
            f += 1e-6 * normal_noise(seed + 303 + a, n * 512, device).view(n, 8, 8, 8)
            out[a] = f
        return out
    raise ValueError(kind)
