"""The paper's equation, initial data and domain as a multi-step run (introduction, Eq. "Inviscid_Burgers" with
the initial condition of Eq. "initial-condition", c = 3, t in [0, 0.2]): u_t + u u_x = 0 from u0 = (1 - cos 6 pi x)/2
steepens into three shocks at t_b = 1/(3 pi) = 0.1061.  It is integrated to t = 0.0996 (94 % of t_b) on adaptive
trees whose finest level is a band around the path of each steepening front, with both ghost rules, and compared

  * with the oracle's own step on every step (the small tree) or from the current state at sampled times (the
    larger tree), to the parity tolerance |gpu - oracle| <= 1e-12 |oracle| + 1e-13;
  * with the exact solution by characteristics u = u0(x - u t) until the front is thinner than the lattice can
    hold; the error history of each rule is printed, so that the time at which it departs can be read off.
"""
import numpy as np
import pytest
import torch

import paper_2007_12792_amd as octfd
import synthdata as sd
from helpers import assert_close, coords

pytestmark = pytest.mark.gpu
TP = 2.0 * np.pi
C = 3.0
T_SHOCK = 1.0 / (C * np.pi)


def band_params(lmax):
    """finest level on 0.25 <= x < 0.375 (+ 1/3, + 2/3): the fronts start at x = 1/4 + k/3 and move at speed 1/2;
    one seed point per column of level-4 octants, so that the refined region is a slab"""
    q = 1 << 20
    g = (np.arange(16) + 0.5) / 16
    pts = np.array([[int(x * q), int(y * q), int(z * q)] for x in (0.29, 0.29 + 1 / 3, 0.29 + 2 / 3) for y in g for z in g], np.uint32)
    return dict(lmin=3, lmax=lmax, pts_q20=pts, radius_q20=np.array([int(0.03 * q)] * (lmax - 3), np.uint32))


def exact(x, t):
    """u = u0(s) on the characteristic x = s + t u0(s); s by bisection (s + t u0(s) is increasing before t_b)"""
    xu, inv = np.unique(x, return_inverse=True)
    lo, hi = xu - t, xu.copy()
    for _ in range(70):
        s = 0.5 * (lo + hi)
        below = s + t * 0.5 * (1 - np.cos(TP * C * s)) < xu
        lo, hi = np.where(below, s, lo), np.where(below, hi, s)
    s = 0.5 * (lo + hi)
    return (0.5 * (1 - np.cos(TP * C * s)))[inv].reshape(x.shape)


def stepper(tree, rule, dev):
    if rule == "centred":
        ws = torch.empty(tree.rk_centred_workspace_bytes(octfd.BURGERS) // 8, dtype=torch.float64, device=dev)
        return lambda u, dt: tree.rk_step_centred(octfd.BURGERS, u, dt, ws, sigma=sd.KO_SIGMA)
    ws = torch.empty(tree.rk_workspace_bytes(octfd.BURGERS) // 8, dtype=torch.float64, device=dev)
    return lambda u, dt: tree.rk_step(octfd.BURGERS, u, dt, ws, sigma=sd.KO_SIGMA)


def oracle_step(to, rule, u, dt):
    return (to.rk4_step_centred if rule == "centred" else to.rk4_step)(octfd.BURGERS, u, dt, sigma=sd.KO_SIGMA)


def test_to_the_shock_on_a_two_level_tree_with_the_oracle_on_every_step(orc, dev):
    p = band_params(4)                                   # levels 3 and 4: 2,304 blocks, h = 1/128 in the bands
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    assert (to.leaves == tg.leaves).all() and len(set(to.leaves[:, 0])) == 2
    x = coords(to.leaves)[0]
    u0 = 0.5 * (1 - np.cos(TP * C * x))
    dt = sd.time_step(4)
    nsteps = int(0.1 / dt)                               # 51 steps, t = 0.0996
    assert 0.9 * T_SHOCK < nsteps * dt < T_SHOCK
    hist = {}
    for rule in ("clamped", "centred"):
        step = stepper(tg, rule, dev)
        ud = torch.from_numpy(u0[None].copy()).to(dev)
        ref = u0[None].copy()
        worst = 0.0
        for s in range(1, nsteps + 1):
            step(ud, dt)
            ref = oracle_step(to, rule, ref, dt)
            got = ud.cpu().numpy()
            err = np.abs(got - ref)
            bound = 1e-12 * np.abs(ref) + 1e-13
            assert (err <= bound).all(), "%s rule, step %d" % (rule, s)
            worst = max(worst, float((err / bound).max()))
            if s % 8 == 0 or s == nsteps:
                hist[rule, s] = float(np.abs(got[0] - exact(x, s * dt)).max())
        print("%s rule: %d steps, each equal to the oracle's (worst |diff|/bound %.3g); max error against characteristics:"
              % (rule, nsteps, worst), flush=True)
        print("   " + "  ".join("t=%.4f: %.2e" % (s * dt, hist[rule, s]) for (r, s) in sorted(hist) if r == rule), flush=True)
        assert np.isfinite(got).all() and got.max() < 1.1 and got.min() > -0.1
    # early on the error sits at the level jumps, where the centred stencils are several times more accurate; once
    # the fronts are a few points wide the error sits there, inside the bands, and the rules agree
    assert hist["centred", 16] < 0.5 * hist["clamped", 16]
    assert hist["clamped", 32] < 5e-3 and hist["centred", 32] < 5e-3
    assert abs(hist["clamped", nsteps] - hist["centred", nsteps]) < 0.1 * hist["clamped", nsteps]


def test_to_the_shock_on_the_finer_tree(orc, dev):
    p = band_params(5)                                   # levels 4 and 5: 14,848 blocks, h = 1/256 in the bands
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    assert (to.leaves == tg.leaves).all()
    x = coords(to.leaves)[0]
    u0 = 0.5 * (1 - np.cos(TP * C * x))
    dt = sd.time_step(5)
    nsteps = int(0.1 / dt)                               # 102 steps
    for rule in ("clamped", "centred"):
        step = stepper(tg, rule, dev)
        ud = torch.from_numpy(u0[None].copy()).to(dev)
        hist = {}
        for s in range(1, nsteps + 1):
            if s in (1, 52, nsteps):                     # the oracle's step from the state the device has reached
                want = oracle_step(to, rule, ud.cpu().numpy(), dt)
            step(ud, dt)
            if s in (1, 52, nsteps):
                assert_close(ud.cpu().numpy(), want, "%s rule, step %d from the device's state" % (rule, s))
            if s % 8 == 0 or s == nsteps:
                hist[s] = float(np.abs(ud.cpu().numpy()[0] - exact(x, s * dt)).max())
        print("%s rule, max error against characteristics: " % rule + "  ".join("t=%.4f: %.2e" % (s * dt, hist[s]) for s in sorted(hist)), flush=True)
        assert hist[64] < 1e-4                           # t = 0.0625: the fronts are still resolved
        assert hist[64] < hist[80] < hist[96]            # then the error climbs as their width falls below h
        assert np.isfinite(hist[nsteps]) and hist[nsteps] < 0.5
