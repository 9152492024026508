"""More parity cases for the HIP path: uniform periodic trees (every neighbour is reached through
the wrap), other seeds, blocks with the maximum number of coarser sources, invariants that must hold
bit for bit, and a multi-step Burgers run against the method of characteristics."""
import numpy as np
import pytest
import torch

import paper_2007_12792_amd as octfd
import synthdata as sd
from helpers import assert_close, dev_empty, trees

pytestmark = pytest.mark.gpu
TP = 2.0 * np.pi


def uniform(orc, level):
    p = dict(lmin=level, lmax=level, pts_q20=np.zeros((1, 3), np.uint32), radius_q20=np.zeros(1, np.uint32))
    return orc.Tree.build(**p), octfd.Tree.build(**p)


@pytest.mark.parametrize("kind", [0, 1, 2, 3])
def test_uniform_level3_every_kind(orc, dev, kind):
    to, tg = uniform(orc, 3)
    rng = np.random.default_rng(30 + kind)
    u = rng.standard_normal((octfd.nvar_in(kind), to.n, 8, 8, 8))
    want = to.F(kind, u, sigma=0.4)
    out = dev_empty((octfd.nvar_out(kind), to.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(kind, torch.from_numpy(u).to(dev), out, sigma=0.4)
    assert_close(out.cpu().numpy(), want, "uniform L3 kind %d" % kind)


@pytest.mark.parametrize("seed", [2, 3])
def test_other_seeds_syn24_rk_step(orc, dev, seed):
    to, tg = trees(orc, "T4", seed)
    u = sd.make_fields("T4", to.leaves, seed).numpy()
    dt = sd.time_step(5)
    want = to.rk4_step(3, u, dt, sigma=0.4)
    ud = torch.from_numpy(u).to(dev)
    ws = torch.empty(tg.rk_workspace_bytes(3) // 8, dtype=torch.float64, device=dev)
    tg.rk_step(3, ud, dt, ws, sigma=0.4)
    assert_close(ud.cpu().numpy(), want, "T4 seed %d" % seed)


def test_block_with_seven_coarser_sources(orc, dev):
    # one level-3 octant refined twice around a single point: the level-5 blocks in the corners of
    # the level-4 octet see coarser leaves on three faces, three edges and one corner
    p = dict(lmin=3, lmax=5, pts_q20=np.array([[530000, 530000, 530000]], np.uint32), radius_q20=np.array([20000, 3000], np.uint32))
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    g = tg.ghost_table()
    nsrc = [len({int(g[b, d, 1]) for d in range(27) if g[b, d, 0] == 2}) for b in range(tg.n)]
    assert max(nsrc) == 7
    rng = np.random.default_rng(40)
    u = rng.standard_normal((24, to.n, 8, 8, 8))
    ud = torch.from_numpy(u).to(dev)
    pd = dev_empty((24, to.n, 14, 14, 14), dev)
    tg.unzip(ud, pd)
    assert (pd.cpu().numpy() == to.unzip(u)).all()
    out = dev_empty((24, to.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(3, ud, out, sigma=0.4)
    assert_close(out.cpu().numpy(), to.F(3, u, sigma=0.4), "seven coarser sources")


def test_invariants_hold_bit_for_bit(orc, dev):
    to, tg = trees(orc, "T3")
    rng = np.random.default_rng(41)
    u = torch.from_numpy(rng.standard_normal((2, to.n, 8, 8, 8))).to(dev)
    f1, f2, f0 = (dev_empty((2, to.n, 8, 8, 8), dev) for _ in range(3))
    tg.rhs_eval_zipped(1, u, f1, sigma=0.5)
    tg.rhs_eval_zipped(1, 2.0 * u, f2, sigma=0.5)
    assert torch.equal(f2, 2.0 * f1)                      # linear kind, power-of-two scaling
    tg.rhs_eval_zipped(1, u, f0, sigma=0.0)
    assert torch.equal(f0[0], u[1])                       # KO contributes exactly nothing
    c = torch.full((2, to.n, 8, 8, 8), 0.75, dtype=torch.float64, device=dev)
    c[1] = 0.0
    ws = torch.empty(tg.rk_workspace_bytes(1) // 8, dtype=torch.float64, device=dev)
    before = c.clone()
    tg.rk_step(1, c, 2.0 ** -10, ws, sigma=0.4)
    assert torch.equal(c, before)                         # a stationary state stays put
    pd = dev_empty((2, to.n, 14, 14, 14), dev)
    back = dev_empty((2, to.n, 8, 8, 8), dev)
    tg.unzip(u, pd)
    tg.zip(pd, back)
    assert torch.equal(back, u)                           # zip(unzip(u)) == u


def test_burgers_many_steps_towards_the_shock(orc, dev):
    # the paper's equation and initial data with c = 1 on a uniform 128^3 lattice, integrated to
    # t = 0.15 (the shock forms at 1/pi = 0.318): compare with the solution by characteristics
    to, tg = uniform(orc, 4)
    lv = to.leaves.astype(np.int64)
    x = ((8 * lv[:, 1])[:, None, None, None] + np.arange(8)[None, None, None, :]) / 128.0
    x = np.broadcast_to(x, (to.n, 8, 8, 8))
    u0 = 0.5 * (1 - np.cos(TP * x))
    dt, nsteps = 2.0 ** -9, 77
    ud = torch.from_numpy(u0[None].copy()).to(dev)
    ws = torch.empty(tg.rk_workspace_bytes(2) // 8, dtype=torch.float64, device=dev)
    for _ in range(nsteps):
        tg.rk_step(2, ud, dt, ws, sigma=0.05)
    t = dt * nsteps
    u = u0.copy()
    for _ in range(200):                                  # Newton on u = u0(x - u t)
        s = x - u * t
        r = u - 0.5 * (1 - np.cos(TP * s))
        u = u - r / (1 + t * 0.5 * TP * np.sin(TP * s))
    got = ud.cpu().numpy()[0]
    assert np.abs(got - u).max() < 2e-6
    assert np.abs(got - u0).max() > 0.2                   # the profile has steepened a lot
    # and the first three steps agree with the oracle to the parity tolerance
    ud = torch.from_numpy(u0[None].copy()).to(dev)
    ref = u0[None].copy()
    for _ in range(3):
        tg.rk_step(2, ud, dt, ws, sigma=0.05)
        ref = to.rk4_step(2, ref, dt, sigma=0.05)
    assert_close(ud.cpu().numpy(), ref, "3 Burgers steps")


def corner_params(lmax=6):
    """refinement centred next to the corner of the periodic cube: the level jumps sit on the wrap"""
    q = 1 << 20
    pts = np.array([[40, q - 30, 17], [q - 5, 9, q - 1]], dtype=np.uint32)
    return dict(lmin=3, lmax=lmax, pts_q20=pts, radius_q20=np.array([90000, 60000, 40000][:lmax - 3], np.uint32))


def test_level_jumps_across_the_periodic_wrap(orc, dev):
    p = corner_params()
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    assert (to.leaves == tg.leaves).all() and (to.ghost_table() == tg.ghost_table()).all()
    lv = to.leaves.astype(np.int64)
    fine = lv[:, 0] == 6
    edge = np.zeros(to.n, dtype=bool)
    for c in (1, 2, 3):
        edge |= (lv[:, c] == 0) | (lv[:, c] == (1 << lv[:, 0]) - 1)
    assert (fine & edge).sum() > 50                   # finest blocks that touch the wrap
    rng = np.random.default_rng(8)
    u = rng.standard_normal((24, to.n, 8, 8, 8))
    ud = torch.from_numpy(u).to(dev)
    # ghost fill, both rules
    for name, fo, fg in (("unzip", to.unzip, tg.unzip), ("unzip_centred", to.unzip_centred, tg.unzip_centred)):
        pad = dev_empty((2, to.n, 14, 14, 14), dev)
        fg(ud[:2].contiguous(), pad)
        assert_close(pad.cpu().numpy(), fo(u[:2]), "%s across the wrap" % name)
    # the 24-field right-hand side and one step with each rule
    out = dev_empty((24, to.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(3, ud, out, sigma=0.4)
    assert_close(out.cpu().numpy(), to.F(3, u, sigma=0.4), "SYN24 right-hand side across the wrap")
    us = 0.01 * u[:2]
    dt = sd.time_step(6)
    for name, so, sg_, wsb in (("rk_step", to.rk4_step, tg.rk_step, tg.rk_workspace_bytes(1)),
                               ("rk_step_centred", to.rk4_step_centred, tg.rk_step_centred, tg.rk_centred_workspace_bytes(1))):
        x = torch.from_numpy(us).to(dev).clone()
        sg_(1, x, dt, torch.empty(wsb // 8, dtype=torch.float64, device=dev), sigma=0.4)
        assert_close(x.cpu().numpy(), so(1, us, dt, 0.4), "%s across the wrap" % name)
    # regrid to centres moved further round the corner
    p2 = dict(p, pts_q20=(p["pts_q20"].astype(np.int64) + np.array([[6000, 6000, -5000], [-7000, 3000, 4000]])) % (1 << 20))
    p2["pts_q20"] = p2["pts_q20"].astype(np.uint32)
    to2, tg2 = orc.Tree.build(**p2), octfd.Tree.build(**p2)
    got = dev_empty((2, to2.n, 8, 8, 8), dev)
    octfd.Transfer(tg, tg2).apply(ud[:2].contiguous(), got)
    assert_close(got.cpu().numpy(), orc.transfer(to, to2, u[:2]), "regrid across the wrap")


def test_thirteen_levels(orc, dev):
    """levels 3..15 around one point: grid spacings from 2^-6 down to 2^-18 in one tree"""
    lmax = 15
    rad = np.array([int(1.6 * 2 ** (20 - l)) for l in range(3, lmax)], np.uint32)
    p = dict(lmin=3, lmax=lmax, pts_q20=np.array([[333333, 777777, 555555]], np.uint32), radius_q20=rad)
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    assert (to.leaves == tg.leaves).all() and (to.ghost_table() == tg.ghost_table()).all()
    assert sorted(set(to.leaves[:, 0])) == list(range(3, lmax + 1))
    u = np.random.default_rng(12).standard_normal((24, to.n, 8, 8, 8))
    ud = torch.from_numpy(u).to(dev)
    out = dev_empty((24, to.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(3, ud, out, sigma=0.4)
    assert_close(out.cpu().numpy(), to.F(3, u, sigma=0.4), "SYN24 right-hand side, levels 3..15")
    us = u[:2].copy()
    dt = sd.time_step(lmax)
    x = torch.from_numpy(us).to(dev).clone()
    tg.rk_step_centred(1, x, dt, torch.empty(tg.rk_centred_workspace_bytes(1) // 8, dtype=torch.float64, device=dev), sigma=0.4)
    assert_close(x.cpu().numpy(), to.rk4_step_centred(1, us, dt, 0.4), "rk_step_centred, levels 3..15")
    # coarsen everything back to level 3: injection through up to twelve levels
    t3o, t3g = uniform(orc, 3)
    got = dev_empty((2, t3g.n, 8, 8, 8), dev)
    octfd.Transfer(tg, t3g).apply(ud[:2].contiguous(), got)
    want = orc.transfer(to, t3o, u[:2])
    assert (got.cpu().numpy() == want).all()


@pytest.mark.parametrize("name,kind,nsteps", [("T3", 1, 3), ("T4", 3, 2)])
def test_rk_step_can_be_captured_in_a_graph_and_replayed(dev, name, kind, nsteps):
    """After octree_upload the device calls only enqueue kernels: no allocation, no synchronisation,
    no memset.  A step captured in a graph must replay to the same bits as eager steps, every time.
    (Two steps only for the 24-field system, whose values overflow after a few steps at this dt.)"""
    tg = octfd.Tree.build(**sd.tree_params(name, 1))
    tg.upload()
    u0 = sd.make_fields(name, tg.leaves, 1, device=dev)
    dt = sd.time_step(5)
    ws = torch.empty(tg.rk_workspace_bytes(kind) // 8, dtype=torch.float64, device=dev)
    eager = []
    u = u0.clone()
    for _ in range(nsteps):
        tg.rk_step(kind, u, dt, ws, sigma=0.4)
        eager.append(u.clone())
    torch.cuda.synchronize()
    assert torch.isfinite(eager[-1]).all()
    ug = u0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        tg.rk_step(kind, ug, dt, ws, sigma=0.4)       # warm-up on a side stream, as graph capture asks
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    ug.copy_(u0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        tg.rk_step(kind, ug, dt, ws, sigma=0.4)       # stream=None -> the current (capturing) stream
    ug.copy_(u0)
    for n in range(nsteps):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ug, eager[n]), "replay %d" % n
        assert np.isfinite((eager[n] * 0.5).sum().item())   # eager work and a synchronisation between replays


def test_two_trees_step_concurrently_on_two_streams(dev):
    # calls on different trees may overlap: steps of a wave tree and of a 24-field tree issued alternately on two
    # streams give the bits of the same steps issued one after the other
    ta, tb = octfd.Tree.build(**sd.tree_params("T3")), octfd.Tree.build(**sd.tree_params("T4"))
    ua0 = sd.make_fields("T3", ta.leaves, device=dev)
    ub0 = sd.make_fields("T4", tb.leaves, device=dev)
    wa = torch.empty(ta.rk_workspace_bytes(1) // 8, dtype=torch.float64, device=dev)
    wb = torch.empty(tb.rk_workspace_bytes(3) // 8, dtype=torch.float64, device=dev)
    dta, dtb = sd.time_step(sd.CONFIGS["T3"]["lmax"]), sd.time_step(sd.CONFIGS["T4"]["lmax"])
    ua, ub = ua0.clone(), ub0.clone()
    for _ in range(2):
        ta.rk_step(1, ua, dta, wa, sigma=sd.KO_SIGMA)
    for _ in range(2):
        tb.rk_step(3, ub, dtb, wb, sigma=sd.KO_SIGMA)
    torch.cuda.synchronize()
    va, vb = ua0.clone(), ub0.clone()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(2):
        with torch.cuda.stream(sa):
            ta.rk_step(1, va, dta, wa, sigma=sd.KO_SIGMA, stream=sa)
        with torch.cuda.stream(sb):
            tb.rk_step(3, vb, dtb, wb, sigma=sd.KO_SIGMA, stream=sb)
    sa.synchronize()
    sb.synchronize()
    assert torch.isfinite(va).all() and torch.isfinite(vb).all()
    assert torch.equal(va, ua) and torch.equal(vb, ub)


@pytest.mark.parametrize("seed", [11, 12, 13, 14, 15, 16])
def test_random_trees_24_field_right_hand_side(orc, dev, seed):
    # random refinement centres, radii and depths: many shapes of level jumps (one to seven coarser sources per
    # block, corner-only sources, units of the launch schedule that are mostly padding), every value compared
    rng = np.random.default_rng(seed)
    lmax = int(rng.integers(4, 7))
    npts = int(rng.integers(1, 4))
    pts = rng.integers(0, 1 << 20, size=(npts, 3)).astype(np.uint32)
    rad = rng.integers(20000, 140000, size=lmax - 3).astype(np.uint32)
    to = orc.Tree.build(3, lmax, pts, rad)
    tg = octfd.Tree.build(3, lmax, pts, rad)
    assert to.n == tg.n and to.n < 30000
    u = rng.standard_normal((24, to.n, 8, 8, 8))
    want = to.F(3, u, sigma=0.4)
    out = torch.full((24, to.n, 8, 8, 8), float("nan"), dtype=torch.float64, device=dev)
    tg.rhs_eval_zipped(3, torch.from_numpy(u).to(dev), out, sigma=0.4)
    got = out.cpu().numpy()
    print("seed %d: %d blocks, levels 3..%d, %d values differ" % (seed, to.n, lmax, int((got != want).sum())), flush=True)
    assert_close(got, want, "random tree %d" % seed)


def test_24_field_system_over_many_steps_with_a_stable_time_step(orc, dev):
    """The prescribed step dt = h/4 is far beyond the explicit stability limit of the 24-field system's second-derivative
    term, so the benchmark workload cannot be evolved.  With dt = h^2/16 it can (h^2/4 still blows up within ten steps): 24
    steps of rk_step and of rk_step_centred on
    the three-level tree, each compared with the oracle's step from the same state, and the state stays bounded."""
    to, tg = trees(orc, "T4")
    u0 = sd.make_fields("T4", to.leaves).numpy()
    dt = 2.0 ** -20                                        # h = 2^-8 on level 5
    for rule in ("clamped", "centred"):
        ud = torch.from_numpy(u0).to(dev)
        ws = torch.empty(tg.rk_workspace_bytes(3) // 8, dtype=torch.float64, device=dev)
        worst = 0.0
        for s in range(24):
            if s % 6 == 0:                                 # the oracle's step from the state the device has reached
                want = (to.rk4_step_centred if rule == "centred" else to.rk4_step)(3, ud.cpu().numpy(), dt, sigma=sd.KO_SIGMA)
            (tg.rk_step_centred if rule == "centred" else tg.rk_step)(3, ud, dt, ws, sigma=sd.KO_SIGMA)
            if s % 6 == 0:
                got = ud.cpu().numpy()
                err = np.abs(got - want)
                bound = 1e-12 * np.abs(want) + 1e-13
                assert (err <= bound).all(), "%s rule, step %d" % (rule, s)
                worst = max(worst, float((err / bound).max()))
        got = ud.cpu().numpy()
        print("%s rule: 24 steps, max |u| %.4f (start %.4f), worst |diff|/bound against the oracle's step %.3g"
              % (rule, np.abs(got).max(), np.abs(u0).max(), worst), flush=True)
        assert np.isfinite(got).all() and np.abs(got).max() < 1.5 * np.abs(u0).max()
        assert np.abs(got - u0).max() > 1e-6               # it has moved
