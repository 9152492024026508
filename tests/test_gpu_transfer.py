"""Parity of the inter-grid transfer kernel (through the C ABI) against the CPU oracle, element by
element.  The copied and injected values must be bit-identical; the interpolated ones follow the
same IEEE operation sequence on both sides, so they are normally bit-identical too
(bound: |gpu - oracle| <= 1e-12 |oracle| + 1e-13)."""
import numpy as np
import pytest
import torch

import paper_2007_12792_amd as octfd
import synthdata as sd
from helpers import ATOL, RTOL

pytestmark = pytest.mark.gpu


def both(orc, params):
    return orc.Tree.build(**params), octfd.Tree.build(**params)


def check(orc, dev, pa, pb, nvar, what, seed=0):
    oa, ga = both(orc, pa)
    ob, gb = both(orc, pb)
    assert (oa.leaves == ga.leaves).all() and (ob.leaves == gb.leaves).all()
    u = np.random.default_rng(seed).standard_normal((nvar, oa.n, 8, 8, 8))
    want = orc.transfer(oa, ob, u)
    plan = octfd.Transfer(ga, gb)
    tab = plan.table
    got = torch.full((nvar, gb.n, 8, 8, 8), float("nan"), dtype=torch.float64, device=dev)
    plan.apply(torch.from_numpy(u).to(dev), got)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    exact = tab[:, 0] != 1
    nz = int((got != want).sum())
    print("%s: %d -> %d blocks, kinds %s, %d of %d values differ" % (what, oa.n, ob.n, np.bincount(tab[:, 0], minlength=3), nz, got.size), flush=True)
    assert np.isfinite(got).all()
    assert (got[:, exact] == want[:, exact]).all()
    assert (np.abs(got - want) <= RTOL * np.abs(want) + ATOL).all()
    return tab


def test_orbit_regrid_small(orc, dev):
    tab = check(orc, dev, sd.tree_params("T4", 1), sd.tree_params("T4", 1, phase=0.35), 3, "T4 phase 0.35")
    assert all((tab[:, 0] == k).any() for k in (0, 1, 2))


def test_identity_and_tiny_move(orc, dev):
    check(orc, dev, sd.tree_params("T4", 1), sd.tree_params("T4", 1), 2, "T4 identity")
    check(orc, dev, sd.tree_params("T2", 1), sd.tree_params("T2", 1, phase=0.0) | {"pts_q20": sd.seed_points("rand", 1) + np.uint32(3000)}, 1, "T2 shifted centres")


def test_deep_injection_and_pure_prolongation(orc, dev):
    fine = dict(lmin=3, lmax=7, pts_q20=np.array([[300000, 500000, 700000]], np.uint32), radius_q20=np.array([30000] * 4, np.uint32))
    uni3 = dict(lmin=3, lmax=3, pts_q20=np.zeros((1, 3), np.uint32), radius_q20=np.zeros(0, np.uint32))
    uni4 = dict(lmin=4, lmax=4, pts_q20=np.zeros((1, 3), np.uint32), radius_q20=np.zeros(0, np.uint32))
    tab = check(orc, dev, fine, uni3, 2, "levels 3-7 -> uniform 3 (injection through up to 4 levels)")
    assert (tab[:, 2] > 512).any()                     # some target block gathers from more than 8^3 leaves
    tab = check(orc, dev, uni3, uni4, 2, "uniform 3 -> uniform 4 (every block interpolated)")
    assert (tab[:, 0] == 1).all() and sorted(np.unique(tab[:, 3])) == list(range(8))
    check(orc, dev, uni4, uni3, 1, "uniform 4 -> uniform 3")


def test_regrid_of_the_largest_tree(orc, dev):
    # the moved centres of a realistic regrid of the 102,075-block tree: the pair has advanced by
    # about one finest block width along its orbit; every element is compared
    tab = check(orc, dev, sd.tree_params("C5", 1), sd.tree_params("C5", 1, phase=0.013), 2, "C5 phase 0.013")
    assert all((tab[:, 0] == k).sum() > 100 for k in (0, 1, 2))
    with pytest.raises(octfd.OctfdError) as e:         # a jump of the centres that needs two levels at once
        octfd.Transfer(octfd.Tree.build(**sd.tree_params("C4", 1)), octfd.Tree.build(**sd.tree_params("C4", 2)))
    assert e.value.status == octfd.OT_E_UNSUPPORTED


def test_refused_plan_leaves_no_device_work(dev):
    coarse = octfd.Tree.build(3, 3, np.zeros((1, 3), np.uint32), np.zeros(1, np.uint32))
    fine = octfd.Tree.build(3, 5, np.array([[1 << 19] * 3], np.uint32), np.array([60000, 40000], np.uint32))
    with pytest.raises(octfd.OctfdError):
        octfd.Transfer(coarse, fine)


def test_step_regrid_step_matches_the_oracle(orc, dev):
    """An adaptive run in miniature: one RK4 step of the 24-field system, a regrid to the tree of the
    moved centres with the state carried over, one more step; the same sequence through the oracle."""
    kind = octfd.SYN24
    pa, pb = sd.tree_params("T4", 1), sd.tree_params("T4", 1, phase=0.2)
    oa, ga = both(orc, pa)
    ob, gb = both(orc, pb)
    dt, sg = sd.time_step(5), sd.KO_SIGMA
    u = sd.make_fields("T4", oa.leaves, 1)
    want = orc.transfer(oa, ob, oa.rk4_step(kind, u.numpy(), dt, sg))
    want = ob.rk4_step(kind, want, dt, sg)
    ua = u.to(dev).clone()
    ga.rk_step(kind, ua, dt, torch.empty(ga.rk_workspace_bytes(kind) // 8, dtype=torch.float64, device=dev), sigma=sg)
    ub = torch.full((24, gb.n, 8, 8, 8), float("nan"), dtype=torch.float64, device=dev)
    octfd.Transfer(ga, gb).apply(ua, ub)
    gb.rk_step(kind, ub, dt, torch.empty(gb.rk_workspace_bytes(kind) // 8, dtype=torch.float64, device=dev), sigma=sg)
    torch.cuda.synchronize()
    got = ub.cpu().numpy()
    print("step, regrid %d -> %d blocks, step: %d of %d values differ" % (oa.n, ob.n, int((got != want).sum()), got.size), flush=True)
    assert (np.abs(got - want) <= RTOL * np.abs(want) + ATOL).all()


def test_adaptive_run_in_miniature_with_the_centred_rule(orc, dev):
    """three cycles of (two centred RK4 steps of the wave system, regrid to centres moved along the
    orbit, transfer); the whole sequence through the library and through the oracle"""
    kind = octfd.WAVE
    dt, sg = sd.time_step(5), sd.KO_SIGMA
    phases = [0.0, 0.07, 0.14, 0.21]
    trees_o = [orc.Tree.build(**sd.tree_params("T4", 1, phase=ph)) for ph in phases]
    trees_g = [octfd.Tree.build(**sd.tree_params("T4", 1, phase=ph)) for ph in phases]
    x, y, z = sd.node_coords(trees_o[0].leaves)
    u = torch.stack([torch.exp(-((x - 0.5) ** 2 + (y - 0.5) ** 2 + (z - 0.5) ** 2) / 0.02), torch.zeros_like(x)]).contiguous()
    want = u.numpy()
    got = u.to(dev)
    for c in range(3):
        to, tg = trees_o[c], trees_g[c]
        ws = torch.empty(tg.rk_centred_workspace_bytes(kind) // 8, dtype=torch.float64, device=dev)
        for _ in range(2):
            want = to.rk4_step_centred(kind, want, dt, sg)
            tg.rk_step_centred(kind, got, dt, ws, sigma=sg)
        want = orc.transfer(to, trees_o[c + 1], want)
        nxt = torch.full((2, trees_g[c + 1].n, 8, 8, 8), float("nan"), dtype=torch.float64, device=dev)
        octfd.Transfer(tg, trees_g[c + 1]).apply(got, nxt)
        got = nxt
    torch.cuda.synchronize()
    g = got.cpu().numpy()
    print("adaptive run: %d of %d values differ, max |u| %.3f" % (int((g != want).sum()), g.size, np.abs(g[0]).max()), flush=True)
    assert (np.abs(g - want) <= RTOL * np.abs(want) + ATOL).all()
    assert np.abs(g[0]).max() < 1.5
