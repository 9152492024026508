"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element.

Tolerance (fp64 values): |gpu - oracle| <= 1e-12 |oracle| + 1e-13.  Both sides execute the same
IEEE operation sequence, so the observed distance is normally 0; the worst distance is printed.
Integer work (tree, ghost table) is compared bit-exactly in test_library_host.py.
"""
import numpy as np
import pytest
import torch

import paper_2007_12792_amd as octfd
import synthdata as sd
from helpers import KIND, assert_close, dev_empty, trees

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,nvar", [("C1", 1), ("T2", 1), ("T4", 2), ("T4", 3), ("T3", 5), ("T4", 7), ("T4", 8), ("T2", 13)])
def test_unzip_and_zip(orc, dev, name, nvar):
    to, tg = trees(orc, name)
    rng = np.random.default_rng(21)
    z = rng.standard_normal((nvar, to.n, 8, 8, 8))
    zd = torch.from_numpy(z).to(dev)
    pd = dev_empty((nvar, to.n, 14, 14, 14), dev)
    tg.unzip(zd, pd)
    want = to.unzip(z)
    got = pd.cpu().numpy()
    assert_close(got, want, "unzip " + name)
    assert (got == want).all()                       # copies, injections and fma chains: bit-exact
    back = dev_empty((nvar, to.n, 8, 8, 8), dev)
    tg.zip(pd, back)
    assert (back.cpu().numpy() == z).all()


@pytest.mark.parametrize("name", ["T2", "T3", "T3B", "T4"])
def test_three_call_pipeline_and_fused_call(orc, dev, name):
    cfg = sd.CONFIGS[name]
    kind = KIND[cfg["kind"]]
    to, tg = trees(orc, name)
    u = sd.make_fields(name, to.leaves).numpy()
    if name == "T3":
        u[1] = 0.3 * np.random.default_rng(22).standard_normal(u[1].shape)
    sig = 0.0 if kind == 0 else sd.KO_SIGMA
    want = to.F(kind, u, sigma=sig)
    ud = torch.from_numpy(u).to(dev)
    vi, vo = octfd.nvar_in(kind), octfd.nvar_out(kind)
    # literal pipeline
    pd = dev_empty((vi, to.n, 14, 14, 14), dev)
    rd = dev_empty((vo, to.n, 14, 14, 14), dev)
    zd = dev_empty((vo, to.n, 8, 8, 8), dev)
    tg.unzip(ud, pd)
    tg.rhs_eval(kind, pd, rd, sigma=sig)
    tg.zip(rd, zd)
    lit = zd.cpu().numpy()
    assert_close(lit, want, "unzip->rhs_eval->zip " + name)
    # rhs_eval on the oracle's own padded input, compared on the padded-shaped output
    pin = to.unzip(u)
    rd2 = dev_empty((vo, to.n, 14, 14, 14), dev)
    tg.rhs_eval(kind, torch.from_numpy(pin).to(dev), rd2, sigma=sig)
    wantp = to.rhs(kind, pin, sigma=sig)
    assert_close(rd2[:, :, 3:11, 3:11, 3:11].cpu().numpy(), wantp[:, :, 3:11, 3:11, 3:11], "rhs_eval " + name)
    assert torch.isnan(rd2[:, :, 0:3]).all()         # ghost layers of the output are left untouched
    # fused
    fd = dev_empty((vo, to.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(kind, ud, fd, sigma=sig)
    fused = fd.cpu().numpy()
    assert_close(fused, want, "rhs_eval_zipped " + name)
    assert (fused == lit).all()                      # fusion changes no bit


@pytest.mark.parametrize("name", ["T3", "T3B", "T4"])
def test_rk_step(orc, dev, name):
    cfg = sd.CONFIGS[name]
    kind = KIND[cfg["kind"]]
    to, tg = trees(orc, name)
    u = sd.make_fields(name, to.leaves).numpy()
    dt = sd.time_step(cfg["lmax"])
    want = to.rk4_step(kind, u, dt, sigma=sd.KO_SIGMA)
    ud = torch.from_numpy(u).to(dev)
    ws = torch.empty(tg.rk_workspace_bytes(kind) // 8, dtype=torch.float64, device=dev)
    tg.rk_step(kind, ud, dt, ws, sigma=sd.KO_SIGMA)
    assert_close(ud.cpu().numpy(), want, "rk_step " + name)
    assert np.abs(want - u).max() > 0
    # a second step from the updated state, same workspace (stale contents must not matter)
    want2 = to.rk4_step(kind, want, dt, sigma=sd.KO_SIGMA)
    tg.rk_step(kind, ud, dt, ws, sigma=sd.KO_SIGMA)
    assert_close(ud.cpu().numpy(), want2, "rk_step #2 " + name)


def test_rk_step_rejects_short_or_misaligned_workspace(dev):
    tg = octfd.Tree.build(**sd.tree_params("T3"))
    u = torch.zeros((2, tg.n, 8, 8, 8), dtype=torch.float64, device=dev)
    ws = torch.empty(tg.rk_workspace_bytes(1) // 8 + 64, dtype=torch.float64, device=dev)
    with pytest.raises(octfd.OctfdError) as e:
        tg.rk_step(1, u, 1e-3, ws[:100])
    assert e.value.status == octfd.OT_E_WORKSPACE
    with pytest.raises(octfd.OctfdError) as e:
        tg.rk_step(1, u, 1e-3, ws[1:])
    assert e.value.status == octfd.OT_E_BADARG


def test_results_do_not_depend_on_run_or_stream(orc, dev):
    to, tg = trees(orc, "T4")
    u = torch.from_numpy(sd.make_fields("T4", to.leaves).numpy()).to(dev)
    a = dev_empty((24, to.n, 8, 8, 8), dev)
    b = dev_empty((24, to.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(3, u, a, sigma=0.4)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        tg.rhs_eval_zipped(3, u, b, sigma=0.4, stream=s)
    s.synchronize()
    assert torch.equal(a, b)


def test_config2_full_parity(orc, dev):
    to, tg = trees(orc, "C2")
    u = sd.make_fields("C2", to.leaves).numpy()
    want = to.F(0, u)
    fd = dev_empty((4, to.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(0, torch.from_numpy(u).to(dev), fd)
    assert_close(fd.cpu().numpy(), want, "C2 DERIVS")


def test_config4_full_parity(orc, dev):
    # the 21,064-block tree, 24 fields: every value of the fused right-hand side and of one whole step
    to, tg = trees(orc, "C4")
    ud = sd.make_fields("C4", to.leaves, device=dev)
    u = ud.cpu().numpy()
    fd = dev_empty((24, to.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(3, ud, fd, sigma=sd.KO_SIGMA)
    assert_close(fd.cpu().numpy(), to.F(3, u, sigma=sd.KO_SIGMA), "C4 SYN24 rhs_eval_zipped, every block")
    dt = sd.time_step(7)
    ws = torch.empty(tg.rk_workspace_bytes(3) // 8, dtype=torch.float64, device=dev)
    tg.rk_step(3, ud, dt, ws, sigma=sd.KO_SIGMA)
    assert_close(ud.cpu().numpy(), to.rk4_step(3, u, dt, sigma=sd.KO_SIGMA), "C4 SYN24 rk_step, every value")


@pytest.mark.parametrize("name", ["C3", "C3B"])
def test_config3_rk_step_full_parity(orc, dev, name):
    # the 47,783-block tree, wave system and Burgers equation: every value of one whole step
    cfg = sd.CONFIGS[name]
    kind = KIND[cfg["kind"]]
    to, tg = trees(orc, name)
    u = sd.make_fields(name, to.leaves).numpy()
    dt = sd.time_step(cfg["lmax"])
    want = to.rk4_step(kind, u, dt, sigma=sd.KO_SIGMA)
    ud = torch.from_numpy(u).to(dev)
    ws = torch.empty(tg.rk_workspace_bytes(kind) // 8, dtype=torch.float64, device=dev)
    tg.rk_step(kind, ud, dt, ws, sigma=sd.KO_SIGMA)
    assert_close(ud.cpu().numpy(), want, "rk_step " + name)
    assert np.abs(want - u).max() > 0
