"""Parity at the benchmark's full size (the ~1e5-block, 24-field tree) in the launch configuration
bench.py times: rk_step against the oracle's step on every value, unzip of every field on every block,
the fused right-hand side on sampled blocks, and a tree just below the library's block limit."""
import numpy as np
import pytest
import torch

import paper_2007_12792_amd as octfd
import synthdata as sd
from helpers import assert_close, dev_empty

pytestmark = pytest.mark.gpu


def test_config5_rk_step_every_value(orc, dev):
    """The call the benchmark times, at its size: one rk_step of the 24-field system on the 102,075-block tree
    against the oracle's rk4_step, every one of the 1.25e9 values; and the fused right-hand side of the
    initial state against the oracle's F on one block in 20 plus one coarse block in 7.  The oracle's step holds
    five copies of the state on the host (about 60 GB with the arrays compared here)."""
    p = sd.tree_params("C5")
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    assert tg.n == 102075
    print("generating fields", flush=True)
    ud = sd.make_fields("C5", to.leaves, device=dev)
    sg, dt = sd.KO_SIGMA, sd.time_step(9)
    k1 = dev_empty((24, tg.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(3, ud, k1, sigma=sg)
    torch.cuda.synchronize()
    print("rhs done", flush=True)
    lev = to.leaves[:, 0]
    coarse = np.flatnonzero(lev < 9)
    sample = np.unique(np.concatenate([np.arange(0, tg.n, 20), coarse[::7], [0, tg.n - 1]]))
    u = ud.cpu().numpy()
    want = to.F(3, u, sigma=sg, blocks=sample)
    sel = torch.from_numpy(sample).to(dev)
    assert_close(k1[:, sel].cpu().numpy(), want, "C5 rhs_eval_zipped, %d sampled blocks" % sample.size)
    del k1, want
    ws = torch.empty(tg.rk_workspace_bytes(3) // 8, dtype=torch.float64, device=dev)
    got = ud.clone()
    tg.rk_step(3, got, dt, ws, sigma=sg)
    torch.cuda.synchronize()
    del ws
    print("rk_step done; oracle step (four evaluations of the whole tree)", flush=True)
    want_u = to.rk4_step(3, u, dt, sigma=sg)
    print("oracle step done", flush=True)
    g = got.cpu().numpy()
    # field by field, to bound the temporaries of the comparison
    for v in range(24):
        assert_close(g[v], want_u[v], "C5 rk_step, field %d" % v)
    assert np.abs(want_u[0] - u[0]).max() > 0


def test_config5_unzip_every_block(orc, dev):
    """unzip of all 24 fields on the 102,075-block tree, every padded value of every field compared to the
    bit, one field at a time (2.2 GB each) to bound the host memory."""
    p = sd.tree_params("C5")
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    ud = sd.make_fields("C5", to.leaves, device=dev)
    pd = dev_empty((24, tg.n, 14, 14, 14), dev)
    tg.unzip(ud, pd)
    torch.cuda.synchronize()
    print("unzip done", flush=True)
    for v in range(24):
        want = to.unzip(ud[v:v + 1].cpu().numpy())
        assert torch.equal(pd[v], torch.from_numpy(want[0]).to(dev)), "field %d" % v
        print("field %d: every value equal" % v, flush=True)
    back = dev_empty((24, tg.n, 8, 8, 8), dev)
    tg.zip(pd, back)
    assert torch.equal(back, ud)


def test_centred_step_of_the_wave_system_on_the_largest_tree(orc, dev):
    """rk_step_centred on the 102,075-block tree (seven levels of source leaves), two fields so that the
    oracle, which pads every block, fits in memory and finishes in seconds; every element is compared."""
    p = sd.tree_params("C5")
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    x, y, z = sd.node_coords(to.leaves)
    u = torch.stack([torch.sin(2 * np.pi * (x + 2 * y)) + 0.1 * torch.cos(6 * np.pi * z), torch.cos(2 * np.pi * (y - z))]).contiguous()
    dt = sd.time_step(9)
    print("oracle step", flush=True)
    want = to.rk4_step_centred(1, u.numpy(), dt, sd.KO_SIGMA)
    ud = u.to(dev)
    ws = torch.empty(tg.rk_centred_workspace_bytes(1) // 8, dtype=torch.float64, device=dev)
    tg.rk_step_centred(1, ud, dt, ws, sigma=sd.KO_SIGMA)
    torch.cuda.synchronize()
    assert_close(ud.cpu().numpy(), want, "C5 tree, WAVE, rk_step_centred")


def test_tree_just_below_the_block_limit(orc, dev):
    # 1,047,656 blocks, 920 short of the 2^20 the library admits: the byte offsets inside one variable's
    # zipped array reach 4.29e9, a few MB below 2^32.  Wave system, two levels with one interface.
    p = dict(lmin=6, lmax=7, pts_q20=np.array([[524288, 524288, 524288]], np.uint32), radius_q20=np.array([477800], np.uint32))
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    assert tg.n == 1047656 and to.n == tg.n
    print("trees built", flush=True)
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    ud = torch.randn((2, tg.n, 8, 8, 8), generator=g, dtype=torch.float64, device=dev)
    lev = to.leaves[:, 0]
    jumps = np.flatnonzero(np.diff(lev.astype(np.int64)) != 0)       # Morton neighbours on different levels
    sample = np.unique(np.concatenate([np.arange(0, tg.n, 26003), jumps[::4001], jumps[::4001] + 1,
                                       [0, 1, tg.n - 2, tg.n - 1]]))
    sel = torch.from_numpy(sample).to(dev)
    u = ud.cpu().numpy()
    # unzip: every value of the sampled blocks, to the bit; zip(unzip) = identity on the whole array
    pd = dev_empty((2, tg.n, 14, 14, 14), dev)
    tg.unzip(ud, pd)
    want = to.unzip(u, blocks=sample)
    assert (pd[:, sel].cpu().numpy() == want).all()
    back = dev_empty((2, tg.n, 8, 8, 8), dev)
    tg.zip(pd, back)
    assert torch.equal(back, ud)
    del pd, back
    print("unzip and zip done", flush=True)
    # fused right-hand side on the sampled blocks
    k1 = dev_empty((2, tg.n, 8, 8, 8), dev)
    tg.rhs_eval_zipped(1, ud, k1, sigma=sd.KO_SIGMA)
    wantk = to.F(1, u, sigma=sd.KO_SIGMA, blocks=sample)
    assert_close(k1[:, sel].cpu().numpy(), wantk, "rhs_eval_zipped near the block limit, %d sampled blocks" % sample.size)
    # one whole step against the oracle's, every value (the oracle holds five copies of the 8.6 GB state)
    dt = sd.time_step(7)
    ws = torch.empty(tg.rk_workspace_bytes(1) // 8, dtype=torch.float64, device=dev)
    got = ud.clone()
    tg.rk_step(1, got, dt, ws, sigma=sd.KO_SIGMA)
    torch.cuda.synchronize()
    del ws, k1
    print("rk_step done; oracle step", flush=True)
    want_u = to.rk4_step(1, u, dt, sigma=sd.KO_SIGMA)
    g = got.cpu().numpy()
    for v in range(2):
        assert_close(g[v], want_u[v], "rk_step near the block limit, field %d" % v)
