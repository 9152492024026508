"""Parity at the benchmark's full size (the ~1e5-block, 24-field tree) in the launch configuration
bench.py times: the fused right-hand side on sampled blocks against the oracle, and rk_step against
its own definition composed from calls that are themselves checked against the oracle."""
import numpy as np
import pytest
import torch

import paper_2007_12792_amd as octfd
import synthdata as sd
from test_gpu_parity import assert_close, dev, dev_empty  # noqa: F401

pytestmark = pytest.mark.gpu


def test_config5_rhs_sampled_and_rk_step(orc, dev):  # noqa: F811
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
    sample = np.unique(np.concatenate([np.arange(0, tg.n, 20), coarse[::7], [0, tg.n - 1]]))      # one block in 20, one coarse block in 7
    u = ud.cpu().numpy()
    want = to.F(3, u, sigma=sg, blocks=sample)
    del u
    sel = torch.from_numpy(sample).to(dev)
    assert_close(k1[:, sel].cpu().numpy(), want, "C5 rhs_eval_zipped, %d sampled blocks" % sample.size)
    # rk_step == the tableau written with the library's F (checked above) and torch vector ops.
    # dt is a power of two, so u + c*k is exact-product-then-add = one fma; only the last line's
    # dt/6 is not, which costs at most one rounding of difference.
    F = lambda v, out: tg.rhs_eval_zipped(3, v, out, sigma=sg)
    k = dev_empty((24, tg.n, 8, 8, 8), dev)
    st = ud + (0.5 * dt) * k1
    acc = k1.clone()
    F(st, k); acc += 2.0 * k; st = ud + (0.5 * dt) * k
    F(st, k); acc += 2.0 * k; st = ud + dt * k
    F(st, k); acc += k
    want_u = ud + (dt / 6.0) * acc
    del st, k, k1
    ws = torch.empty(tg.rk_workspace_bytes(3) // 8, dtype=torch.float64, device=dev)
    got = ud.clone()
    tg.rk_step(3, got, dt, ws, sigma=sg)
    torch.cuda.synchronize()
    err = (got - want_u).abs()
    bound = 1e-12 * want_u.abs() + 1e-13
    print("rk_step C5: worst |diff|/bound = %.3g" % float((err / bound).max()), flush=True)
    assert bool((err <= bound).all())
    assert float((got - ud).abs().max()) > 0


def test_config5_unzip_every_block(orc, dev):  # noqa: F811
    """unzip of all 24 fields on the 102,075-block tree; three of the fields (one from each group of
    variables a workgroup fills, first, middle, last) are compared on every block, to the bit."""
    p = sd.tree_params("C5")
    to, tg = orc.Tree.build(**p), octfd.Tree.build(**p)
    ud = sd.make_fields("C5", to.leaves, device=dev)
    pd = dev_empty((24, tg.n, 14, 14, 14), dev)
    tg.unzip(ud, pd)
    torch.cuda.synchronize()
    print("unzip done", flush=True)
    for v in (0, 13, 23):
        want = to.unzip(ud[v:v + 1].cpu().numpy())
        assert torch.equal(pd[v], torch.from_numpy(want[0]).to(dev)), "field %d" % v
        print("field %d: every value equal" % v, flush=True)
    back = dev_empty((24, tg.n, 8, 8, 8), dev)
    tg.zip(pd, back)
    assert torch.equal(back, ud)


def test_centred_step_of_the_wave_system_on_the_largest_tree(orc, dev):  # noqa: F811
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


def test_tree_just_below_the_block_limit(orc, dev):  # noqa: F811
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
    del u
    assert_close(k1[:, sel].cpu().numpy(), wantk, "rhs_eval_zipped near the block limit, %d sampled blocks" % sample.size)
    # the first stage of rk_step leaves u + dt/2 k1 nowhere visible, but its result after one step must be the
    # tableau written with the library's F; dt is a power of two (see the test above)
    dt = sd.time_step(7)
    F = lambda v, out: tg.rhs_eval_zipped(1, v, out, sigma=sd.KO_SIGMA)
    k = dev_empty((2, tg.n, 8, 8, 8), dev)
    st = ud + (0.5 * dt) * k1
    acc = k1.clone()
    F(st, k); acc += 2.0 * k; st = ud + (0.5 * dt) * k
    F(st, k); acc += 2.0 * k; st = ud + dt * k
    F(st, k); acc += k
    want_u = ud + (dt / 6.0) * acc
    ws = torch.empty(tg.rk_workspace_bytes(1) // 8, dtype=torch.float64, device=dev)
    got = ud.clone()
    tg.rk_step(1, got, dt, ws, sigma=sd.KO_SIGMA)
    torch.cuda.synchronize()
    err = (got - want_u).abs()
    bound = 1e-12 * want_u.abs() + 1e-13
    print("rk_step near the block limit: worst |diff|/bound = %.3g" % float((err / bound).max()), flush=True)
    assert bool((err <= bound).all())
