"""rk_step_static (the entry point for callers that cannot allocate: its workspace is a static device array
of the library) against rk_step, through the C ABI: same results to the bit, on two calls in a row on the
same GPU, the second on a smaller input, and the documented refusals."""
import numpy as np
import pytest
import torch

import paper_2007_12792_amd as octfd
import synthdata as sd

pytestmark = pytest.mark.gpu


def test_static_workspace_step_equals_rk_step(dev):
    cases = [("T3", octfd.WAVE), ("C1", octfd.BURGERS)]      # 2 fields on ~800 blocks, then 1 field on 512
    sizes = []
    for name, kind in cases:
        t = octfd.Tree.build(**sd.tree_params(name))
        nv = octfd.nvar_in(kind)
        u = torch.from_numpy(np.random.default_rng(7).standard_normal((nv, t.n, 8, 8, 8))).to(dev)
        dt = sd.time_step(sd.CONFIGS[name]["lmax"])
        need = t.rk_workspace_bytes(kind)
        assert need <= octfd.STATIC_WORKSPACE_BYTES
        sizes.append(need)
        a, b = u.clone(), u.clone()
        with pytest.raises(octfd.OctfdError) as e:           # tables not on the device yet: refused, nothing allocated
            t.rk_step_static(kind, b, dt, sigma=sd.KO_SIGMA)
        assert e.value.status == octfd.OT_E_UNSUPPORTED and torch.equal(b, u)
        t.upload()
        ws = torch.empty(need // 8, dtype=torch.float64, device=dev)
        for _ in range(2):                                   # two steps each, so that the second reads what the first left
            t.rk_step(kind, a, dt, ws, sigma=sd.KO_SIGMA)
            t.rk_step_static(kind, b, dt, sigma=sd.KO_SIGMA)
        torch.cuda.synchronize()
        assert torch.isfinite(a).all() and not torch.equal(a, u)
        assert torch.equal(a, b), name
        print("%s: rk_step_static == rk_step on every value (%d blocks, workspace %d bytes)" % (name, t.n, need), flush=True)
    assert sizes[1] < sizes[0]


def test_static_workspace_limit(dev):
    t = octfd.Tree.build(**sd.tree_params("T4"))             # 24 fields on 792 blocks need 234 MB
    t.upload()
    assert t.rk_workspace_bytes(octfd.SYN24) > octfd.STATIC_WORKSPACE_BYTES
    u = torch.zeros((24, t.n, 8, 8, 8), dtype=torch.float64, device=dev)
    with pytest.raises(octfd.OctfdError) as e:
        t.rk_step_static(octfd.SYN24, u, 1e-3)
    assert e.value.status == octfd.OT_E_WORKSPACE
