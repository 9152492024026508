"""Host-side checks of liboctfd that need no GPU: exported symbols, tree and ghost table bit-exact
against the oracle, error paths."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2007_12792_amd as octfd
import synthdata as sd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "octfd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(?:int|const char \*)\s*\**\s*(\w+)\s*\(", header))
    assert declared == set(octfd.EXPORTS)
    L = C.CDLL(octfd.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("name", ["C1", "T2", "T4", "C2", "C4", "C3", "C5"])
def test_tree_and_ghost_table_bit_exact(orc, name):
    p = sd.tree_params(name)
    a = orc.Tree.build(**p)
    b = octfd.Tree.build(**p)
    assert b.n == a.n
    assert (b.leaves == a.leaves).all()
    if a.n <= 25000:      # the oracle locates 2,744 points per block: keep the CPU suite short
        assert (b.ghost_table() == a.ghost_table()).all()


def test_ghost_table_bit_exact_on_sampled_blocks_of_the_largest_tree(orc):
    # the oracle's table is all-or-nothing, so compare through a sub-tree-independent property
    # instead: for sampled blocks of C5, every table entry must name exactly the leaves that the
    # oracle's point location finds in that part of the padded box (checked through unzip of a
    # field that stores each block's own index).
    p = sd.tree_params("C5")
    a = orc.Tree.build(**p)
    b = octfd.Tree.build(**p)
    ids = np.broadcast_to(np.arange(a.n, dtype=np.float64)[:, None, None, None], (a.n, 8, 8, 8))[None]
    sample = np.arange(0, a.n, 997)
    pad = a.unzip(ids, blocks=sample)[0]            # interpolating a constant-per-leaf field returns it
    g = b.ghost_table()[sample]
    lo = {0: (0, 3), 1: (3, 11), 2: (11, 14)}
    for s in range(sample.size):
        for d in range(27):
            rx, ry, rz = d % 3, (d // 3) % 3, d // 9
            reg = pad[s, lo[rz][0]:lo[rz][1], lo[ry][0]:lo[ry][1], lo[rx][0]:lo[rx][1]]
            found = sorted(set(np.rint(reg).astype(np.int64).ravel().tolist()))
            want = sorted(i for i in g[s, d, 1:].tolist() if i >= 0)
            assert found == want, (sample[s], d)
            lev = a.leaves[found[0], 0].astype(int) - a.leaves[sample[s], 0].astype(int)
            assert g[s, d, 0] == {0: 0, 1: 1, -1: 2}[lev]


def test_from_leaves_round_trip_and_errors(orc):
    p = sd.tree_params("T4")
    t = octfd.Tree.build(**p)
    lv = t.leaves
    rng = np.random.default_rng(0)
    again = octfd.Tree.from_leaves(lv[rng.permutation(t.n)])
    assert (again.leaves == lv).all() and (again.ghost_table() == t.ghost_table()).all()
    with pytest.raises(octfd.OctfdError) as e:
        octfd.Tree.from_leaves(lv[:-1])
    assert e.value.status == octfd.OT_E_INCOMPLETE
    with pytest.raises(octfd.OctfdError) as e:
        octfd.Tree.from_leaves(np.vstack([lv, lv[:1]]))
    assert e.value.status == octfd.OT_E_INCOMPLETE
    # replace one complete sibling octet deep inside the fine region by its parent
    fine = lv[lv[:, 0] == lv[:, 0].max()].astype(np.int64)
    S = {tuple(r) for r in lv.astype(np.int64).tolist()}
    for l, x, y, z in fine.tolist():
        if (x | y | z) & 1:
            continue
        sibs = {(l, x + (c & 1), y + ((c >> 1) & 1), z + ((c >> 2) & 1)) for c in range(8)}
        if sibs <= S:
            trial = np.array(sorted((S - sibs) | {(l - 1, x >> 1, y >> 1, z >> 1)}), dtype=np.uint32)
            try:
                orc.Tree.from_leaves(trial)
                oracle_ok = True
            except ValueError:
                oracle_ok = False
            if oracle_ok:
                octfd.Tree.from_leaves(trial)
            else:
                with pytest.raises(octfd.OctfdError) as e:
                    octfd.Tree.from_leaves(trial)
                assert e.value.status == octfd.OT_E_UNBALANCED
    # unbalanced by construction: one level-5 octet inside a level-3 tree
    base = [(3, x, y, z) for z in range(8) for y in range(8) for x in range(8) if (x, y, z) != (0, 0, 0)]
    kids4 = [(4, cx, cy, cz) for cz in range(2) for cy in range(2) for cx in range(2) if (cx, cy, cz) != (0, 0, 0)]
    kids5 = [(5, cx, cy, cz) for cz in range(2) for cy in range(2) for cx in range(2)]
    with pytest.raises(octfd.OctfdError) as e:
        octfd.Tree.from_leaves(np.array(base + kids4 + kids5, dtype=np.uint32))
    assert e.value.status == octfd.OT_E_UNBALANCED


def test_bad_arguments_are_reported_not_crashed():
    L = octfd.lib()
    assert L.octree_build(None, None) == octfd.OT_E_BADARG
    h = C.c_void_p()
    p = octfd.BuildParams(2, 3, 0, None, None, 8, 3, 1)          # lmin < 3
    assert L.octree_build(C.byref(p), C.byref(h)) == octfd.OT_E_BADARG
    p = octfd.BuildParams(3, 3, 0, None, None, 8, 2, 1)          # pad != 3
    assert L.octree_build(C.byref(p), C.byref(h)) == octfd.OT_E_UNSUPPORTED
    assert L.octree_free(None) == octfd.OT_OK
    assert L.ot_rhs_nvar_in(7) == octfd.OT_E_BADARG
    assert [octfd.nvar_in(k) for k in range(4)] == [1, 2, 1, 24]
    assert [octfd.nvar_out(k) for k in range(4)] == [4, 2, 1, 24]
    t = octfd.Tree.build(3, 3, np.zeros((0, 3), np.uint32), np.zeros(0, np.uint32))
    assert t.n == 512
    n = C.c_size_t()
    assert L.rk_workspace_bytes(t._h, octfd.DERIVS, C.byref(n)) == octfd.OT_E_UNSUPPORTED
    assert t.rk_workspace_bytes(octfd.WAVE) == 3 * 2 * 512 * 512 * 8
    assert L.unzip(t._h, 1, None, None, None) == octfd.OT_E_BADARG
    one = C.c_void_p(256)
    rp = octfd.RhsParams(0.4)
    assert L.rk_step(t._h, octfd.WAVE, C.byref(rp), 0.1, one, one, 16, None) == octfd.OT_E_WORKSPACE
    assert octfd.strerror(octfd.OT_E_WORKSPACE) == "workspace too small"
    # buffers of the stepping calls (checked before any device work): alignment, and u apart from the workspace
    need = t.rk_workspace_bytes(octfd.WAVE)
    u, ws = C.c_void_p(1 << 30), C.c_void_p(1 << 32)
    for fn in (L.rk_step, L.rk_step_centred):
        assert fn(t._h, octfd.WAVE, C.byref(rp), 0.1, C.c_void_p((1 << 30) + 4), ws, need, None) == octfd.OT_E_BADARG    # u not 8-byte aligned
        assert fn(t._h, octfd.WAVE, C.byref(rp), 0.1, u, C.c_void_p((1 << 32) + 128), need, None) == octfd.OT_E_BADARG   # workspace not 256-byte aligned
        assert fn(t._h, octfd.WAVE, C.byref(rp), 0.1, C.c_void_p((1 << 32) + need - 256), ws, need, None) == octfd.OT_E_BADARG   # u begins inside the workspace
        assert fn(t._h, octfd.WAVE, C.byref(rp), 0.1, C.c_void_p((1 << 32) - 256), ws, need, None) == octfd.OT_E_BADARG          # u ends inside it
    assert L.unzip(t._h, 1, C.c_void_p(4100), C.c_void_p(8192), None) == octfd.OT_E_BADARG
    # the static-workspace step refuses a tree whose tables are not on the device, and a step that does not fit
    assert L.rk_step_static(t._h, octfd.WAVE, C.byref(rp), 0.1, u, None) == octfd.OT_E_UNSUPPORTED
    assert L.rk_step_static(t._h, octfd.SYN24, C.byref(rp), 0.1, u, None) == octfd.OT_E_UNSUPPORTED   # 151 MB: fits, but not uploaded
    t4 = octfd.Tree.build(4, 4, np.zeros((0, 3), np.uint32), np.zeros(0, np.uint32))
    assert t4.rk_workspace_bytes(octfd.SYN24) > octfd.STATIC_WORKSPACE_BYTES
    assert L.rk_step_static(t4._h, octfd.SYN24, C.byref(rp), 0.1, u, None) == octfd.OT_E_WORKSPACE


def test_radii_beyond_the_cube_are_refused(orc):
    # R > 2^21 lattice units (twice the cube's edge) is refused by the library and by the oracle alike; 2^21 itself
    # refines everything, like any radius beyond the cube's diagonal
    pts = np.array([[5, 6, 7]], np.uint32)
    with pytest.raises(octfd.OctfdError) as e:
        octfd.Tree.build(3, 4, pts, np.array([(1 << 21) + 1], np.uint32))
    assert e.value.status == octfd.OT_E_BADARG
    with pytest.raises(ValueError):
        orc.Tree.build(3, 4, pts, np.array([(1 << 21) + 1], np.uint32))
    with pytest.raises(octfd.OctfdError):
        octfd.Tree.build(3, 4, pts, np.array([0xffffffff], np.uint32))
    a, b = octfd.Tree.build(3, 4, pts, np.array([1 << 21], np.uint32)), orc.Tree.build(3, 4, pts, np.array([1 << 21], np.uint32))
    assert a.n == 4096 and (a.leaves == b.leaves).all()


def test_device_calls_report_missing_gpu_without_crashing():
    import torch
    if torch.cuda.is_available():
        pytest.skip("only meaningful on a machine without a GPU")
    t = octfd.Tree.build(3, 3, np.zeros((0, 3), np.uint32), np.zeros(0, np.uint32))
    L = octfd.lib()
    fake = C.c_void_p(4096)
    rp = octfd.RhsParams(0.4)
    for rc in (L.unzip(t._h, 1, fake, fake, None), L.zip(t._h, 1, fake, fake, None),
               L.rhs_eval_zipped(t._h, octfd.WAVE, C.byref(rp), fake, fake, None), L.octree_upload(t._h)):
        assert rc in (octfd.OT_E_NODEVICE, octfd.OT_E_HIP)


# ---------------------------------------------------------------- regrid plan (host only)
def _containing_source(src_leaves, leaf):
    """brute force: index of the source leaf that contains the first point of `leaf`, and all source
    leaves inside `leaf` (independent of the library's merge walk)"""
    s = src_leaves.astype(np.int64)
    l, ix, iy, iz = (int(v) for v in leaf)
    down = np.maximum(l - s[:, 0], 0)
    up = np.maximum(s[:, 0] - l, 0)
    holds = (((ix >> down) << up) == s[:, 1]) & (((iy >> down) << up) == s[:, 2]) & (((iz >> down) << up) == s[:, 3])
    sh = np.maximum(s[:, 0] - l, 0)
    within = (s[:, 0] > l) & ((s[:, 1] >> sh) == ix) & ((s[:, 2] >> sh) == iy) & ((s[:, 3] >> sh) == iz)
    return np.nonzero(holds)[0], np.nonzero(within)[0]


@pytest.mark.parametrize("name,phase", [("T4", 0.35), ("T4", 0.05), ("C4", 0.0)])
def test_regrid_plan_matches_brute_force(name, phase):
    a = octfd.Tree.build(**sd.tree_params(name, 1))
    b = octfd.Tree.build(**sd.tree_params(name, 1, phase=phase)) if phase else octfd.Tree.build(**sd.tree_params(name, 2))
    la, lb = a.leaves, b.leaves
    try:
        tab = octfd.Transfer(a, b).table
    except octfd.OctfdError as e:
        # a far jump of the centres may ask for a two-level refinement: then brute force must agree
        assert e.status == octfd.OT_E_UNSUPPORTED
        assert any(la[_containing_source(la, lf)[0][0], 0] < lf[0] - 1 for lf in lb)
        return
    assert tab.shape == (b.n, 4)
    step = max(1, b.n // 400)
    for j in list(range(0, b.n, step)) + list(np.nonzero(tab[:, 0] != 0)[0][:200]):
        holds, within = _containing_source(la, lb[j])
        kind, first, count, octant = (int(v) for v in tab[j])
        if within.size:
            assert kind == 2 and first == within[0] and count == within.size and (np.diff(within) == 1).all()
        else:
            assert holds.size == 1 and first == holds[0] and count == 1
            dl = int(la[first, 0]) - int(lb[j, 0])
            assert dl in (0, -1) and kind == (0 if dl == 0 else 1)
            if kind == 1:
                assert octant == (lb[j, 1] & 1) | ((lb[j, 2] & 1) << 1) | ((lb[j, 3] & 1) << 2)
                assert tuple(lb[j, 1:] >> 1) == tuple(la[first, 1:])
    assert set(np.unique(tab[:, 0])) <= {0, 1, 2}


def test_regrid_plan_refuses_two_level_refinement_and_bad_arguments():
    coarse = octfd.Tree.build(3, 3, np.zeros((1, 3), np.uint32), np.zeros(1, np.uint32))
    fine = octfd.Tree.build(3, 5, np.array([[1 << 19] * 3], np.uint32), np.array([60000, 40000], np.uint32))
    with pytest.raises(octfd.OctfdError) as e:
        octfd.Transfer(coarse, fine)
    assert e.value.status == octfd.OT_E_UNSUPPORTED
    t = octfd.Transfer(fine, coarse)                  # coarsening by any number of levels is fine
    assert (t.table[:, 0] != 1).all() and (t.table[:, 0] == 2).any()
    L = octfd.lib()
    h = C.c_void_p()
    assert L.regrid_plan(None, coarse._h, C.byref(h)) == octfd.OT_E_BADARG
    assert L.regrid_transfer(None, 1, None, None, None) == octfd.OT_E_BADARG
    assert L.regrid_free(None) == octfd.OT_OK


def test_trees_of_a_million_blocks_are_refused_by_the_device_calls():
    # 2^21 leaves: the host tables exist, but the kernels' 32-bit offsets would not reach
    t = octfd.Tree.build(7, 7, np.zeros((1, 3), np.uint32), np.zeros(0, np.uint32))
    assert t.n == 1 << 21
    with pytest.raises(octfd.OctfdError) as e:
        t.upload()
    assert e.value.status == octfd.OT_E_UNSUPPORTED


def test_refinement_radius_is_a_strict_bound_in_the_library_too():
    # hand-counted case of tests/test_oracle_tree.py: face neighbours at distance exactly R_3 stay whole
    s = 1 << 17
    c = 4 * s + s // 2
    pt = np.array([(c, c, c)], np.uint32)
    assert octfd.Tree.build(3, 4, pt, np.array([s // 2], np.uint32)).n == 519
    assert octfd.Tree.build(3, 4, pt, np.array([s // 2 + 1], np.uint32)).n == 561


def test_zip_refuses_more_workgroups_than_a_grid_holds():
    # one workgroup per block and variable: 512 blocks x 2^23 variables would be 2^32 of them.
    # The size check precedes every device call, so the fake pointers are never touched.
    t = octfd.Tree.build(3, 3, np.zeros((0, 3), np.uint32), np.zeros(0, np.uint32))
    fake = C.c_void_p(4096)
    assert octfd.lib().zip(t._h, 1 << 23, fake, fake, None) == octfd.OT_E_UNSUPPORTED


def test_binding_rejects_wrong_shapes_and_host_tensors():
    import torch
    t = octfd.Tree.build(3, 3, np.zeros((0, 3), np.uint32), np.zeros(0, np.uint32))
    z = torch.zeros((1, t.n, 8, 8, 8), dtype=torch.float64)
    with pytest.raises(ValueError, match="padded has shape"):
        t.unzip(z, torch.zeros((1, t.n, 14, 14, 13), dtype=torch.float64))
    with pytest.raises(ValueError, match="u has shape"):
        t.rk_step(octfd.WAVE, z, 1e-3, z)
    # a host tensor of the right shape is not computed on: there is no CPU path
    with pytest.raises(ValueError, match="CUDA tensor"):
        t.unzip(z, torch.zeros((1, t.n, 14, 14, 14), dtype=torch.float64))


def test_header_is_valid_c_and_a_c_program_can_use_the_library(tmp_path):
    # the boundary is a C ABI: compile a C11 client against include/octfd.h with gcc (not hipcc, not C++),
    # link it to the built library and run the host-only calls
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "host_calls")
    libdir = os.path.dirname(octfd.LIB_PATH)
    cc = subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(root, "include"),
                         os.path.join(root, "tests", "c_abi", "host_calls.c"), "-o", exe, "-L", libdir, "-loctfd",
                         "-Wl,-rpath," + libdir], capture_output=True, text=True, timeout=120)
    assert cc.returncode == 0, cc.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert r.stdout.strip() == "blocks 519 fine 8 copies 519 self 0"


def test_source_lists_virtual_blocks_and_pairs_of_the_host_tree(tmp_path):
    # internal host tables that no C-ABI call returns: checked by a small C++ program built with g++ from the
    # library's host source (see tests/host_logic/tables_check.cpp for what it asserts)
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2007_12792_amd", "csrc")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    exe = str(tmp_path / "tables_check")
    cc = subprocess.run(["g++", "-std=c++17", "-O1", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
                         "-I", os.path.join(root, "include"), "-I", csrc,
                         os.path.join(root, "tests", "host_logic", "tables_check.cpp"), os.path.join(csrc, "octree_host.cpp"),
                         "-o", exe], capture_output=True, text=True, timeout=300)
    assert cc.returncode == 0, cc.stderr[-2000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    assert "FAILED" not in r.stdout and sum(line.startswith("blocks ") for line in r.stdout.splitlines()) == 3, r.stdout


def test_bench_refuses_more_than_one_gpu_and_a_missing_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr
    import torch
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "1"], capture_output=True, text=True, timeout=300)
        assert r.returncode != 0 and "no GPU" in r.stderr and "{" not in r.stdout
