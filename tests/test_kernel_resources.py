"""Resource limits that the kernels' speed depends on, read from the compiler's own report (no GPU needed).

The right-hand-side kernels of the kinds other than the 24-field system are compiled for 64 registers and 40 KB of LDS
so that four workgroups share a compute unit; at that occupancy a kernel that spills even a few registers was measured
a quarter slower.  The 24-field kernels need 128 registers and half the LDS of a compute unit.  A change that breaks one
of these silently costs tens of per cent, so the build is checked here.
"""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2007_12792_amd", "csrc")


@pytest.fixture(scope="module")
def usage():
    hipcc = os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "bin", "hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-x", "hip", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only", "-c",
           "-o", os.devnull, "-Rpass-analysis=kernel-resource-usage"]
    kernels, cur, lines = {}, None, []
    for src in ("kernels.hip", "pair.hip"):
        r = subprocess.run(cmd + [os.path.join(CSRC, src)], capture_output=True, text=True, timeout=900)
        assert r.returncode == 0, r.stderr[-2000:]
        lines += r.stderr.splitlines()
    for line in lines:
        m = re.search(r"remark:\s+(.*?)\s+\[-Rpass", line)
        if not m:
            continue
        key, _, val = m.group(1).partition(":")
        key, val = key.strip(), val.strip()
        if key == "Function Name":
            cur = kernels.setdefault(val, {})
        elif cur is not None and val.isdigit():
            cur[key] = int(val)
    assert kernels
    return kernels


def rhs_kernels(usage):
    """(kind, zipped input, epilogue) -> resources, from the mangled template arguments"""
    out = {}
    for name, res in usage.items():
        m = re.search(r"k_rhsILi(\d)ELb(\d)ELi(\d)EEE", name)
        if m:
            out[tuple(int(g) for g in m.groups())] = res
    return out


def test_small_kinds_fit_four_workgroups_per_compute_unit_without_spilling(usage):
    ks = rhs_kernels(usage)
    checked = 0
    for (kind, zin, epi), res in ks.items():
        if kind == 3 or not zin:
            continue
        assert res["LDS Size [bytes/block]"] <= 160 * 1024 // 4, (kind, epi)
        assert res["ScratchSize [bytes/lane]"] == 0 and res["VGPRs Spill"] == 0, (kind, epi, res)
        assert res["VGPRs"] <= 64, (kind, epi)
        checked += 1
    assert checked >= 3 * 4                # three kinds, four epilogues


def test_24_field_kernels_fit_two_workgroups_per_compute_unit(usage):
    ks = {k: v for k, v in rhs_kernels(usage).items() if k[0] == 3}      # padded input only: zipped input runs k_rhs_pair
    assert len(ks) == 5
    for key, res in ks.items():
        assert res["VGPRs"] + res.get("AGPRs", 0) <= 128, key
        assert res["LDS Size [bytes/block]"] <= 160 * 1024 // 2, key
        assert res["VGPRs Spill"] == 0 and res["ScratchSize [bytes/lane]"] == 0, (key, res)   # no interpolation code left in them


def test_two_block_kernel_fits_one_compute_unit(usage):
    """k_rhs_pair: 1,024 threads, so 128 registers at most, and all its LDS from one compute unit's 160 KB"""
    names = [n for n in usage if "k_rhs_pair" in n]
    assert len(names) == 4
    for n in names:
        assert usage[n]["VGPRs"] + usage[n].get("AGPRs", 0) <= 128, n
        assert usage[n]["LDS Size [bytes/block]"] <= 160 * 1024, n
        assert usage[n]["VGPRs Spill"] == 0 and usage[n]["ScratchSize [bytes/lane]"] == 0, (n, usage[n])


def test_fill_kernels_fit_three_workgroups_per_compute_unit(usage):
    names = [n for n in usage if "k_unzip" in n or "k_virtual" in n]
    assert len(names) == 3
    for n in names:
        assert usage[n]["LDS Size [bytes/block]"] <= 160 * 1024 // 3, n
        assert usage[n]["VGPRs Spill"] == 0, n
