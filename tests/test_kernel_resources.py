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
           os.path.join(CSRC, "kernels.hip"), "-o", os.devnull, "-Rpass-analysis=kernel-resource-usage"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    kernels, cur = {}, None
    for line in r.stderr.splitlines():
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
    """(kind, zipped input, epilogue, centred, over the schedule) -> resources, from the mangled template arguments"""
    out = {}
    for name, res in usage.items():
        m = re.search(r"k_rhsILi(\d)ELb(\d)ELi(\d)ELb(\d)ELb(\d)E", name)
        if m:
            out[tuple(int(g) for g in m.groups())] = res
    return out


def test_small_kinds_fit_four_workgroups_per_compute_unit_without_spilling(usage):
    ks = rhs_kernels(usage)
    checked = 0
    for (kind, zin, epi, centred, sched), res in ks.items():
        if kind == 3 or not zin:
            continue
        assert res["LDS Size [bytes/block]"] <= 160 * 1024 // 4, (kind, epi, centred)
        assert res["ScratchSize [bytes/lane]"] == 0 and res["VGPRs Spill"] == 0, (kind, epi, centred, res)
        assert res["VGPRs"] <= (80 if centred else 64), (kind, epi, centred)
        checked += 1
    assert checked >= 3 * 4 * 2            # three kinds, four epilogues, two ghost rules


def test_24_field_kernels_fit_two_workgroups_per_compute_unit(usage):
    ks = {k: v for k, v in rhs_kernels(usage).items() if k[0] == 3}
    assert len(ks) >= 12
    for key, res in ks.items():
        assert res["VGPRs"] + res.get("AGPRs", 0) <= 128, key
        assert res["LDS Size [bytes/block]"] <= 160 * 1024 // 2, key
        assert res["VGPRs Spill"] <= 16, (key, res)     # a handful, outside the loops; more means the body changed shape


def test_fill_kernels_fit_three_workgroups_per_compute_unit(usage):
    names = [n for n in usage if "k_unzip" in n]
    assert len(names) >= 3
    for n in names:
        assert usage[n]["LDS Size [bytes/block]"] <= 160 * 1024 // 3, n
        assert usage[n]["VGPRs Spill"] == 0, n
