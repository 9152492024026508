"""AddressSanitizer and UndefinedBehaviorSanitizer runs of the host code (the GPU side has no sanitizer here):
the library's host sources (tree engine and regrid plan) and the whole CPU oracle, each built together with a
small driver under tests/host_logic/ and run as a program of its own."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the program's own link order


def run(cmd, exe, timeout):
    cc = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert cc.returncode == 0, cc.stderr[-3000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=timeout, env=ENV)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "FAILED" not in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
    return r.stdout


def test_library_host_sources_under_asan_and_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_2007_12792_amd", "csrc")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    exe = str(tmp_path / "sanitizer_drive")
    out = run(["g++", "-std=c++17", "-O1", *SAN, "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
               "-I", os.path.join(ROOT, "include"), "-I", csrc, os.path.join(ROOT, "tests", "host_logic", "sanitizer_drive.cpp"),
               os.path.join(csrc, "octree_host.cpp"), os.path.join(csrc, "transfer_host.cpp"), "-o", exe], exe, 600)
    assert "all host checks passed" in out


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_drive")
    out = run(["gcc", "-std=c11", "-O1", *SAN, "-ffp-contract=off", "-mfma", "-fopenmp",
               os.path.join(ROOT, "tests", "host_logic", "oracle_drive.c"), os.path.join(ROOT, "oracle", "octfd_oracle.c"),
               "-o", exe, "-lm"], exe, 900)
    assert "all oracle calls ran clean" in out
