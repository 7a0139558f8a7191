"""Host-side logic under AddressSanitizer and UBSan, without a GPU.

host_check: the library's whole host side (validation, ring chunk scheduler, launch
plans, the fork / join of the second stream) compiled with g++ against recording
stand-ins for the HIP runtime and the kernel launchers, its launch plans executed on
symbolic memory (tests/host/host_check.cpp says what that proves).
oracle_check: the CPU oracle driven with exact-size heap buffers.
Both are built here with -fsanitize=address,undefined and must exit 0 with no report."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST = os.path.join(ROOT, "tests", "host")
OUT = os.path.join(HOST, "_build")
CSRC = os.path.join(ROOT, "paper_2601_22585_amd", "csrc")
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)    # the sanitizer runtime must come first in the link order of a fresh process
ENV.pop("HCL_DEBUG", None)


def _build_host_check():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "host_check")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    subprocess.check_call(["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
                           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", HOST,
                           os.path.join(CSRC, "hcl_api.cpp"), os.path.join(HOST, "hip_stub.cpp"),
                           os.path.join(HOST, "host_check.cpp"), "-o", exe])
    return exe


@pytest.fixture(scope="module")
def host_check():
    return _build_host_check()


def test_host_side_of_the_library_under_sanitizers(host_check):
    r = subprocess.run([host_check], capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "host_check: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]


def test_debug_dump_lists_the_work_items_of_the_call(host_check):
    """HCL_DEBUG=1: the call's arguments and, per ring step, one line per work item."""
    r = subprocess.run([host_check, "dump"], capture_output=True, text=True, env=ENV, timeout=120)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    lines = [ln for ln in r.stderr.splitlines() if ln.startswith("hcl:")]
    assert lines[0].startswith("hcl: all-reduce W=4 elements=10 dtype=fp32 op=sum chunk_bytes=8 sched=stepwise xport=direct")
    assert "ring=[2 0 3 1]" in lines[0]
    steps = [ln for ln in lines if re.match(r"hcl:  (reduce-scatter|all-gather) step \d+: \d+ work items", ln)]
    assert len(steps) == 2 * 3                                   # W - 1 steps per phase
    items = [ln for ln in lines if ln.startswith("hcl:   rank ")]
    assert len(items) == sum(int(re.search(r": (\d+) work items", ln).group(1)) for ln in steps)
    # 10 elements in blocks of 3, 3, 3, 1 and chunks of 2 elements
    for ln in items:
        lo, hi = map(int, re.search(r"elements \[(\d+), (\d+)\)", ln).groups())
        assert 0 <= lo < hi <= 10 and hi - lo <= 2
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr


def test_oracle_under_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_check")
    subprocess.check_call(["gcc", "-std=gnu11", *SAN, "-fopenmp", "-ffp-contract=off",
                           os.path.join(ROOT, "oracle", "ring_oracle.c"), os.path.join(HOST, "oracle_check.c"),
                           "-o", exe, "-lm"])
    r = subprocess.run([exe], capture_output=True, text=True, env=dict(ENV, OMP_NUM_THREADS="4"), timeout=600)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "oracle_check: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
