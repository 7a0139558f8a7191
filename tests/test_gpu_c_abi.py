"""The C ABI driven from a plain C program (no binding, no Python in the call path):
paper_2601_22585_amd/examples/allreduce_from_file.c reads rank buffers from a file, runs
the ring All-Reduce in three schedules through include/hcl.h and writes every rank's
result to a file, which is compared with the CPU oracle bit for bit."""
import os
import subprocess

import numpy as np
import pytest

import workloads as wl
from oracle import ring_oracle as orc
from paper_2601_22585_amd import build as hcl_build

pytestmark = pytest.mark.gpu

EXE = os.path.join(hcl_build.HERE, "examples", "allreduce_from_file")


@pytest.fixture(scope="module")
def exe():
    if not os.path.exists(EXE):
        hcl_build.build_examples()
    return EXE


@pytest.mark.parametrize("W,count,dtype,dist,chunk_bytes", [
    (8, 1_000_003, "bf16", ("normal", 0.0, 1e-3), 64 * 1024),
    (4, 262_144, "fp32", ("uniform", -1.0, 1.0), 262_144),
    (5, 70_001, "int32", ("randint", -1000, 1000), 0),
    (16, 300_007, "fp16", ("normal", 0.0, 1.0), 2 * 4099),
])
def test_allreduce_through_the_c_program(exe, tmp_path, W, count, dtype, dist, chunk_bytes):
    cpu = [wl.to_wire(t) for t in wl.make_inputs(950, W, count, dtype, dist)]
    fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(fin, "wb") as f:
        for a in cpu:
            f.write(a.tobytes())
    r = subprocess.run([exe, str(W), str(count), str(wl.DTYPE_CODE[dtype]), str(chunk_bytes), str(fin), str(fout)],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    want = orc.allreduce(cpu, wl.DTYPE_CODE[dtype], chunk_elems=chunk_bytes // wl.ESIZE[dtype])
    got = np.fromfile(fout, dtype=cpu[0].dtype)
    assert got.size == 3 * W * count
    got = got.reshape(3, W, count)
    for v, name in enumerate(("stepwise", "stepwise in place, fused last step", "fused")):
        for r_ in range(W):
            eq = wl.bits_equal_nan_aware(got[v, r_], want[r_], dtype)
            assert eq.all(), f"{name}: rank {r_}: {int((~eq).sum())} elements differ from the oracle"
