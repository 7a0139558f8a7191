"""GPU parity of Reduce, Broadcast and All-to-All against the CPU oracle, bit for bit."""
import pytest
import torch

import workloads as wl
from gpu_util import run_alltoall, run_broadcast, run_reduce
from paper_2601_22585_amd import hcl

pytestmark = pytest.mark.gpu

DIST = {"fp32": ("uniform", -1.0, 1.0), "bf16": ("normal", 0.0, 1e-3), "fp16": ("normal", 0.0, 1.0),
        "int32": ("randint", -1000, 1000)}
DTYPES = ["fp32", "bf16", "fp16", "int32"]
CASES = [(1, 1000, None, 0), (2, 10_001, None, 0), (3, 262_147, [2, 0, 1], 4096), (8, 1_000_003, None, 64 * 1024),
         (8, 524_288, [7, 2, 5, 0, 3, 6, 1, 4], 0), (16, 300_001, None, 32 * 1024)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("sched", ["stepwise", "fused"])
def test_reduce(dtype, sched):
    for k, (W, count, ring, chunk) in enumerate(CASES):
        for root in sorted({0, W - 1, W // 2}):
            for inplace in (False, True):
                n = run_reduce(800 + k, W, count, dtype, DIST[dtype], root, ring=ring, chunk_bytes=chunk,
                               inplace=inplace, sched=sched)
                if W > 1:
                    assert n == (W - 1 if sched == "stepwise" else 1)
    run_reduce(820, 4, 50_001, dtype, DIST[dtype], 2, misalign=1, sched=sched)
    run_reduce(821, 4, 5, dtype, DIST[dtype], 1, sched=sched)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("sched", ["stepwise", "fused"])
def test_broadcast(dtype, sched):
    for k, (W, count, ring, chunk) in enumerate(CASES):
        for root in sorted({0, W - 1}):
            for inplace in (False, True):
                run_broadcast(830 + k, W, count, dtype, DIST[dtype], root, ring=ring, chunk_bytes=chunk,
                              inplace=inplace, sched=sched)
    run_broadcast(840, 4, 50_001, dtype, DIST[dtype], 3, misalign=1, sched=sched)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("sched", ["stepwise", "fused"])
def test_alltoall(dtype, sched):
    for k, (W, count, ring, chunk) in enumerate(CASES):
        n = max(1, count // W)
        nl = run_alltoall(850 + k, W, n, dtype, DIST[dtype], ring=ring, chunk_bytes=chunk, sched=sched)
        assert nl == (W if sched == "stepwise" else -(-W // (32 // W)))
    run_alltoall(860, 4, 12_501, dtype, DIST[dtype], misalign=1, sched=sched)


def test_other_collectives_reject_bad_calls():
    W, n = 4, 64
    bufs = [torch.zeros(W * n, dtype=torch.float32, device="cuda") for _ in range(W)]
    outs = [torch.zeros(W * n, dtype=torch.float32, device="cuda") for _ in range(W)]
    with pytest.raises(hcl.HclError, match="ALIAS"):
        hcl.alltoall_sim(bufs, bufs)
    with pytest.raises(hcl.HclError, match="WORKSPACE"):
        hcl.reduce_sim(bufs, outs, 0)
    with pytest.raises(hcl.HclError, match="INVALID_ARG"):
        hcl.reduce_sim(bufs, outs, 4, sched="fused")
    with pytest.raises(hcl.HclError, match="UNSUPPORTED"):
        hcl.broadcast_sim(bufs, outs, 0, xport="host_staged", host_stage=torch.empty(1 << 20, dtype=torch.uint8, pin_memory=True))
    with pytest.raises(hcl.HclError, match="ALIAS"):
        hcl.broadcast_sim([bufs[0], None, None, None], [outs[0], bufs[0], outs[2], outs[3]], 0)
