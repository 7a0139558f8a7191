"""GPU parity of the further wire types (fp64, int64, uint8): every collective,
both schedules, every operator, tree order -- bit for bit against the oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import (CODE, assert_same_bits, device_inputs, fresh, run_all_gather, run_allreduce, run_alltoall,
                      run_broadcast, run_reduce, run_reduce_scatter)
from oracle import ring_oracle as orc
from paper_2601_22585_amd import hcl

pytestmark = pytest.mark.gpu

OPS = {"sum": orc.SUM, "prod": orc.PROD, "max": orc.MAX, "min": orc.MIN}
DIST = {"fp64": ("normal", 0.0, 1.0), "int64": ("randint", -10**12, 10**12), "uint8": ("randint", 0, 255)}
TYPES = ["fp64", "int64", "uint8"]


@pytest.mark.parametrize("sched", ["stepwise", "fused"])
@pytest.mark.parametrize("dtype", TYPES)
def test_allreduce_sum_shapes(dtype, sched):
    for k, (W, count, ring, chunk, mis) in enumerate([(2, 10_001, None, 0, 0), (3, 262_147, [2, 0, 1], 4096, 1),
                                                      (8, 1_000_003, None, 64 * 1024, 0), (16, 300_001, None, 32 * 1024, 0),
                                                      (4, 3, None, 0, 0), (5, 65_536, [4, 2, 0, 3, 1], 0, 3)]):
        run_allreduce(1000 + k, W, count, dtype, DIST[dtype], ring=ring, chunk_bytes=chunk, misalign=mis, sched=sched)
    run_allreduce(1010, 8, 500_000, dtype, DIST[dtype], inplace=True, chunk_bytes=65536, sched=sched)
    if sched == "stepwise":
        run_allreduce(1011, 8, 500_000, dtype, DIST[dtype], chunk_bytes=65536, fuse_rs_ag=True)
        run_allreduce(1012, 4, 200_000, dtype, DIST[dtype], xport="host_staged")


@pytest.mark.parametrize("sched", ["stepwise", "fused"])
@pytest.mark.parametrize("dtype", TYPES)
def test_other_collectives(dtype, sched):
    run_reduce_scatter(1020, 8, 40_001, dtype, DIST[dtype], chunk_bytes=8192, sched=sched)
    run_reduce_scatter(1021, 4, 65_536, dtype, DIST[dtype], ring=[1, 3, 0, 2], inplace=True, sched=sched)
    run_all_gather(1022, 8, 40_001, dtype, DIST[dtype], chunk_bytes=8192, sched=sched)
    run_all_gather(1023, 4, 65_536, dtype, DIST[dtype], inplace=True, sched=sched)
    run_reduce(1024, 8, 300_001, dtype, DIST[dtype], 5, sched=sched)
    run_broadcast(1025, 8, 300_001, dtype, DIST[dtype], 2, sched=sched)
    run_alltoall(1026, 8, 20_001, dtype, DIST[dtype], sched=sched)


@pytest.mark.parametrize("sched", ["stepwise", "fused"])
@pytest.mark.parametrize("dtype", TYPES)
@pytest.mark.parametrize("op", ["prod", "max", "min"])
def test_operators(op, dtype, sched):
    dists = [DIST[dtype], ("bits",)] if dtype != "uint8" else [DIST[dtype]]
    for k, (W, count, ring, chunk) in enumerate([(3, 262_147, [2, 0, 1], 4096), (8, 1_000_003, None, 64 * 1024),
                                                 (16, 100_001, None, 0)]):
        for d, dist in enumerate(dists):
            mis = (k + d) & 1
            cpu, dev = device_inputs(1040 + 10 * k + d, W, count, dtype, dist, mis)
            es = wl.ESIZE[dtype]
            want = orc.allreduce([wl.to_wire(t) for t in cpu], CODE[dtype], ring=ring, chunk_elems=chunk // es, op=OPS[op])
            recv = fresh(W, count, dtype, mis, fill=0)
            hcl.allreduce_sim(dev, recv, chunk_bytes=chunk, ring=ring, sched=sched, op=op)
            torch.cuda.synchronize()
            for r in range(W):
                assert_same_bits(recv[r], want[r], dtype, f"allreduce {op} {sched} W={W} {dtype} {dist[0]} mis={mis} rank {r}")


@pytest.mark.parametrize("dtype", TYPES)
def test_tree_order(dtype):
    for k, (W, count, ring) in enumerate([(5, 65_537, [4, 2, 0, 3, 1]), (8, 500_000, None), (13, 130_001, None)]):
        for op in ("sum", "prod", "max"):
            cpu, dev = device_inputs(1080 + k, W, count, dtype, DIST[dtype], k & 1)
            want = orc.allreduce_var([wl.to_wire(t) for t in cpu], CODE[dtype], op=OPS[op], ring=ring, order=orc.ORDER_TREE)
            for acc in ("per_hop", "fp32"):       # the same result: these types are their own accumulation type
                recv = fresh(W, count, dtype, k & 1, fill=0)
                hcl.allreduce_sim(dev, recv, ring=ring, sched="fused", order="tree", op=op, accumulate=acc)
                torch.cuda.synchronize()
                for r in range(W):
                    assert_same_bits(recv[r], want[r], dtype, f"tree {op} {acc} W={W} {dtype} rank {r}")


def test_fp64_cancellation_example_and_uint8_wrap():
    M = 2.0 ** 53
    dev = [torch.full((64,), v, dtype=torch.float64, device="cuda") for v in (M, 1.0, -M, 1.0)]
    for sched in ("stepwise", "fused"):
        recv = fresh(4, 64, "fp64", fill=0)
        hcl.allreduce_sim(dev, recv, sched=sched)
        torch.cuda.synchronize()
        want = torch.tensor([2.0, 2.0, 0.0, 1.0], dtype=torch.float64).repeat_interleave(16)
        for r in range(4):
            assert torch.equal(recv[r].cpu(), want)
    d8 = [torch.full((1000,), 200, dtype=torch.uint8, device="cuda") for _ in range(3)]
    out = fresh(3, 1000, "uint8", fill=0)
    hcl.allreduce_sim(d8, out)
    torch.cuda.synchronize()
    assert torch.equal(out[1].cpu(), torch.full((1000,), 600 % 256, dtype=torch.uint8))
