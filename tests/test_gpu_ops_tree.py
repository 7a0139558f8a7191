"""GPU parity of the other reduction operators (product, maximum, minimum) on
both schedules, and of the tree-order variants of the fused schedule: every
output element against the oracle's bits (any NaN equals any NaN)."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import CODE, assert_same_bits, device_inputs, fresh, pinned_stage
from oracle import ring_oracle as orc
from paper_2601_22585_amd import hcl

pytestmark = pytest.mark.gpu

OPS = {"prod": orc.PROD, "max": orc.MAX, "min": orc.MIN, "sum": orc.SUM}
# value inputs, and raw bit patterns (NaNs, infinities, subnormals, both zeros) for the float types
DISTS = {"fp32": [("uniform", -2.0, 2.0), ("bits",)], "bf16": [("normal", 0.0, 1.0), ("bits",)],
         "fp16": [("normal", 0.0, 1.0), ("bits",)], "int32": [("randint", -1000, 1000), ("randint", -2**31, 2**31 - 1)]}
CASES = [(2, 10_001, None, 0), (3, 262_147, [2, 0, 1], 4096), (8, 1_000_003, None, 64 * 1024),
         (5, 65_536, [4, 2, 0, 3, 1], 0), (16, 300_001, None, 32 * 1024)]


@pytest.mark.parametrize("sched", ["stepwise", "fused"])
@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32", "int32"])
@pytest.mark.parametrize("op", ["prod", "max", "min"])
def test_allreduce_with_operator_bit_exact(op, dtype, sched):
    for k, (W, count, ring, chunk) in enumerate(CASES):
        for d, dist in enumerate(DISTS[dtype]):
            mis = (k + d) & 1
            cpu, dev = device_inputs(700 + 10 * k + d, W, count, dtype, dist, mis)
            es = wl.ESIZE[dtype]
            want = orc.allreduce([wl.to_wire(t) for t in cpu], CODE[dtype], ring=ring, chunk_elems=chunk // es, op=OPS[op])
            recv = fresh(W, count, dtype, mis, fill=0)
            n = hcl.allreduce_sim(dev, recv, chunk_bytes=chunk, ring=ring, sched=sched, op=op)
            torch.cuda.synchronize()
            assert n == (1 if sched == "fused" else 2 * (W - 1))
            for r in range(W):
                assert_same_bits(recv[r], want[r], dtype, f"allreduce {op} {sched} W={W} count={count} {dtype} {dist[0]} mis={mis} rank {r}")
                assert_same_bits(dev[r], wl.to_wire(cpu[r]), dtype, "send must stay untouched")


@pytest.mark.parametrize("sched", ["stepwise", "fused"])
@pytest.mark.parametrize("dtype", ["bf16", "fp32", "int32"])
def test_reduce_scatter_and_reduce_with_operator(dtype, sched):
    for op in ("prod", "max", "min"):
        for k, (W, n, ring, chunk) in enumerate([(4, 50_001, [1, 3, 0, 2], 8192), (8, 131_072, None, 0)]):
            cpu, dev = device_inputs(760 + k, W, W * n, dtype, DISTS[dtype][k % 2])
            wire = [wl.to_wire(t) for t in cpu]
            es = wl.ESIZE[dtype]
            want = orc.reduce_scatter(wire, CODE[dtype], ring=ring, chunk_elems=chunk // es, op=OPS[op])
            shard = fresh(W, n, dtype, fill=0)
            opt = {}
            wsb = hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, W, n, CODE[dtype], chunk, sched=sched)
            if wsb:
                opt["workspace"] = torch.empty(wsb, dtype=torch.uint8, device="cuda")
            hcl.reduce_scatter_sim(dev, shard, chunk_bytes=chunk, ring=ring, sched=sched, op=op, **opt)
            root = W - 2
            wantr = orc.reduce(wire, CODE[dtype], root, ring=ring, chunk_elems=chunk // es, op=OPS[op])
            out = [None] * W
            out[root] = fresh(1, W * n, dtype, fill=0)[0]
            opt = {}
            wsb = hcl.workspace_bytes(hcl.KIND_REDUCE, W, W * n, CODE[dtype], chunk, sched=sched)
            if wsb:
                opt["workspace"] = torch.empty(wsb, dtype=torch.uint8, device="cuda")
            hcl.reduce_sim(dev, out, root, chunk_bytes=chunk, ring=ring, sched=sched, op=op, **opt)
            torch.cuda.synchronize()
            for r in range(W):
                assert_same_bits(shard[r], want[r], dtype, f"reduce_scatter {op} {sched} W={W} {dtype} rank {r}")
            assert_same_bits(out[root], wantr, dtype, f"reduce {op} {sched} W={W} {dtype}")


def test_operator_through_in_place_fused_last_step_and_staged_transport():
    W, count, dtype = 8, 400_003, "bf16"
    for op in ("prod", "max"):
        cpu, dev = device_inputs(780, W, count, dtype, ("normal", 0.0, 1.0))
        want = orc.allreduce([wl.to_wire(t) for t in cpu], CODE[dtype], op=OPS[op])
        # in place, with the last Reduce-Scatter step writing into the next rank as well
        hcl.allreduce_sim(dev, dev, chunk_bytes=16384, fuse_rs_ag=True, op=op)
        torch.cuda.synchronize()
        for r in range(W):
            assert_same_bits(dev[r], want[r], dtype, f"in-place fused-last-step {op} rank {r}")
        cpu, dev = device_inputs(780, W, count, dtype, ("normal", 0.0, 1.0))
        stage = pinned_stage(hcl.host_stage_bytes(hcl.KIND_ALLREDUCE, W, count, CODE[dtype], 0, xport="host_staged"))
        recv = fresh(W, count, dtype, fill=0)
        hcl.allreduce_sim(dev, recv, xport="host_staged", host_stage=stage, op=op)
        torch.cuda.synchronize()
        for r in range(W):
            assert_same_bits(recv[r], want[r], dtype, f"host-staged {op} rank {r}")


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32", "int32"])
@pytest.mark.parametrize("rounding", ["per_hop", "fp32"])
def test_tree_order_bit_exact(dtype, rounding):
    rnd = orc.ROUND_ONCE if rounding == "fp32" else orc.ROUND_EACH
    for k, (W, count, ring, chunk) in enumerate(CASES + [(7, 99_999, [6, 5, 4, 3, 2, 1, 0], 0), (13, 130_000, None, 0)]):
        for op in ("sum", "prod", "max"):
            mis = k & 1
            cpu, dev = device_inputs(800 + k, W, count, dtype, DISTS[dtype][0], mis)
            wire = [wl.to_wire(t) for t in cpu]
            want = orc.allreduce_var(wire, CODE[dtype], op=OPS[op], ring=ring, order=orc.ORDER_TREE, rounding=rnd)
            recv = fresh(W, count, dtype, mis, fill=0)
            assert hcl.allreduce_sim(dev, recv, chunk_bytes=chunk, ring=ring, sched="fused", order="tree",
                                     accumulate=rounding, op=op) == 1
            torch.cuda.synchronize()
            for r in range(W):
                assert_same_bits(recv[r], want[r], dtype, f"tree {rounding} {op} W={W} count={count} {dtype} mis={mis} rank {r}")
        n = count // W
        cpu, dev = device_inputs(830 + k, W, W * n, dtype, DISTS[dtype][0])
        wire = [wl.to_wire(t) for t in cpu]
        want = orc.reduce_scatter_var(wire, CODE[dtype], ring=ring, order=orc.ORDER_TREE, rounding=rnd)
        shard = fresh(W, n, dtype, fill=0)
        hcl.reduce_scatter_sim(dev, shard, chunk_bytes=chunk, ring=ring, sched="fused", order="tree", accumulate=rounding)
        root = W // 3
        wantr = orc.reduce_var(wire, CODE[dtype], root, ring=ring, order=orc.ORDER_TREE, rounding=rnd)
        out = [None] * W
        out[root] = fresh(1, W * n, dtype, fill=0)[0]
        hcl.reduce_sim(dev, out, root, chunk_bytes=chunk, ring=ring, sched="fused", order="tree", accumulate=rounding)
        torch.cuda.synchronize()
        for r in range(W):
            assert_same_bits(shard[r], want[r], dtype, f"reduce_scatter tree {rounding} W={W} {dtype} rank {r}")
        assert_same_bits(out[root], wantr, dtype, f"reduce tree {rounding} W={W} {dtype}")


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_ring_order_rounding_once_with_product(dtype):
    """(ring order, binary32 intermediates) for an operator other than the sum runs in the general kernel."""
    W, count = 8, 500_000
    cpu, dev = device_inputs(850, W, count, dtype, ("normal", 0.0, 1.0))
    want = orc.allreduce_var([wl.to_wire(t) for t in cpu], CODE[dtype], op=orc.PROD, rounding=orc.ROUND_ONCE)
    recv = fresh(W, count, dtype, fill=0)
    hcl.allreduce_sim(dev, recv, sched="fused", accumulate="fp32", op="prod", threads=512)
    torch.cuda.synchronize()
    for r in range(W):
        assert_same_bits(recv[r], want[r], dtype, f"ring order, one rounding, prod {dtype} rank {r}")


@pytest.mark.parametrize("dtype,fb", [("bf16", 7), ("fp16", 10)])
def test_tree_with_one_rounding_is_within_two_ulp_of_the_exact_sum(dtype, fb):
    W, count = 16, 1_000_000
    cpu, dev = device_inputs(860, W, count, dtype, ("normal", 0.0, 1.0))
    recv = fresh(W, count, dtype, fill=0)
    hcl.allreduce_sim(dev, recv, sched="fused", order="tree", accumulate="fp32")
    torch.cuda.synchronize()
    vals = torch.stack([t.double() for t in cpu])
    exact = vals.sum(0)
    ref = exact.to(wl.TORCH_DTYPE[dtype]).double()
    got = recv[0].cpu().double()
    ulp = torch.exp2(torch.floor(torch.log2(ref.abs().clamp_min(1e-30))) - fb)
    assert bool(((got - ref).abs() <= 2 * ulp).all())


def test_tree_order_and_operators_reject_what_does_not_exist():
    d = fresh(4, 1024, "bf16", fill=1)
    with pytest.raises(hcl.HclError, match="UNSUPPORTED"):
        hcl.allreduce_sim(d, d, order="tree")
    with pytest.raises(hcl.HclError, match="UNSUPPORTED"):
        hcl.allreduce_sim(d, d, op=7)
