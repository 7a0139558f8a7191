"""GPU parity of the binary32-accumulation variant (fused schedule, accumulate=fp32):
bit for bit against the oracle's replay of the same arithmetic, and within the
stated tolerance of the correctly rounded exact sum."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import CODE, assert_same_bits, device_inputs, fresh
from oracle import ring_oracle as orc
from paper_2601_22585_amd import hcl

pytestmark = pytest.mark.gpu

DIST = {"fp32": ("uniform", -1.0, 1.0), "bf16": ("normal", 0.0, 1e-3), "fp16": ("normal", 0.0, 1.0),
        "int32": ("randint", -1000, 1000)}


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32", "int32"])
def test_allreduce_reduce_scatter_reduce_bit_exact(dtype):
    cases = [(2, 10_001, None, 0), (3, 262_147, [2, 0, 1], 4096), (8, 1_000_003, None, 64 * 1024),
             (8, 524_288, [7, 2, 5, 0, 3, 6, 1, 4], 0), (16, 300_001, None, 32 * 1024)]
    for k, (W, count, ring, chunk) in enumerate(cases):
        for mis in (0, 1):
            cpu, dev = device_inputs(900 + k, W, count, dtype, DIST[dtype], mis)
            want = orc.allreduce_fp32acc([wl.to_wire(t) for t in cpu], CODE[dtype], ring=ring)
            recv = fresh(W, count, dtype, mis, fill=0)
            assert hcl.allreduce_sim(dev, recv, chunk_bytes=chunk, ring=ring, sched="fused", accumulate="fp32") == 1
            torch.cuda.synchronize()
            for r in range(W):
                assert_same_bits(recv[r], want[r], dtype, f"allreduce fp32acc W={W} count={count} {dtype} mis={mis} rank {r}")
        n = count // W
        cpu, dev = device_inputs(920 + k, W, W * n, dtype, DIST[dtype])
        wire = [wl.to_wire(t) for t in cpu]
        want = orc.reduce_scatter_fp32acc(wire, CODE[dtype], ring=ring)
        shard = fresh(W, n, dtype, fill=0)
        hcl.reduce_scatter_sim(dev, shard, chunk_bytes=chunk, ring=ring, sched="fused", accumulate="fp32")
        root = W // 2
        wantr = orc.reduce_fp32acc(wire, CODE[dtype], root, ring=ring)
        out = [None] * W
        out[root] = fresh(1, W * n, dtype, fill=0)[0]
        hcl.reduce_sim(dev, out, root, chunk_bytes=chunk, ring=ring, sched="fused", accumulate="fp32")
        torch.cuda.synchronize()
        for r in range(W):
            assert_same_bits(shard[r], want[r], dtype, f"reduce_scatter fp32acc W={W} n={n} {dtype} rank {r}")
        assert_same_bits(out[root], wantr, dtype, f"reduce fp32acc W={W} {dtype}")


@pytest.mark.parametrize("dtype,fb", [("bf16", 7), ("fp16", 10)])
def test_within_two_ulp_of_the_exact_sum_and_not_the_ring_result(dtype, fb):
    W, count = 8, 2_000_000
    cpu, dev = device_inputs(940, W, count, dtype, ("normal", 0.0, 1.0))
    recv = fresh(W, count, dtype, fill=0)
    hcl.allreduce_sim(dev, recv, sched="fused", accumulate="fp32")
    ring = fresh(W, count, dtype, fill=0)
    hcl.allreduce_sim(dev, ring, sched="fused")
    torch.cuda.synchronize()
    vals = torch.stack([t.double() for t in cpu])
    exact = vals.sum(0)
    ref = exact.to(wl.TORCH_DTYPE[dtype]).double()
    got = recv[0].cpu().double()
    big = torch.maximum(ref.abs(), vals.cumsum(0).abs().max(0).values)
    ulp = torch.exp2(torch.floor(torch.log2(big.clamp_min(1e-30))) - fb)
    assert bool(((got - ref).abs() <= 2 * ulp).all())
    # the variant is a different result from the per-hop ring, and closer to the exact sum
    rg = ring[0].cpu().double()
    assert bool((rg != got).any())
    assert float((got - exact).abs().mean()) < float((rg - exact).abs().mean())


def test_stepwise_rejects_fp32_accumulation():
    d = fresh(4, 1024, "bf16", fill=1)
    with pytest.raises(hcl.HclError, match="UNSUPPORTED"):
        hcl.allreduce_sim(d, d, accumulate="fp32")
    with pytest.raises(hcl.HclError, match="UNSUPPORTED"):
        hcl.allreduce_sim(d, d, sched="fused", accumulate=7)
