"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
element by element and bit for bit (NaN compared as NaN), on seeded inputs.
Sizes here finish in seconds on the oracle and still span many tiles, several
chunks and ragged tails."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import (CODE, assert_same_bits, device_inputs, fresh, run_all_gather, run_allreduce,
                      run_reduce_scatter)
from oracle import ring_oracle as orc
from paper_2601_22585_amd import hcl

pytestmark = pytest.mark.gpu

DIST = {"fp32": ("uniform", -1.0, 1.0), "bf16": ("normal", 0.0, 1e-3), "fp16": ("normal", 0.0, 1.0),
        "int32": ("randint", -1000, 1000)}
DTYPES = ["fp32", "bf16", "fp16", "int32"]


def test_config1_allreduce_w4_fp32_1mib():
    c = wl.CONFIGS[1]
    for sched in ("stepwise", "fused"):
        n = run_allreduce(1, c["W"], c["count"], c["dtype"], c["dist"], chunk_bytes=c["chunk_bytes"], sched=sched)
        assert n == (6 if sched == "stepwise" else 1)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("sched", ["stepwise", "fused"])
def test_allreduce_ragged_sizes_rings_chunks(dtype, sched):
    es = wl.ESIZE[dtype]
    # (W, count, ring, chunk_bytes): counts not divisible by W or by the vector width
    cases = [
        (2, 100_003, None, 0),
        (3, 262_147, [2, 0, 1], 4096),
        (5, 1_000_001, [3, 1, 4, 0, 2], 64 * 1024),
        (8, 1_048_576 + 8, None, 16 * 1024),
        (8, 999_983, [7, 2, 5, 0, 3, 6, 1, 4], es * 1001),      # chunk not a multiple of 16 bytes
        (16, 2_000_003, None, 32 * 1024),
        (16, 65_536, list(range(15, -1, -1)), 0),
    ]
    for k, (W, count, ring, chunk) in enumerate(cases):
        for inplace in (False, True):
            run_allreduce(100 + k, W, count, dtype, DIST[dtype], ring=ring, chunk_bytes=chunk,
                          inplace=inplace, sched=sched)


@pytest.mark.parametrize("dtype", DTYPES)
def test_allreduce_buffers_aligned_to_the_element_size_only(dtype):
    for sched in ("stepwise", "fused"):
        for mis in (1, 3):
            run_allreduce(120, 4, 50_001, dtype, DIST[dtype], chunk_bytes=0, misalign=mis, sched=sched)
            run_allreduce(121, 4, 50_001, dtype, DIST[dtype], chunk_bytes=wl.ESIZE[dtype] * 777, misalign=mis,
                          inplace=True, sched=sched)


@pytest.mark.parametrize("dtype", DTYPES)
def test_allreduce_degenerate_shapes(dtype):
    for sched in ("stepwise", "fused"):
        for W, count in [(1, 1000), (4, 1), (4, 3), (8, 9), (16, 17), (16, 15), (3, 2)]:
            for inplace in (False, True):
                run_allreduce(130, W, count, dtype, DIST[dtype], inplace=inplace, sched=sched)
    # count == 0 is a no-op that touches nothing
    d = fresh(4, 16, dtype, fill=1)
    assert hcl.allreduce_sim(d, d, count=0) == 0
    torch.cuda.synchronize()
    assert all(bool((t == 1).all()) for t in d)


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
def test_allreduce_fused_last_rs_step(dtype):
    for W, count, chunk in [(2, 10_007, 0), (4, 300_000, 8192), (8, 1_000_003, 64 * 1024)]:
        for inplace in (False, True):
            n = run_allreduce(140, W, count, dtype, DIST[dtype], chunk_bytes=chunk, inplace=inplace, fuse_rs_ag=True)
            assert n == 2 * (W - 1) - 1


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("sched", ["stepwise", "fused"])
def test_reduce_scatter_and_all_gather(dtype, sched):
    for k, (W, n, ring, chunk) in enumerate([(2, 10_001, None, 0), (4, 65_536, [1, 3, 0, 2], 16 * 1024),
                                             (8, 125_003, None, 4096), (16, 40_000, None, 0)]):
        for inplace in (False, True):
            run_reduce_scatter(200 + k, W, n, dtype, DIST[dtype], ring=ring, chunk_bytes=chunk, inplace=inplace, sched=sched)
            run_all_gather(220 + k, W, n, dtype, DIST[dtype], ring=ring, chunk_bytes=chunk, inplace=inplace, sched=sched)
    run_reduce_scatter(240, 1, 1000, dtype, DIST[dtype], sched=sched)
    run_all_gather(241, 1, 1000, dtype, DIST[dtype], sched=sched)
    run_reduce_scatter(242, 4, 50_001, dtype, DIST[dtype], misalign=1, sched=sched)
    run_all_gather(243, 4, 50_001, dtype, DIST[dtype], misalign=1, sched=sched)


@pytest.mark.parametrize("dtype", DTYPES)
def test_allreduce_equals_all_gather_of_reduce_scatter_on_device(dtype):
    W, n = 8, 70_000
    cpu, dev = device_inputs(300, W, W * n, dtype, DIST[dtype])
    ar = fresh(W, W * n, dtype, fill=0)
    hcl.allreduce_sim(dev, ar, chunk_bytes=8192)
    shard = fresh(W, n, dtype, fill=0)
    hcl.reduce_scatter_sim(dev, shard, sched="fused")
    full = fresh(W, W * n, dtype, fill=0)
    hcl.all_gather_sim(shard, full, chunk_bytes=4096)
    torch.cuda.synchronize()
    for r in range(W):
        assert np.array_equal(wl.to_wire(ar[r]), wl.to_wire(full[r]))
        assert np.array_equal(wl.to_wire(ar[0]), wl.to_wire(ar[r]))


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_host_staged_transport(dtype):
    for W, count, chunk in [(2, 20_001, 0), (4, 262_144, 64 * 1024), (8, 500_003, 0)]:
        for inplace in (False, True):
            n = run_allreduce(400, W, count, dtype, DIST[dtype], chunk_bytes=chunk, inplace=inplace, xport="host_staged")
            assert n == 2 * (W - 1) + 1
    run_reduce_scatter(401, 4, 30_001, dtype, DIST[dtype], xport="host_staged")
    run_reduce_scatter(402, 8, 30_000, dtype, DIST[dtype], inplace=True, xport="host_staged")
    run_all_gather(403, 4, 30_001, dtype, DIST[dtype], xport="host_staged")
    run_all_gather(404, 8, 30_000, dtype, DIST[dtype], inplace=True, xport="host_staged")


def test_launch_shapes_do_not_change_the_bits():
    W, count, dtype = 8, 600_011, "bf16"
    for kw in [dict(threads=64, unroll=1), dict(threads=1024, unroll=8), dict(blocks=1), dict(blocks=7, unroll=2),
               dict(nontemporal=-1), dict(nontemporal=1), dict(nontemporal=2), dict(threads=512, unroll=4, blocks=3000)]:
        for sched in ("stepwise", "fused"):
            run_allreduce(500, W, count, dtype, DIST[dtype], chunk_bytes=32 * 1024, sched=sched, **kw)


@pytest.mark.parametrize("dtype", ["bf16", "fp32", "int32"])
def test_written_through_stores_in_strided_unrolled_launches(dtype):
    """The stores that hand a step's output to the next launch are spelled out as an instruction
    (wire.h) and carry their own wait states; a capped grid with several vectors per thread is where
    a register that still holds store data is reused soonest."""
    for kw in [dict(threads=256, unroll=4, blocks=64), dict(threads=64, unroll=8, blocks=301), dict(threads=128, unroll=2, blocks=1000)]:
        run_allreduce(510, 8, 1_200_011, dtype, DIST[dtype], chunk_bytes=256 * 1024, nontemporal=2, **kw)
        run_reduce_scatter(511, 4, 300_007, dtype, DIST[dtype], nontemporal=2, **kw)
        run_all_gather(512, 4, 300_007, dtype, DIST[dtype], nontemporal=2, **kw)


def _special_inputs(dtype, W, count):
    """Rank buffers salted with infinities, NaN, signed zeros, subnormals and near-overflow values."""
    g = torch.Generator().manual_seed(77)
    td = wl.TORCH_DTYPE[dtype]
    big = {"fp16": 6.0e4, "bf16": 3.0e38, "fp32": 3.0e38}[dtype]
    tiny = {"fp16": 6.0e-8, "bf16": 1.0e-40, "fp32": 1.0e-44}[dtype]
    menu = torch.tensor([0.0, -0.0, float("inf"), float("-inf"), float("nan"), big, -big, tiny, -tiny,
                         1.0, -1.0, 0.5 * tiny, 3 * tiny], dtype=torch.float64)
    out = []
    for r in range(W):
        base = torch.empty(count).normal_(0, 1, generator=g).double()
        pick = torch.randint(0, menu.numel(), (count,), generator=g)
        use = torch.rand(count, generator=g) < 0.3
        out.append(torch.where(use, menu[pick], base).to(td))
    return out


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_special_values(dtype):
    W, count = 4, 40_003
    cpu = _special_inputs(dtype, W, count)
    for sched in ("stepwise", "fused"):
        run_allreduce(0, W, count, dtype, None, cpu_inputs=cpu, sched=sched)
    run_allreduce(0, W, count, dtype, None, cpu_inputs=cpu, misalign=1)


def test_int32_wraps():
    W, count = 4, 10_000
    g = torch.Generator().manual_seed(5)
    cpu = [torch.randint(-2**31, 2**31, (count,), generator=g, dtype=torch.int64).to(torch.int32) for _ in range(W)]
    for sched in ("stepwise", "fused"):
        run_allreduce(0, W, count, "int32", None, cpu_inputs=cpu, sched=sched)


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_cancellation_example_on_device(dtype):
    M = {"fp32": 2.0 ** 24, "bf16": 256.0, "fp16": 2048.0}[dtype]
    n = 4096
    cpu = [torch.full((n,), v, dtype=wl.TORCH_DTYPE[dtype]) for v in (M, 1.0, -M, 1.0)]
    for sched in ("stepwise", "fused"):
        dev = [t.cuda() for t in cpu]
        hcl.allreduce_sim(dev, dev, sched=sched)
        torch.cuda.synchronize()
        got = dev[2].float().cpu().view(4, n // 4)
        assert [float(got[c, 0]) for c in range(4)] == [2.0, 2.0, 0.0, 1.0]
        assert all(bool((got[c] == got[c, 0]).all()) for c in range(4))


def test_events_hook_brackets_every_launch():
    W, count = 4, 1 << 20
    cpu, dev = device_inputs(600, W, count, "fp32", DIST["fp32"])
    ev = hcl.EventList(2 * (W - 1) + 1)
    n = hcl.allreduce_sim(dev, dev, events=ev)
    torch.cuda.synchronize()
    assert n == 2 * (W - 1)
    per = [ev.elapsed_ms(i, i + 1) for i in range(n)]
    assert all(p > 0 for p in per) and abs(sum(per) - ev.elapsed_ms(0, n)) < 0.05 * ev.elapsed_ms(0, n) + 0.01
    ev.close()


def test_runs_on_a_side_stream_and_under_graph_capture():
    W, count, dtype = 4, 300_000, "bf16"
    cpu, dev = device_inputs(700, W, count, dtype, DIST[dtype])
    want = orc.allreduce([wl.to_wire(t) for t in cpu], CODE[dtype])
    recv = fresh(W, count, dtype, fill=0)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        hcl.allreduce_sim(dev, recv, chunk_bytes=16384)
    s.synchronize()
    for r in range(W):
        assert_same_bits(recv[r], want[r], dtype, f"side stream rank {r}")
    # captured once, replayed three times with eager work in between; every replay must match
    g = torch.cuda.CUDAGraph()
    for t in recv:
        t.zero_()
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        hcl.allreduce_sim(dev, recv, chunk_bytes=16384)
    for rep in range(3):
        for t in recv:
            t.fill_(float(rep))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for r in range(W):
            assert_same_bits(recv[r], want[r], dtype, f"graph replay {rep} rank {r}")


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_single_hop_over_all_bit_patterns(dtype):
    """W = 2 makes every output one hop: all 2^16 patterns of one operand against a
    set of partners chosen to hit ties, subnormal results, overflow, zeros, inf and NaN."""
    allp = torch.arange(0, 1 << 16, dtype=torch.int32).to(torch.int16)
    inf = 0x7F80 if dtype == "bf16" else 0x7C00
    partners = [0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x03FF, 0x0400, inf, inf | 0x8000, inf + 1,
                inf - 1, (inf - 1) | 0x8000, 0x3F80, 0xBF80, 0x3C00, 0xBC00, 0x3F81, 0x3C01, 0x0002, 0x8002]
    g = torch.Generator().manual_seed(3)
    partners += torch.randint(0, 1 << 16, (43,), generator=g).tolist()
    a = allp.repeat(len(partners)).view(wl.TORCH_DTYPE[dtype])
    b = torch.tensor(partners, dtype=torch.int32).to(torch.int16).repeat_interleave(1 << 16).view(wl.TORCH_DTYPE[dtype])
    for sched in ("stepwise", "fused"):
        run_allreduce(0, 2, a.numel(), dtype, None, cpu_inputs=[a, b], sched=sched)
        run_allreduce(0, 2, a.numel(), dtype, None, cpu_inputs=[b, a], sched=sched, misalign=1)


@pytest.mark.parametrize("dtype", ["bf16", "fp32", "int32"])
def test_two_dependency_chains_give_the_same_bits(dtype):
    """opts.aux_stream: the second half of every step's chunks runs as a chain of its own on a
    second stream.  Every collective of the stepwise schedule, both transports, in and out of
    place, ragged blocks, chunk counts that are odd, one and two."""
    s2, ev = torch.cuda.Stream(), hcl.EventList(2)
    es = wl.ESIZE[dtype]
    kw = dict(aux_stream=s2, aux_events=ev)
    for k, (W, count, ring, chunk) in enumerate([(8, 1_000_003, None, 16 * 1024), (5, 262_147, [3, 1, 4, 0, 2], 4096),
                                                 (4, 300_000, None, es * 25_000), (16, 2_000_003, None, 64 * 1024),
                                                 (3, 100_000, None, es * 40_000), (2, 50_001, None, 0)]):
        for inplace in (False, True):
            n = run_allreduce(800 + k, W, count, dtype, DIST[dtype], ring=ring, chunk_bytes=chunk, inplace=inplace, **kw)
            B = -(-count // W)
            nch = -(-B * es // chunk) if chunk else 1
            assert n == 2 * (W - 1) * (2 if nch >= 2 else 1), (n, W, nch)
            run_allreduce(810 + k, W, count, dtype, DIST[dtype], ring=ring, chunk_bytes=chunk, inplace=inplace,
                          fuse_rs_ag=True, **kw)
    for inplace in (False, True):
        run_allreduce(820, 8, 500_003, dtype, DIST[dtype], chunk_bytes=32 * 1024, inplace=inplace, xport="host_staged", **kw)
        run_reduce_scatter(821, 8, 125_003, dtype, DIST[dtype], chunk_bytes=8192, inplace=inplace, **kw)
        run_all_gather(822, 8, 125_003, dtype, DIST[dtype], chunk_bytes=8192, inplace=inplace, **kw)
        run_reduce_scatter(823, 4, 30_001, dtype, DIST[dtype], chunk_bytes=4096, inplace=inplace, xport="host_staged", **kw)
    ev.close()


def test_two_dependency_chains_under_graph_capture():
    """The fork onto the second stream and the join back are event record / wait pairs, so a call
    with aux_stream can be captured from the caller's stream; replays must reproduce the result."""
    W, count, dtype = 4, 600_000, "bf16"
    cpu, dev = device_inputs(830, W, count, dtype, DIST[dtype])
    want = orc.allreduce([wl.to_wire(t) for t in cpu], CODE[dtype])
    recv = fresh(W, count, dtype, fill=0)
    s2, ev = torch.cuda.Stream(), hcl.EventList(2)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        n = hcl.allreduce_sim(dev, recv, chunk_bytes=32768, aux_stream=s2, aux_events=ev)
    assert n == 4 * (W - 1)
    for rep in range(3):
        for t in recv:
            t.fill_(float(rep))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for r in range(W):
            assert_same_bits(recv[r], want[r], dtype, f"two chains, graph replay {rep} rank {r}")
    del g
    ev.close()


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_slabs_do_not_change_the_bits(dtype):
    """opts.slab_bytes: the ring runs to completion on one slab of every block before the next.
    Budgets that give 1, 2, 7 and many slabs, ragged blocks, both chains, in and out of place."""
    es = wl.ESIZE[dtype]
    for k, (W, count, chunk, slab) in enumerate([(8, 1_000_003, 16 * 1024, 8 * 64 * 1024), (4, 300_000, 4096, 4 * 4096),
                                                 (5, 262_147, 0, 5 * es * 70_000), (16, 2_000_003, 64 * 1024, 1 << 20),
                                                 (3, 100_000, es * 1000, -1)]):
        for inplace in (False, True):
            run_allreduce(850 + k, W, count, dtype, DIST[dtype], chunk_bytes=chunk, inplace=inplace, slab_bytes=slab)
            run_allreduce(860 + k, W, count, dtype, DIST[dtype], chunk_bytes=chunk, inplace=inplace, slab_bytes=slab, fuse_rs_ag=True)
    s2, ev = torch.cuda.Stream(), hcl.EventList(2)
    n = run_allreduce(870, 8, 1_000_003, dtype, DIST[dtype], chunk_bytes=16 * 1024, slab_bytes=8 * 32 * 1024)
    B = -(-1_000_003 // 8)
    slabs = -(-B * es // (32 * 1024))
    assert n == 14 * slabs
    run_allreduce(871, 8, 1_000_003, dtype, DIST[dtype], chunk_bytes=16 * 1024, slab_bytes=8 * 64 * 1024, aux_stream=s2, aux_events=ev)
    for inplace in (False, True):
        run_reduce_scatter(872, 8, 125_003, dtype, DIST[dtype], chunk_bytes=8192, inplace=inplace, slab_bytes=8 * 16384)
        run_all_gather(873, 8, 125_003, dtype, DIST[dtype], chunk_bytes=8192, inplace=inplace, slab_bytes=8 * 16384)
    ev.close()
