"""GPU parity at the full sizes of the named workloads, in the launch
configuration bench.py times (library defaults), against the CPU oracle.
Where the oracle can replay the whole workload in seconds it does, otherwise
it replays windows: the ring is element-wise, so the leading m elements of
every block of every rank form a smaller instance with the same block
membership, whose result must equal the same windows of the full result."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import ring_oracle as orc
from paper_2601_22585_amd import hcl

pytestmark = pytest.mark.gpu


def _device_inputs(cfg_id, W, count, dtype, dist):
    send = [torch.empty(count, dtype=wl.TORCH_DTYPE[dtype], device="cuda") for _ in range(W)]
    for r in range(W):
        wl.fill_rank(send[r], wl.rank_seed(cfg_id, r), dist)
    return send


def _windows(count, W, m, extra=()):
    """Leading and trailing m elements of every block, plus windows around the given offsets."""
    B = -(-count // W)
    offs = sorted(set([0, B - m] + [max(0, min(B - m, int(o))) for o in extra]))
    return B, offs


def _check_allreduce_windows(send, recv, W, count, dtype, m, offs, chunk_elems):
    B = -(-count // W)
    for off in offs:
        ins = [np.concatenate([wl.to_wire(send[r][c * B + off:c * B + off + m]) for c in range(W)]) for r in range(W)]
        want = orc.allreduce(ins, wl.DTYPE_CODE[dtype], chunk_elems=chunk_elems)
        for r in range(W):
            got = np.concatenate([wl.to_wire(recv[r][c * B + off:c * B + off + m]) for c in range(W)])
            assert wl.bits_equal_nan_aware(got, want[r], dtype).all(), (off, r)


@pytest.mark.parametrize("sched,fuse", [("stepwise", False), ("stepwise", True), ("fused", False)])
def test_config2_full_size_every_element(sched, fuse):
    c = wl.CONFIGS[2]
    W, count, dtype = c["W"], c["count"], c["dtype"]
    send = _device_inputs(2, W, count, dtype, c["dist"])
    recv = [torch.empty_like(t) for t in send]
    hcl.allreduce_sim(send, recv, chunk_bytes=c["chunk_bytes"], sched=sched, fuse_rs_ag=fuse)
    torch.cuda.synchronize()
    work = [wl.to_wire(t) for t in send]               # D2H copies: the oracle replays them in place
    orc.set_threads(0)
    orc.allreduce_inplace(work, wl.DTYPE_CODE[dtype], chunk_elems=c["chunk_bytes"] // 2)
    for r in range(W):
        got = wl.to_wire(recv[r])
        assert np.array_equal(got, work[r]), f"rank {r}: {(got != work[r]).sum()} elements differ"
        if r:
            assert torch.equal(recv[r].view(torch.int16), recv[0].view(torch.int16))


@pytest.mark.parametrize("nbytes", [8 << 10, 1 << 20, 64 << 20])
def test_config3_sweep_points_every_element(nbytes):
    c = wl.CONFIGS[3]
    W, dtype = c["W"], c["dtype"]
    count = nbytes // 2
    chunk = min(count // W * 2, c["chunk_bytes"])
    send = _device_inputs(3, W, count, dtype, c["dist"])
    want = orc.allreduce([wl.to_wire(t) for t in send], wl.DTYPE_CODE[dtype], chunk_elems=chunk // 2)
    for sched in ("stepwise", "fused"):
        recv = [torch.zeros_like(t) for t in send]
        hcl.allreduce_sim(send, recv, chunk_bytes=chunk, sched=sched)
        torch.cuda.synchronize()
        for r in range(W):
            assert np.array_equal(wl.to_wire(recv[r]), want[r]), (sched, r)


def test_config3_one_gib_per_rank_windows():
    c = wl.CONFIGS[3]
    W, dtype = c["W"], c["dtype"]
    count = (1 << 30) // 2
    send = _device_inputs(3, W, count, dtype, c["dist"])
    recv = [torch.empty_like(t) for t in send]
    m = 1 << 16
    B, offs = _windows(count, W, m, extra=[(4 << 20) // 2 - m // 2, 12345678])
    for sched in ("stepwise", "fused"):
        for t in recv:
            t.zero_()
        hcl.allreduce_sim(send, recv, chunk_bytes=c["chunk_bytes"], sched=sched)
        torch.cuda.synchronize()
        _check_allreduce_windows(send, recv, W, count, dtype, m, offs, 0)
        for r in range(1, W):
            assert torch.equal(recv[r].view(torch.int16), recv[0].view(torch.int16))


@pytest.mark.parametrize("cfg_id", [4, 41])
def test_config4_reduce_scatter_then_all_gather_windows(cfg_id):
    """Shards of 2^27 elements (one eighth of the named 2 GiB shards, so that this
    test stays within a minute; bench.py runs the named size), out of place with
    workspace, then All-Gather of the shards; oracle on windows."""
    c = wl.CONFIGS[cfg_id]
    W, dtype = c["W"], c["dtype"]
    es = wl.ESIZE[dtype]
    n = (1 << 28) // es                    # 256 MiB shards
    count = n * W
    send = _device_inputs(cfg_id, W, count, dtype, c["dist"])
    shard = [torch.zeros(n, dtype=wl.TORCH_DTYPE[dtype], device="cuda") for _ in range(W)]
    ws = torch.empty(hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, W, n, wl.DTYPE_CODE[dtype]), dtype=torch.uint8, device="cuda")
    hcl.reduce_scatter_sim(send, shard, chunk_bytes=c["chunk_bytes"], workspace=ws)
    torch.cuda.synchronize()
    m = 1 << 16
    for off in (0, n - m, (4 << 20) // es - m // 2, 7654321 // es * es):
        ins = [np.concatenate([wl.to_wire(send[r][q * n + off:q * n + off + m]) for q in range(W)]) for r in range(W)]
        want = orc.reduce_scatter(ins, wl.DTYPE_CODE[dtype])
        for r in range(W):
            assert np.array_equal(wl.to_wire(shard[r][off:off + m]), want[r]), (off, r)
    if dtype == "int32":
        # exact and order-free: the whole result equals the plain integer sum
        for r in range(W):
            tot = torch.zeros(n, dtype=torch.int64, device="cuda")
            for q in range(W):
                tot += send[q][r * n:(r + 1) * n]
            assert torch.equal(tot.to(torch.int32), shard[r])
    del ws
    full = send                             # reuse the inputs' memory for the gathered result
    hcl.all_gather_sim(shard, full, chunk_bytes=c["chunk_bytes"])
    torch.cuda.synchronize()
    for r in range(W):
        for q in range(W):
            assert torch.equal(full[r][q * n:(q + 1) * n].view(torch.int16 if es == 2 else torch.int32),
                               shard[q].view(torch.int16 if es == 2 else torch.int32)), (r, q)
