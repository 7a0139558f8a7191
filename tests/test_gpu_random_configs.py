"""Seeded random sweep over the call space -- collective, wire type, W, count,
ring, chunk size, schedule, operator, order, rounding, in place or not,
alignment, launch shape -- each case compared bit for bit with the oracle.
Small sizes; the point is the combinations."""
import random

import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import (CODE, assert_same_bits, check_guards, device_inputs, fresh, pinned_stage, run_all_gather,
                      run_alltoall, run_broadcast)
from oracle import ring_oracle as orc
from paper_2601_22585_amd import hcl

pytestmark = pytest.mark.gpu

OPS = {"sum": orc.SUM, "prod": orc.PROD, "max": orc.MAX, "min": orc.MIN}
DIST = {"fp32": ("uniform", -2.0, 2.0), "bf16": ("normal", 0.0, 1.0), "fp16": ("normal", 0.0, 1.0),
        "int32": ("randint", -1000, 1000), "fp64": ("normal", 0.0, 1.0), "int64": ("randint", -10**9, 10**9),
        "uint8": ("randint", 0, 255)}


_CHAIN = []


def _second_chain():
    """One side stream and one pair of events for every call that wants two chains."""
    if not _CHAIN:
        _CHAIN.extend([torch.cuda.Stream(), hcl.EventList(2)])
    return _CHAIN[0], _CHAIN[1]


def _case(rnd):
    dtype = rnd.choice(list(DIST))
    es = wl.ESIZE[dtype]
    W = rnd.choice([1, 2, 3, 4, 5, 7, 8, 11, 16])
    sched = rnd.choice(["stepwise", "fused"])
    c = dict(dtype=dtype, W=W, sched=sched, op=rnd.choice(["sum", "sum", "prod", "max", "min"]),
             kind=rnd.choice(["allreduce", "allreduce", "reduce_scatter", "reduce"]),
             ring=None if rnd.random() < 0.4 else rnd.sample(range(W), W),
             mis=rnd.choice([0, 0, 0, 1, 3]), inplace=rnd.random() < 0.3,
             threads=rnd.choice([0, 0, 64, 128, 256, 1024]), unroll=rnd.choice([0, 0, 1, 2, 4, 8]),
             blocks=rnd.choice([0, 0, 0, 7, 64, 1000]), nontemporal=rnd.choice([0, 0, -1, 1, 2]))
    c["order"] = rnd.choice(["ring", "tree"]) if sched == "fused" else "ring"
    c["acc"] = rnd.choice(["per_hop", "fp32"]) if sched == "fused" else "per_hop"
    c["fuse"] = sched == "stepwise" and c["kind"] == "allreduce" and rnd.random() < 0.3
    # blocks travelling through pinned host memory: STEPWISE All-Reduce and Reduce-Scatter have that transport
    c["xport"] = "host_staged" if (sched == "stepwise" and c["kind"] != "reduce" and rnd.random() < 0.3) else "direct"
    # the chunk range split over two streams, each half a dependency chain of its own
    c["two_chains"] = sched == "stepwise" and rnd.random() < 0.35
    # slabs: what one step may write before the ring moves on to the next slab of every block
    c["slab"] = rnd.choice([0, 0, -1, 4096, 65536, 1 << 20])
    n = rnd.choice([1, 17, 1000, 4096, 65_536, rnd.randrange(1, 200_000)])
    c["n"] = n
    chunk_elems = rnd.choice([0, 0, 1, 16, 1024, 8192, rnd.randrange(1, 50_000)])
    c["chunk"] = chunk_elems * es
    return c


def _run(c, seed):
    dtype, W, n = c["dtype"], c["W"], c["n"]
    es = wl.ESIZE[dtype]
    code, op = CODE[dtype], OPS[c["op"]]
    variant = c["order"] == "tree" or c["acc"] == "fp32"
    vkw = dict(op=op, ring=c["ring"], order=orc.ORDER_TREE if c["order"] == "tree" else orc.ORDER_RING,
               rounding=orc.ROUND_ONCE if c["acc"] == "fp32" else orc.ROUND_EACH)
    opt = dict(chunk_bytes=c["chunk"], ring=c["ring"], sched=c["sched"], op=c["op"], order=c["order"],
               accumulate=c["acc"], threads=c["threads"], unroll=c["unroll"], blocks=c["blocks"],
               nontemporal=c["nontemporal"], xport=c["xport"], slab_bytes=c["slab"])
    tag = f"seed {seed}: {c}"
    if c["two_chains"]:
        opt["aux_stream"], opt["aux_events"] = _second_chain()
    if c["xport"] == "host_staged":
        kind = hcl.KIND_ALLREDUCE if c["kind"] == "allreduce" else hcl.KIND_REDUCE_SCATTER
        opt["host_stage"] = pinned_stage(hcl.host_stage_bytes(kind, W, n, code, c["chunk"], xport="host_staged"))
    if c["kind"] == "allreduce":
        cpu, dev = device_inputs(seed, W, n, dtype, DIST[dtype], c["mis"])
        wire = [wl.to_wire(t) for t in cpu]
        want = (orc.allreduce_var(wire, code, **vkw) if variant
                else orc.allreduce(wire, code, ring=c["ring"], chunk_elems=c["chunk"] // es, op=op))
        recv = dev if c["inplace"] else fresh(W, n, dtype, c["mis"], fill=0)
        hcl.allreduce_sim(dev, recv, fuse_rs_ag=c["fuse"], **opt)
        torch.cuda.synchronize()
        for r in range(W):
            assert_same_bits(recv[r], want[r], dtype, f"{tag} rank {r}")
    elif c["kind"] == "reduce_scatter":
        cpu, dev = device_inputs(seed, W, W * n, dtype, DIST[dtype], c["mis"])
        wire = [wl.to_wire(t) for t in cpu]
        want = (orc.reduce_scatter_var(wire, code, **vkw) if variant
                else orc.reduce_scatter(wire, code, ring=c["ring"], chunk_elems=c["chunk"] // es, op=op))
        if c["inplace"]:
            recv = [dev[r][r * n:(r + 1) * n] for r in range(W)]
        else:
            recv = fresh(W, n, dtype, c["mis"], fill=0)
            wsb = hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, W, n, code, c["chunk"], sched=c["sched"], xport=c["xport"])
            if wsb:
                opt["workspace"] = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        hcl.reduce_scatter_sim(dev, recv, **opt)
        torch.cuda.synchronize()
        for r in range(W):
            assert_same_bits(recv[r], want[r], dtype, f"{tag} rank {r}")
    else:
        root = seed % W
        cpu, dev = device_inputs(seed, W, n, dtype, DIST[dtype], c["mis"])
        wire = [wl.to_wire(t) for t in cpu]
        want = (orc.reduce_var(wire, code, root, **vkw) if variant
                else orc.reduce(wire, code, root, ring=c["ring"], chunk_elems=c["chunk"] // es, op=op))
        out = [None] * W
        out[root] = dev[root] if c["inplace"] else fresh(1, n, dtype, c["mis"], fill=0)[0]
        wsb = hcl.workspace_bytes(hcl.KIND_REDUCE, W, n, code, c["chunk"], sched=c["sched"])
        if wsb:
            opt["workspace"] = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        hcl.reduce_sim(dev, out, root, **opt)
        torch.cuda.synchronize()
        assert_same_bits(out[root], want, dtype, tag)
    check_guards()


@pytest.mark.parametrize("batch", range(3))
def test_random_configurations_of_the_copying_collectives(batch):
    rnd = random.Random(30260 + batch)
    for i in range(40):
        seed = 7000 + 100 * batch + i
        dtype = rnd.choice(list(DIST))
        es = wl.ESIZE[dtype]
        W = rnd.choice([1, 2, 3, 5, 8, 13, 16])
        n = rnd.choice([1, 17, 4096, rnd.randrange(1, 60_000)])
        opt = dict(ring=None if rnd.random() < 0.4 else rnd.sample(range(W), W),
                   chunk_bytes=rnd.choice([0, 0, 1, 64, 4096, rnd.randrange(1, 20_000)]) * es,
                   misalign=rnd.choice([0, 0, 1, 3]), sched=rnd.choice(["stepwise", "fused"]),
                   threads=rnd.choice([0, 0, 64, 256]), unroll=rnd.choice([0, 0, 1, 2, 4]),
                   blocks=rnd.choice([0, 0, 5, 300]))
        kind = rnd.choice(["all_gather", "broadcast", "alltoall"])
        if kind == "all_gather" and opt["sched"] == "stepwise" and rnd.random() < 0.4:
            opt["xport"] = "host_staged"
        if kind == "all_gather":
            run_all_gather(seed, W, n, dtype, DIST[dtype], inplace=rnd.random() < 0.3 and opt["misalign"] == 0, **opt)
        elif kind == "broadcast":
            run_broadcast(seed, W, n, dtype, DIST[dtype], seed % W, inplace=rnd.random() < 0.3, **opt)
        else:
            run_alltoall(seed, W, n, dtype, DIST[dtype], **opt)


@pytest.mark.parametrize("batch", range(6))
def test_random_configurations(batch):
    rnd = random.Random(20260 + batch)
    for i in range(50):
        seed = 5000 + 100 * batch + i
        _run(_case(rnd), seed)
