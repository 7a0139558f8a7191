"""Host-side checks of the C ABI that need no GPU: exported symbols, argument
validation (every call here fails validation or has count == 0, so nothing is
ever enqueued), and the ring chunk scheduler against the oracle's tables."""
import ctypes
import os
import random
import re

import pytest

from oracle import ring_oracle as orc
from paper_2601_22585_amd import hcl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "hcl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(hcl_[a-z_0-9]+)\s*\(", text))
    assert declared == set(hcl.EXPORTS)
    L = hcl.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert hcl.version() == 104


def _call_ar(send, recv, W, count, dtype=hcl.FP32, op=hcl.SUM, chunk=0, **opt):
    o, keep = hcl.make_opts(W, **opt)
    ps = (ctypes.c_void_p * len(send))(*send) if send is not None else None
    pr = (ctypes.c_void_p * len(recv))(*recv) if recv is not None else None
    return hcl.lib().hcl_allreduce_sim(ps, pr, W, count, dtype, op, chunk, ctypes.byref(o), None)


def _call_rs(send, recv, W, n, dtype=hcl.FP32, chunk=0, **opt):
    o, keep = hcl.make_opts(W, **opt)
    ps, pr = (ctypes.c_void_p * W)(*send), (ctypes.c_void_p * W)(*recv)
    return hcl.lib().hcl_reduce_scatter_sim(ps, pr, W, n, dtype, hcl.SUM, chunk, ctypes.byref(o), None)


def _call_ag(send, recv, W, n, dtype=hcl.FP32, chunk=0, **opt):
    o, keep = hcl.make_opts(W, **opt)
    ps, pr = (ctypes.c_void_p * W)(*send), (ctypes.c_void_p * W)(*recv)
    return hcl.lib().hcl_all_gather_sim(ps, pr, W, n, dtype, chunk, ctypes.byref(o), None)


BASE = 0x10000000  # made-up, well separated addresses; never dereferenced


def bufs(W, stride=0x100000, base=BASE):
    return [base + r * stride for r in range(W)]


def test_allreduce_validation_codes():
    s, r = bufs(4), bufs(4, base=BASE * 2)
    assert _call_ar(s, r, 4, 0) == hcl.OK                                  # count 0: no-op
    assert _call_ar(s, r, 0, 16) == hcl.ERR_INVALID_ARG
    assert _call_ar(bufs(17), bufs(17, base=BASE * 2), 17, 16) == hcl.ERR_INVALID_ARG
    assert _call_ar(None, r, 4, 16) == hcl.ERR_INVALID_ARG
    assert _call_ar([s[0], 0, s[2], s[3]], r, 4, 16) == hcl.ERR_INVALID_ARG  # null rank buffer
    assert _call_ar([s[0] + 2, s[1], s[2], s[3]], r, 4, 16) == hcl.ERR_INVALID_ARG  # misaligned for fp32
    assert _call_ar(s, r, 4, 16, chunk=6) == hcl.ERR_INVALID_ARG           # not a multiple of 4
    assert _call_ar(s, r, 4, 16, op=4) == hcl.ERR_UNSUPPORTED                # beyond sum, prod, max, min
    assert _call_ar(s, r, 4, 16, op=-1) == hcl.ERR_UNSUPPORTED
    assert _call_ar(s, r, 4, 16, order="tree") == hcl.ERR_UNSUPPORTED         # stepwise adds in ring order
    assert _call_ar(s, r, 4, 16, sched="fused", order=2) == hcl.ERR_UNSUPPORTED
    assert _call_ar(s, r, 4, 16, dtype=7) == hcl.ERR_UNSUPPORTED
    assert _call_ar(s, r, 4, 16, ring=[0, 1, 2, 2]) == hcl.ERR_INVALID_ARG
    assert _call_ar(s, r, 4, 16, ring=[0, 1, 2, 4]) == hcl.ERR_INVALID_ARG
    assert _call_ar(s, r, 4, 16, sched=5) == hcl.ERR_UNSUPPORTED
    assert _call_ar(s, r, 4, 16, accumulate="fp32") == hcl.ERR_UNSUPPORTED     # stepwise has no such mode
    assert _call_ar(s, r, 4, 16, sched="fused", accumulate=3) == hcl.ERR_UNSUPPORTED
    assert _call_ar(s, r, 4, 16, xport=5) == hcl.ERR_UNSUPPORTED
    assert _call_ar(s, r, 4, 16, threads=100) == hcl.ERR_INVALID_ARG
    assert _call_ar(s, r, 4, 16, unroll=3) == hcl.ERR_INVALID_ARG
    assert _call_ar(s, r, 4, 16, nontemporal=3) == hcl.ERR_INVALID_ARG
    assert _call_ar(s, r, 4, 2**62) == hcl.ERR_INVALID_ARG                 # byte size overflows
    assert "overflow" in hcl.lib().hcl_last_error().decode()


def test_second_stream_validation():
    """aux_stream: STEPWISE only, distinct from the call's stream, two events alongside."""
    s, r = bufs(4), bufs(4, base=BASE * 2)
    ps, pr = (ctypes.c_void_p * 4)(*s), (ctypes.c_void_p * 4)(*r)
    ev = (ctypes.c_void_p * 2)(0x1000, 0x2000)

    def call(sched, aux, events, stream=None, count=16):
        o, keep = hcl.make_opts(4, sched=sched)
        o.aux_stream = aux
        o.aux_events = ctypes.cast(events, ctypes.POINTER(ctypes.c_void_p)) if events is not None else None
        return hcl.lib().hcl_allreduce_sim(ps, pr, 4, count, hcl.FP32, hcl.SUM, 0, ctypes.byref(o), stream)

    assert call("fused", 0x5000, ev) == hcl.ERR_UNSUPPORTED
    assert call("stepwise", 0x5000, None) == hcl.ERR_INVALID_ARG
    assert call("stepwise", 0x5000, (ctypes.c_void_p * 2)(0x1000, 0)) == hcl.ERR_INVALID_ARG
    assert call("stepwise", 0x5000, ev, stream=0x5000) == hcl.ERR_INVALID_ARG
    assert call("stepwise", 0x5000, ev, count=0) == hcl.OK              # nothing to do, nothing forked


def test_allreduce_alias_rules():
    s = bufs(4)
    # partially in place
    assert _call_ar(s, [s[0], s[1], BASE * 2, BASE * 3], 4, 16) == hcl.ERR_ALIAS
    # recv of one rank overlaps send of another
    assert _call_ar(s, [s[1] + 16, BASE * 2, BASE * 3, BASE * 4], 4, 16) == hcl.ERR_ALIAS
    # two recv buffers overlap
    assert _call_ar(s, [BASE * 2, BASE * 2 + 32, BASE * 3, BASE * 4], 4, 16) == hcl.ERR_ALIAS
    # in place with overlapping ranks
    t = [BASE, BASE + 32, BASE + 0x1000, BASE + 0x2000]
    assert _call_ar(t, t, 4, 16) == hcl.ERR_ALIAS


def test_staging_and_workspace_rules():
    s, r = bufs(8), bufs(8, base=BASE * 2)
    # fused schedule has no staged transport
    assert _call_ar(s, r, 8, 64, sched="fused", xport="host_staged") == hcl.ERR_UNSUPPORTED
    # staged transport without staging memory
    assert _call_ar(s, r, 8, 64, xport="host_staged") == hcl.ERR_WORKSPACE
    # out-of-place stepwise reduce-scatter without workspace
    assert _call_rs(s, r, 8, 64) == hcl.ERR_WORKSPACE
    assert "workspace" in hcl.lib().hcl_last_error().decode()
    # partially in-place reduce-scatter / all-gather
    rs_recv = [s[k] + k * 64 * 4 for k in range(8)]
    rs_recv[3] = BASE * 3
    assert _call_rs(s, rs_recv, 8, 64) == hcl.ERR_ALIAS
    ag_send = [r[k] + k * 64 * 4 for k in range(8)]
    ag_send[5] = BASE * 3
    assert _call_ag(ag_send, r, 8, 64) == hcl.ERR_ALIAS
    assert _call_ag(ag_send, r, 8, 0) == hcl.OK


def test_workspace_and_host_stage_sizes():
    # out-of-place stepwise reduce-scatter: one slot per block, each one block rounded up to
    # 256 bytes plus 4 KiB (so that slots are not a power of two apart)
    skew = 4096
    assert hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, 8, 1 << 20, hcl.BF16) == 8 * ((1 << 21) + skew)
    assert hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, 8, 100, hcl.FP32) == 8 * (512 + skew)
    assert hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, 2, 1 << 20, hcl.BF16) == 0
    assert hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, 8, 1 << 20, hcl.BF16, sched="fused") == 0
    assert hcl.workspace_bytes(hcl.KIND_ALLREDUCE, 8, 1 << 20, hcl.BF16) == 0
    assert hcl.workspace_bytes(hcl.KIND_ALL_GATHER, 8, 1 << 20, hcl.BF16) == 0
    # staged: two inbox slots of one block per rank; All-Reduce blocks are ceil(count / W)
    assert hcl.host_stage_bytes(hcl.KIND_ALLREDUCE, 8, 134217728, hcl.FP32, xport="host_staged") == 8 * 2 * ((64 << 20) + skew)
    assert hcl.host_stage_bytes(hcl.KIND_ALLREDUCE, 8, 134217728, hcl.FP32) == 0
    assert hcl.host_stage_bytes(hcl.KIND_REDUCE_SCATTER, 4, 1000, hcl.FP16, xport="host_staged") == 4 * 2 * (2048 + skew)


@pytest.mark.parametrize("W", list(range(1, 17)))
def test_ring_step_matches_oracle_tables(W):
    rnd = random.Random(W)
    for trial in range(3):
        ring = None
        if trial:
            ring = list(range(W))
            rnd.shuffle(ring)
        for phase in (hcl.PHASE_RS, hcl.PHASE_AG):
            for s in range(W - 1):
                for r in range(W):
                    assert hcl.ring_step(W, ring, phase, s, r) == orc.ring_step(W, ring, phase, s, r)
    with pytest.raises(hcl.HclError):
        hcl.ring_step(W, None, hcl.PHASE_RS, W - 1, 0)
    with pytest.raises(hcl.HclError):
        hcl.ring_step(W, None, 3, 0, 0)


def test_schedule_items_counts_for_the_named_workloads():
    # 4 ranks, 1 MiB fp32, chunk = block: 2 * 3 steps * 4 ranks = 24 items
    total = sum(len(hcl.schedule_items(4, None, 262144, hcl.FP32, 262144, ph, s)) for ph in (0, 1) for s in range(3))
    assert total == 24
    # 8 ranks, 256 MiB bf16, 4 MiB chunks: 14 steps * 8 ranks * 8 chunks = 896 items
    total = sum(len(hcl.schedule_items(8, None, 134217728, hcl.BF16, 4 << 20, ph, s)) for ph in (0, 1) for s in range(7))
    assert total == 896


@pytest.mark.parametrize("W,count,chunk_elems", [(4, 1000, 0), (5, 1003, 64), (8, 7, 1), (16, 100000, 4096), (3, 2, 0)])
def test_schedule_items_cover_every_block_exactly_once(W, count, chunk_elems):
    rnd = random.Random(count)
    ring = list(range(W))
    rnd.shuffle(ring)
    B = -(-count // W)
    blk = lambda c: (min(c * B, count), min((c + 1) * B, count))
    for phase in (hcl.PHASE_RS, hcl.PHASE_AG):
        seen = {r: {} for r in range(W)}          # rank -> block -> covered element ranges
        for s in range(W - 1):
            items = hcl.schedule_items(W, ring, count, hcl.FP32, chunk_elems * 4, phase, s)
            per_rank = {}
            for it in items:
                assert it["phase"] == phase and it["step"] == s
                assert (it["send_block"], it["block"]) == orc.ring_step(W, ring, phase, s, it["rank"])
                assert it["from_rank"] == ring[(ring.index(it["rank"]) - 1) % W]
                lo, hi = blk(it["block"])
                assert it["vec_offset"] == lo + it["elem_offset"] and it["elem_count"] > 0
                assert it["vec_offset"] + it["elem_count"] <= hi
                if chunk_elems:
                    assert it["elem_offset"] == it["chunk"] * chunk_elems and it["elem_count"] <= chunk_elems
                per_rank.setdefault(it["rank"], []).append(it)
                seen[it["rank"]].setdefault(it["block"], []).append((it["elem_offset"], it["elem_count"]))
            # launch order is chunk-major
            chunks = [it["chunk"] for it in items]
            assert chunks == sorted(chunks)
        for r in range(W):
            # every rank receives W-1 distinct blocks per phase, each fully and exactly once
            nonempty = [c for c in range(W) if blk(c)[1] > blk(c)[0]]
            skipped = ring[(ring.index(r) - 1) % W] if phase == hcl.PHASE_RS else r
            assert sorted(seen[r]) == sorted(c for c in nonempty if c != skipped)
            for c, runs in seen[r].items():
                runs.sort()
                pos = 0
                for off, n in runs:
                    assert off == pos
                    pos += n
                assert pos == blk(c)[1] - blk(c)[0]


def test_other_collectives_validation_codes():
    L = hcl.lib()
    s, r = bufs(4), bufs(4, base=BASE * 2)
    ps, pr = (ctypes.c_void_p * 4)(*s), (ctypes.c_void_p * 4)(*r)
    o, keep = hcl.make_opts(4)
    # count 0 is a no-op for all three
    assert L.hcl_reduce_sim(ps, pr, 4, 0, hcl.FP32, hcl.SUM, 0, 0, ctypes.byref(o), None) == hcl.OK
    assert L.hcl_broadcast_sim(ps, pr, 4, 0, hcl.FP32, 0, 0, ctypes.byref(o), None) == hcl.OK
    assert L.hcl_alltoall_sim(ps, pr, 4, 0, hcl.FP32, 0, ctypes.byref(o), None) == hcl.OK
    # bad root, bad op, missing workspace, staged transport, aliasing
    assert L.hcl_reduce_sim(ps, pr, 4, 16, hcl.FP32, hcl.SUM, 4, 0, ctypes.byref(o), None) == hcl.ERR_INVALID_ARG
    assert L.hcl_reduce_sim(ps, pr, 4, 16, hcl.FP32, 9, 0, 0, ctypes.byref(o), None) == hcl.ERR_UNSUPPORTED
    assert L.hcl_reduce_sim(ps, pr, 4, 16, hcl.FP32, hcl.SUM, 0, 0, ctypes.byref(o), None) == hcl.ERR_WORKSPACE
    assert L.hcl_broadcast_sim(ps, pr, 4, 16, hcl.FP32, -1, 0, ctypes.byref(o), None) == hcl.ERR_INVALID_ARG
    st, keep2 = hcl.make_opts(4, xport="host_staged")
    assert L.hcl_alltoall_sim(ps, pr, 4, 16, hcl.FP32, 0, ctypes.byref(st), None) == hcl.ERR_UNSUPPORTED
    assert L.hcl_alltoall_sim(ps, ps, 4, 16, hcl.FP32, 0, ctypes.byref(o), None) == hcl.ERR_ALIAS
    pr_null = (ctypes.c_void_p * 4)(None, r[1], r[2], r[3])
    assert L.hcl_reduce_sim(ps, pr_null, 4, 16, hcl.FP32, hcl.SUM, 0, 0, ctypes.byref(o), None) == hcl.ERR_INVALID_ARG
    assert hcl.workspace_bytes(hcl.KIND_REDUCE, 8, 1 << 20, hcl.BF16) == (1 << 21) + 4096
    assert hcl.workspace_bytes(hcl.KIND_REDUCE, 8, 1 << 20, hcl.BF16, sched="fused") == 0
    assert hcl.workspace_bytes(hcl.KIND_BROADCAST, 8, 1 << 20, hcl.BF16) == 0
