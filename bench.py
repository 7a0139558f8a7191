#!/usr/bin/env python3
"""Benchmark of the ring collectives' hot path on one MI355X.

Default run: one "step" is one complete ring All-Reduce (every Reduce-Scatter
and All-Gather step of all W simulated ranks) of the headline workload -- W = 8
ranks, 256 MiB of bf16 per rank, 4 MiB chunks -- over seeded synthetic rank
buffers that are already resident in HBM.  Prints ONE JSON line:

  value        S / t in GB/s  (S = bytes per rank buffer: the collective's
               algorithm bandwidth with one GPU doing all W ranks' work)
  roofline     the dominant kernel's algorithmic HBM bytes per launch divided
               by its average launch duration, against 8 TB/s.  The duration
               comes from HIP events the library records, inside the timed
               region and on the stream the launches run on, around each phase
               of a step (Reduce-Scatter launches, All-Gather launches); with
               --per-launch-events around every single launch instead
  cpu_baseline the CPU oracle timed on a bounded sample of the same workload,
               whose result is also bit-compared with the GPU's first run

Other workloads (not bench lines of their own):
  --config 1            4 ranks, 1 MiB fp32
  --config 3 --bytes-per-rank N   fp16, 16 ranks, message-size sweep point
  --config 4 | 41       ZeRO-style Reduce-Scatter then All-Gather, bf16 | int32,
                        --shard-elems to scale the 2 GiB shards down
  --config 5            host-staged All-Reduce, 512 MiB fp32 per rank
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X datasheet, HBM3E
KERNEL_SOURCES = ["paper_2601_22585_amd/csrc/reduce_copy.hip", "paper_2601_22585_amd/csrc/ring_fused.hip",
                  "paper_2601_22585_amd/csrc/wire.h", "paper_2601_22585_amd/csrc/reduce_copy.h"]


def kernel_source_hash():
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, f), "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 counter runs, or None
    when there are none for this kernel / workload or the kernel source has
    changed since they were taken."""
    path = os.path.join(ROOT, "profiles", "traffic.md")
    if not os.path.exists(path):
        return None
    try:
        text = open(path).read()
        rec = json.loads(text.split("```json", 1)[1].split("```", 1)[0])
    except Exception:
        return None
    for e in rec.get("entries", []):
        if e.get("kernel") == kernel and e.get("workload") == workload and e.get("source_hash") == kernel_source_hash():
            return e.get("hbm_bytes_per_launch")
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 41, 5])
    ap.add_argument("--op", default=None, choices=["allreduce", "reduce_scatter", "all_gather", "reduce", "broadcast", "alltoall"],
                    help="collective to time (default: the config's; config 4 times reduce_scatter unless told otherwise)")
    ap.add_argument("--sched", default="stepwise", choices=["stepwise", "fused"])
    ap.add_argument("--fuse-rs-ag", action="store_true")
    ap.add_argument("--accumulate", default="per_hop", choices=["per_hop", "fp32"],
                    help="fp32: fused sums with binary32 accumulation and one rounding (a reordered-class result)")
    ap.add_argument("--reduce-op", default="sum", choices=["sum", "prod", "max", "min"],
                    help="reduction operator of the reducing collectives")
    ap.add_argument("--order", default="ring", choices=["ring", "tree"],
                    help="tree: fused reductions over a neighbours-first tree (a reordered-class result)")
    ap.add_argument("--inplace", action="store_true")
    ap.add_argument("--bytes-per-rank", type=int, default=0,
                    help="config 3: bytes per rank buffer; configs 1, 2, 5: the same workload at this size")
    ap.add_argument("--shard-elems", type=int, default=0, help="config 4: elements per shard (default 2 GiB worth)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-elems", type=int, default=1 << 24,
                    help="oracle sample: at most this many leading elements of every block")
    ap.add_argument("--no-events", action="store_true", help="record no events inside the timed region")
    ap.add_argument("--per-launch-events", action="store_true",
                    help="bracket every launch (about 3 us each) instead of each phase")
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--blocks", type=int, default=0)
    ap.add_argument("--unroll", type=int, default=0)
    ap.add_argument("--nontemporal", type=int, default=0)
    ap.add_argument("--chunk-bytes", type=int, default=-1)
    ap.add_argument("--graph", action="store_true",
                    help="capture one call into a HIP graph and time K replays (latency regime; no events)")
    ap.add_argument("--pad-bytes", type=int, default=0,
                    help="gap between consecutive rank buffers inside the one allocation they are carved from "
                         "(a multiple of 256; layout experiments)")
    ap.add_argument("--separate-allocations", action="store_true",
                    help="give every rank buffer an allocation of its own instead of carving all of them out of one")
    ap.add_argument("--chains", type=int, default=1, choices=[1, 2],
                    help="2: stepwise schedule with the chunk range split over two streams (opts.aux_stream)")
    ap.add_argument("--slab-bytes", type=int, default=0,
                    help="opts.slab_bytes: 0 = library default (a step's output per slab fits the last-level cache), -1 = no slabs")
    ap.add_argument("--no-cache-free-probe", action="store_true",
                    help="default workload only: skip the extra measurement of the dominant kernel at a footprint far beyond the last-level cache")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU: all W ranks are simulated in one MI355X's memory; "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as wl
    from paper_2601_22585_amd import hcl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    hcl.lib()   # raises if the HIP library has not been built: there is no fallback

    cfg = dict(wl.CONFIGS[args.config])
    W, dtype = cfg["W"], cfg["dtype"]
    es = wl.ESIZE[dtype]
    code = wl.DTYPE_CODE[dtype]
    xport = cfg.get("xport", "direct")
    op = args.op or ("reduce_scatter" if cfg["op"] == "rs+ag" else "allreduce")
    name = cfg["name"]
    if args.config == 3:
        nbytes = args.bytes_per_rank or (256 << 20)
        count = nbytes // es
        name = f"{name}_{nbytes}B"
        chunk_default = min(-(-count // W) * es, cfg["chunk_bytes"])
    elif args.config in (4, 41):
        shard = args.shard_elems or cfg["count"] // W
        count = shard * W
        if args.shard_elems:
            name = f"{name}_shard{shard}"
        chunk_default = cfg["chunk_bytes"]
    else:
        count = cfg["count"]
        chunk_default = cfg["chunk_bytes"]
        if args.bytes_per_rank:          # the same workload family at another message size
            count = args.bytes_per_rank // es
            name = f"{name}_resized_{args.bytes_per_rank}B"
            chunk_default = min(-(-count // W) * es, cfg["chunk_bytes"])
    chunk_bytes = chunk_default if args.chunk_bytes < 0 else args.chunk_bytes
    S = count * es                 # bytes of a full vector (per rank)
    B = -(-count // W)             # elements per block
    if op != "allreduce":
        assert count % W == 0
        name = f"{name}:{op}"

    # ---- buffers: seeded inputs generated on the device ----
    # All rank buffers (and the workspace) are carved out of ONE allocation at fixed relative
    # offsets, in the order they are asked for, each starting on a 256-byte boundary: where the
    # buffers lie relative to each other is then the same in every process.
    assert args.pad_bytes % 256 == 0
    plan = []          # (elements, dtype) in request order; filled in by new(), resolved by carve()

    class Slot:
        def __init__(self, n, td):
            self.n, self.td, self.t = n, td, None

    def new(n, td=None):
        sl = Slot(n, td or wl.TORCH_DTYPE[dtype])
        plan.append(sl)
        return sl

    def carve():
        if args.separate_allocations:
            for sl in plan:
                sl.t = torch.empty(sl.n, dtype=sl.td, device="cuda")
            return None
        offs, total = [], 0
        for sl in plan:
            offs.append(total)
            nb = sl.n * torch.empty(0, dtype=sl.td).element_size()
            total += -(-nb // 256) * 256 + args.pad_bytes
        arena = torch.empty(total, dtype=torch.uint8, device="cuda")
        for sl, o in zip(plan, offs):
            nb = sl.n * torch.empty(0, dtype=sl.td).element_size()
            sl.t = arena[o:o + nb].view(sl.td)
        return arena

    opt = dict(sched=args.sched, xport=xport, threads=args.threads, blocks=args.blocks, unroll=args.unroll,
               nontemporal=args.nontemporal)
    if args.slab_bytes:
        opt["slab_bytes"] = args.slab_bytes
    if args.accumulate != "per_hop":
        opt["accumulate"] = args.accumulate
    if args.order != "ring":
        opt["order"] = args.order
    reducing = op in ("allreduce", "reduce_scatter", "reduce")
    if args.reduce_op != "sum":
        assert reducing, "--reduce-op applies to allreduce, reduce_scatter and reduce"
        opt["op"] = args.reduce_op
    ws_slot = None
    if op == "allreduce":
        opt["fuse_rs_ag"] = args.fuse_rs_ag
        send_s = [new(count) for _ in range(W)]
        recv_s = send_s if args.inplace else [new(count) for _ in range(W)]
        kind = hcl.KIND_ALLREDUCE
        call = hcl.allreduce_sim
        per_call_count = count
    elif op == "reduce_scatter":
        send_s = [new(count) for _ in range(W)]
        recv_s = None if args.inplace else [new(B) for _ in range(W)]
        kind = hcl.KIND_REDUCE_SCATTER
        call = hcl.reduce_scatter_sim
        per_call_count = B
        if not args.inplace:
            wsb = hcl.workspace_bytes(kind, W, B, code, chunk_bytes, sched=args.sched, xport=xport)
            if wsb:
                ws_slot = new(wsb, torch.uint8)
    elif op == "all_gather":
        recv_s = [new(count) for _ in range(W)]
        send_s = None if args.inplace else [new(B) for _ in range(W)]
        kind = hcl.KIND_ALL_GATHER
        call = hcl.all_gather_sim
        per_call_count = B
    elif op == "reduce":
        send_s = [new(count) for _ in range(W)]
        recv_s = [send_s[0] if args.inplace else new(count)] + [None] * (W - 1)
        kind = hcl.KIND_REDUCE
        call = lambda s_, r_, **kw: hcl.reduce_sim(s_, r_, 0, **kw)
        per_call_count = count
        wsb = hcl.workspace_bytes(kind, W, count, code, chunk_bytes, sched=args.sched)
        if wsb:
            ws_slot = new(wsb, torch.uint8)
    elif op == "broadcast":
        recv_s = [new(count) for _ in range(W)]
        send_s = [recv_s[0] if args.inplace else new(count)] + [None] * (W - 1)
        kind = hcl.KIND_BROADCAST
        call = lambda s_, r_, **kw: hcl.broadcast_sim(s_, r_, 0, **kw)
        per_call_count = count
    else:
        send_s = [new(count) for _ in range(W)]
        recv_s = [new(count) for _ in range(W)]
        kind = hcl.KIND_ALLTOALL
        call = hcl.alltoall_sim
        per_call_count = B
    arena = carve()
    tens = lambda slots: None if slots is None else [None if x is None else x.t for x in slots]
    send, recv = tens(send_s), tens(recv_s)
    if op == "reduce_scatter" and args.inplace:
        recv = [send[r][r * B:(r + 1) * B] for r in range(W)]
    if op == "all_gather" and args.inplace:
        send = [recv[r][r * B:(r + 1) * B] for r in range(W)]
    if ws_slot is not None:
        opt["workspace"] = ws_slot.t
    aux = None
    if args.chains == 2:
        assert args.sched == "stepwise", "--chains 2 applies to the stepwise schedule"
        aux = (torch.cuda.Stream(), hcl.EventList(2))
        opt["aux_stream"], opt["aux_events"] = aux

    def refill():
        for r in range(W):
            if send[r] is not None:
                wl.fill_rank(send[r], wl.rank_seed(args.config, r), cfg["dist"])

    refill()
    if xport == "host_staged":
        nb = hcl.host_stage_bytes(kind, W, per_call_count, code, chunk_bytes, xport=xport)
        opt["host_stage"] = torch.empty(nb, dtype=torch.uint8, pin_memory=True)
    torch.cuda.synchronize()

    # ---- CPU oracle on a bounded sample: leading m elements of every block ----
    cpu_baseline = None
    m = min(B, max(1, args.cpu_sample_elems))
    win = [(min(c * B, count), min(min(c * B, count) + m, min((c + 1) * B, count))) for c in range(W)]
    want = None
    if not args.no_cpu_baseline:
        from oracle import ring_oracle as orc
        assert count % W == 0, "the sampled replay assumes equal blocks"
        ce = min(chunk_bytes // es, m) if chunk_bytes else 0
        if op == "all_gather":
            ins = [wl.to_wire(send[r][:m]) for r in range(W)]
        elif op == "broadcast":
            ins = [np.concatenate([wl.to_wire(send[0][lo:hi]) for lo, hi in win])]
        else:
            ins = [np.concatenate([wl.to_wire(send[r][lo:hi]) for lo, hi in win]) for r in range(W)]
        wide = args.accumulate == "fp32"
        oop = {"sum": orc.SUM, "prod": orc.PROD, "max": orc.MAX, "min": orc.MIN}[args.reduce_op]
        # the closed-form replay for the reordered modes; otherwise the ring as message passing
        rkw = dict(op=oop, order=orc.ORDER_TREE if args.order == "tree" else orc.ORDER_RING,
                   rounding=orc.ROUND_ONCE if wide else orc.ROUND_EACH, W=W, root=0)
        if op in ("all_gather", "broadcast", "alltoall"):
            rkw.update(op=orc.SUM, order=orc.ORDER_RING, rounding=orc.ROUND_EACH)
        # one thread first, on an eighth of the sample, then every host core on all of it; the
        # clock runs around the replay only (working copies are made before it starts)
        m1 = max(1, m // 8)
        if op == "all_gather":
            small = [a[:m1] for a in ins]
        else:
            small = [np.concatenate([a[c * m:c * m + m1] for c in range(W)]) for a in ins]
        orc.set_threads(1)
        _, t_one = orc.replay_timed(op, small, code, chunk_elems=min(ce, m1), **rkw)
        del small
        threads = orc.set_threads(os.cpu_count() or 1)
        want, t_cpu = orc.replay_timed(op, ins, code, chunk_elems=ce, **rkw)
        del ins
        sample_bytes = W * m * es      # bytes of the sampled full vector, per rank
        cpu_baseline = {"value": round(sample_bytes / t_cpu / 1e9, 6), "unit": "GB/s", "cores": threads, "kind": "oracle",
                        "sample": f"{op}: leading {m} of {B} elements of each of the {W} blocks of every rank "
                                  f"({sample_bytes / 2**20:.1f} MiB of vector per rank), replayed in {t_cpu:.2f} s "
                                  f"(wall clock around the replay only)",
                        "seconds": round(t_cpu, 3),
                        "one_thread": {"value": round(W * m1 * es / t_one / 1e9, 6), "unit": "GB/s",
                                       "sample_MiB_per_rank": round(W * m1 * es / 2**20, 2), "seconds": round(t_one, 3)}}

    def check_first_run():
        for r in range(1 if op == "reduce" else W):
            if op == "reduce_scatter":
                got = wl.to_wire(recv[r][:m])
            else:
                got = np.concatenate([wl.to_wire(recv[r][lo:hi]) for lo, hi in win])
            if not wl.bits_equal_nan_aware(got, want[r], dtype).all():
                raise SystemExit(f"bench.py: {op}: rank {r} differs from the CPU oracle on the sampled elements")
        cpu_baseline["parity"] = "bit-exact on the sample"

    # ---- warm-up (the first run is also checked against the oracle sample) ----
    clobbers = args.inplace and op in ("allreduce", "reduce_scatter", "reduce")
    launches = 0
    for i in range(max(1, args.warmup)):
        launches = call(send, recv, chunk_bytes=chunk_bytes, **opt)
        if i == 0:
            torch.cuda.synchronize()
            if want is not None:
                check_first_run()
                want = None
            if clobbers:   # in-place sums overwrite their inputs: start the timed runs from fresh values
                refill()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps ----
    K = args.steps
    phase_mode = not args.per_launch_events
    n_phases = 2 if (op == "allreduce" and args.sched == "stepwise" and W > 1) else 1
    per = (n_phases if phase_mode else launches) + 1
    ev = None if (args.no_events or args.graph or launches == 0) else hcl.EventList(K * per)
    stream = torch.cuda.current_stream()
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            call(send, recv, chunk_bytes=chunk_bytes, **opt)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(K):
            graph.replay()
        torch.cuda.synchronize()
        t_total = time.perf_counter() - t0
    else:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(K):
            o = dict(opt)
            if ev is not None:
                o["events"] = (ev, k * per, per)
                o["events_per_phase"] = phase_mode
            call(send, recv, chunk_bytes=chunk_bytes, stream=stream, **o)
        torch.cuda.synchronize()
        t_total = time.perf_counter() - t0
    ms_per_step = t_total / K * 1e3

    # ---- algorithmic bytes: of the whole call, and of one launch of the dominant kernel ----
    staged = xport == "host_staged"
    fuse = bool(opt.get("fuse_rs_ag")) and not staged
    if op == "alltoall":
        # every rank's W blocks read once and written once; a stepwise launch moves one block per rank
        kernel = "reduce_copy_vec<copy,NSRC=1,NDST=1>"
        call_bytes = 2 * W * S
        bytes_per_launch = call_bytes / launches
        n_dom, dom, units = launches, list(range(launches)), float(launches)
    elif args.sched == "fused":
        general = args.reduce_op != "sum" or args.order == "tree"
        kernel = ((f"ring_fused_gen<{dtype},W={W}>" if general else f"ring_fused_vec<{dtype},W={W}>")
                  if reducing else "gather_fused_vec")
        call_bytes = 2 * W * S if op == "allreduce" else (W + 1) * S
        bytes_per_launch, n_dom, dom, units = call_bytes, 1, [0], 1.0
    elif op == "broadcast":
        # W - 1 hops of the whole vector (S read, S written each); out of place one more copy, in the first launch
        kernel = "reduce_copy_vec<copy,NSRC=1,NDST=1>"
        own_copy = 0 if args.inplace else 2 * S
        call_bytes = 2 * (W - 1) * S + own_copy
        bytes_per_launch = 2 * S
        n_dom, dom = W - 1, list(range(1, launches))
        units = (W - 1) + (0 if args.inplace else 1)
    elif op == "all_gather":
        kernel = "reduce_copy_vec<copy,NSRC=1,NDST=1>"
        # a step copies one block per rank: S bytes read and S written, all ranks together; out of
        # place, every rank also copies its own shard into its result, which is one more such launch
        own_copy = 0 if args.inplace else 2 * S
        call_bytes = 2 * (W - 1) * S + own_copy
        bytes_per_launch = 2 * S
        n_dom, dom = W - 1, list(range(0 if args.inplace else 1, launches))
        units = (W - 1) + (0 if args.inplace else 1)
    else:
        # a Reduce-Scatter launch reads two blocks and writes one per rank: 3 * S bytes
        kernel = f"reduce_copy_vec<{dtype},NSRC=2,NDST=1>"
        bytes_per_launch = 3 * S
        first_rs = 1 if staged else 0
        n_dom = W - 1
        dom = list(range(first_rs, first_rs + n_dom))
        units = (W - 1) + (1.0 / 3.0 if fuse else 0.0) + (2.0 / 3.0 if staged else 0.0)
        call_bytes = 3 * (W - 1) * S
        if op == "allreduce":
            call_bytes = 5 * (W - 1) * S - (S if fuse else 0)
    # slabs (opts.slab_bytes): the library runs the whole ring on one slab of every block before the
    # next, so a "step" of the ring is n_slabs launches, each moving 1 / n_slabs of the step's bytes
    n_slabs = 1
    if args.sched == "stepwise" and not staged and op != "alltoall" and args.slab_bytes >= 0:
        budget = args.slab_bytes or (256 << 20)
        one_block = op in ("reduce", "broadcast")
        gran = chunk_bytes // es if chunk_bytes else 65536
        slab = max(gran, budget // ((1 if one_block else W) * es) // gran * gran)
        blk, lo, n_slabs = (count if one_block else B), 0, 0
        while lo < blk:   # the library's rule: a remainder of less than 1/32 of a slab joins the last slab
            hi = lo + slab
            if hi >= blk or blk - hi <= slab // 32:
                hi = blk
            n_slabs, lo = n_slabs + 1, hi
        n_slabs = max(1, n_slabs)
    bytes_per_launch /= n_slabs
    units *= n_slabs
    n_dom *= n_slabs
    if n_slabs > 1:
        dom = list(range(launches))
    roof = None
    if ev is not None and n_slabs > 1 and op == "allreduce":
        # with several slabs the Reduce-Scatter and All-Gather launches of a call interleave: there is
        # no phase to bracket, the figure is the whole call's
        achieved = call_bytes / (ms_per_step * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": f"reduce_copy_vec<{dtype},NSRC=2,NDST=1> and reduce_copy_vec<copy,NSRC=1,NDST=1>, every launch of the call",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": None, "bytes_per_launch": int(call_bytes / launches), "avg_launch_ms": round(ms_per_step / launches, 5),
                "launches_timed": K * launches, "timing": f"whole call / launches ({n_slabs} slabs: the phases interleave)"}
        ev.close()
    elif ev is not None:
        if phase_mode:
            # phase 0 holds the dominant kernel's launches; launches of another shape in the same
            # phase (fused last RS step, staged pre-step, own-shard copy) count by their share of bytes
            ph = [ev.elapsed_ms(k * per, k * per + 1) for k in range(K)]
            avg_ms = sum(ph) / len(ph) / units
            timed = K * n_dom
            how = "phase events: (duration of the phase's launches, gaps included) / launches"
        else:
            durs = [ev.elapsed_ms(k * per + i, k * per + i + 1) for k in range(K) for i in dom]
            avg_ms = sum(durs) / len(durs)
            timed = len(durs)
            how = "one event pair per launch"
        achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": stored_traffic(kernel, name),
                "bytes_per_launch": int(bytes_per_launch), "avg_launch_ms": round(avg_ms, 5), "launches_timed": timed,
                "timing": how}
        if staged:
            # every block that travels is written to host memory once and read back once; the host
            # link bounds this path (PCIe Gen5 x16: 64 GB/s nominal each way), not HBM
            link = (2 * (W - 1) if op == "allreduce" else (W - 1)) * S
            link_gbps = link / (ms_per_step * 1e-3) / 1e9
            roof = {"bound": "pcie", "kernel": "reduce_copy_vec with pinned-host operands", "achieved": round(link_gbps, 2),
                    "peak": 64.0, "unit": "GB/s", "frac": round(link_gbps / 64.0, 4), "traffic": None,
                    "bytes_each_way_per_step": int(link),
                    "timing": "whole step; every transfer crosses the link once in each direction",
                    "hbm_kernel": roof}
        ev.close()

    # ---- a measured copy ceiling beside the datasheet peak: the library's plain-copy kernel moving
    # the same buffers (All-to-All: every block read once and written once), outside the timed region
    if roof is not None and roof.get("bound") == "hbm" and op == "allreduce" and not args.inplace and count % W == 0 \
            and not staged and S >= (64 << 20):
        cev = hcl.EventList(2)
        reps = 5
        hcl.alltoall_sim(send, recv, chunk_bytes=chunk_bytes, stream=stream)
        cev.record(0, stream)
        for _ in range(reps):
            hcl.alltoall_sim(send, recv, chunk_bytes=chunk_bytes, stream=stream)
        cev.record(1, stream)
        torch.cuda.synchronize()
        copy_gbps = reps * 2 * W * S / (cev.elapsed_ms(0, 1) * 1e-3) / 1e9
        cev.close()
        roof["copy_ceiling"] = {"achieved": round(copy_gbps, 1), "unit": "GB/s",
                                "what": "plain copy of the same buffers by reduce_copy_vec<copy,1,1> (W launches, gaps included)",
                                "frac_of_it": round(roof["achieved"] / copy_gbps, 4)}

    # ---- the same step kernel where no cache can help: the in-place Reduce-Scatter of the ZeRO-style
    # workload (W = 8, 2 GiB blocks, 16 GiB per rank: every launch moves 48 GiB, the last-level cache
    # holds 256 MiB).  At the headline size the partial sums one step writes (256 MiB in all) are what
    # the next step reads, so part of its reads may be served from that cache, which the HBM counters
    # cannot tell apart.  Default workload only; outside the timed region.
    if (roof is not None and args.config == 2 and op == "allreduce" and args.sched == "stepwise" and not args.bytes_per_rank
            and not args.no_cache_free_probe and torch.cuda.mem_get_info()[0] > (140 << 30)):
        c4 = wl.CONFIGS[4]
        n4 = c4["count"] // c4["W"]
        big = [torch.empty(n4 * c4["W"], dtype=torch.bfloat16, device="cuda") for _ in range(c4["W"])]
        for r in range(c4["W"]):
            wl.fill_rank(big[r], wl.rank_seed(4, r), c4["dist"])
        shards = [big[r][r * n4:(r + 1) * n4] for r in range(c4["W"])]
        reps = 3
        pev = hcl.EventList(2 * (reps + 1))
        for k in range(reps + 1):
            hcl.reduce_scatter_sim(big, shards, chunk_bytes=c4["chunk_bytes"], stream=stream, slab_bytes=-1,
                                   events=(pev, 2 * k, 2), events_per_phase=True)
        torch.cuda.synchronize()
        ms4 = sum(pev.elapsed_ms(2 * k, 2 * k + 1) for k in range(1, reps + 1)) / reps / (c4["W"] - 1)
        pev.close()
        b4 = 3 * n4 * c4["W"] * 2
        roof["cache_free"] = {"workload": "cfg4_rs_ag_w8_bf16_2GiB_shard:reduce_scatter, in place, every step one pass over the whole "
                                          "2 GiB blocks (opts.slab_bytes = -1)",
                              "kernel": "reduce_copy_vec<bf16,NSRC=2,NDST=1> (one wavefront x 1 vector per workgroup at this size)",
                              "bytes_per_launch": b4, "avg_launch_ms": round(ms4, 4),
                              "achieved": round(b4 / (ms4 * 1e-3) / 1e9, 1), "unit": "GB/s",
                              "frac": round(b4 / (ms4 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        del big, shards

    value = S / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "ring all-reduce algorithm GB/s on 1 MI355X" if op == "allreduce"
                  else f"ring {op.replace('_', '-')} algorithm GB/s on 1 MI355X",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": name, "op": op, "W": W, "count_per_rank": count, "bytes_per_rank": S,
                   "chunk_bytes": chunk_bytes, "sched": args.sched, "xport": xport, "fuse_rs_ag": fuse,
                   "inplace": bool(args.inplace), "launches_per_step": launches, "graph_replay": bool(args.graph), "accumulate": args.accumulate,
                   "reduce_op": args.reduce_op if reducing else None, "order": args.order, "chains": args.chains, "slabs": n_slabs,
                   "layout": "separate allocations" if args.separate_allocations
                             else f"all buffers carved from one allocation, 256-byte aligned, {args.pad_bytes} bytes between them"},
        "algbw_rank_equiv_GBps": round(W * value, 2),
        "call_hbm_GBps": round(call_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "call_hbm_frac_of_peak": round(call_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": roof, "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
