#!/usr/bin/env python3
"""Benchmark of the ring All-Reduce hot path on one MI355X.

One "step" is one complete ring All-Reduce (every Reduce-Scatter and All-Gather
step of all W simulated ranks) over one batch of seeded synthetic rank buffers
that are already resident in HBM.  Prints ONE JSON line:

  value        S / t in GB/s  (S = bytes per rank buffer: the collective's
               algorithm bandwidth with one GPU doing all W ranks' work)
  roofline     the dominant kernel's algorithmic HBM bytes per launch divided
               by its average launch duration, against 8 TB/s.  The duration
               comes from HIP events the library records, inside the timed
               region and on the stream the launches run on, around each phase
               of a step (Reduce-Scatter launches, All-Gather launches); with
               --per-launch-events around every single launch instead
  cpu_baseline the CPU oracle timed on a bounded sample of the same workload

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]
                       [--sched stepwise|fused] [--fuse-rs-ag] [--no-cpu-baseline]
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
KERNEL_SOURCES = ["paper_2601_22585_amd/csrc/reduce_copy.hip", "paper_2601_22585_amd/csrc/reduce_copy.h"]


def kernel_source_hash():
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, f), "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 counter runs, or None
    when there are none for this kernel / workload or the kernel source has
    changed since they were taken."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    try:
        rec = json.load(open(path))
    except Exception:
        return None
    for e in rec.get("entries", []):
        if e.get("kernel") == kernel and e.get("workload") == workload and e.get("source_hash") == kernel_source_hash():
            return e.get("hbm_bytes_per_launch")
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 5])
    ap.add_argument("--sched", default="stepwise", choices=["stepwise", "fused"])
    ap.add_argument("--fuse-rs-ag", action="store_true")
    ap.add_argument("--inplace", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="record no events inside the timed region")
    ap.add_argument("--per-launch-events", action="store_true",
                    help="bracket every launch (about 3 us each) instead of each phase")
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--blocks", type=int, default=0)
    ap.add_argument("--unroll", type=int, default=0)
    ap.add_argument("--nontemporal", type=int, default=0)
    ap.add_argument("--chunk-bytes", type=int, default=-1)
    ap.add_argument("--cpu-sample-div", type=int, default=1, help="oracle sample = leading 1/div of every block")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU: all W ranks are simulated in one MI355X's memory; "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as wl
    from paper_2601_22585_amd import hcl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    hcl.lib()

    cfg = wl.CONFIGS[args.config]
    W, dtype, count = cfg["W"], cfg["dtype"], cfg["count"]
    es = wl.ESIZE[dtype]
    chunk_bytes = cfg["chunk_bytes"] if args.chunk_bytes < 0 else args.chunk_bytes
    xport = cfg.get("xport", "direct")
    S = count * es
    B = -(-count // W)

    # seeded inputs, generated on the device
    send = [torch.empty(count, dtype=wl.TORCH_DTYPE[dtype], device="cuda") for _ in range(W)]
    for r in range(W):
        wl.fill_rank(send[r], wl.rank_seed(args.config, r), cfg["dist"])
    recv = send if args.inplace else [torch.empty_like(t) for t in send]
    opt = dict(sched=args.sched, xport=xport, threads=args.threads, blocks=args.blocks, unroll=args.unroll,
               nontemporal=args.nontemporal, fuse_rs_ag=args.fuse_rs_ag)
    stage = None
    if xport == "host_staged":
        nb = hcl.host_stage_bytes(hcl.KIND_ALLREDUCE, W, count, wl.DTYPE_CODE[dtype], chunk_bytes, xport=xport)
        stage = torch.empty(nb, dtype=torch.uint8, pin_memory=True)
        opt["host_stage"] = stage
    torch.cuda.synchronize()

    # ---- CPU oracle on a bounded sample (also the parity check of the first run) ----
    cpu_baseline = None
    m = max(1, B // max(1, args.cpu_sample_div))           # leading m elements of every block
    sample_idx = [(min(c * B, count), min(min(c * B, count) + m, min((c + 1) * B, count))) for c in range(W)]
    if not args.no_cpu_baseline:
        from oracle import ring_oracle as orc
        assert count % W == 0, "the sampled replay assumes equal blocks"
        work = [np.concatenate([wl.to_wire(send[r][lo:hi]) for lo, hi in sample_idx]) for r in range(W)]
        ce = min(chunk_bytes // es, m) if chunk_bytes else 0
        # one thread first, on an eighth of the sample, then every host core on all of it
        m1 = max(1, m // 8)
        small = [np.concatenate([w[c * m:c * m + m1] for c in range(W)]) for w in work]
        orc.set_threads(1)
        t0 = time.perf_counter()
        orc.allreduce_inplace(small, wl.DTYPE_CODE[dtype], chunk_elems=min(ce, m1))
        t_one = time.perf_counter() - t0
        del small
        threads = orc.set_threads(os.cpu_count() or 1)
        t0 = time.perf_counter()
        orc.allreduce_inplace(work, wl.DTYPE_CODE[dtype], chunk_elems=ce)
        t_cpu = time.perf_counter() - t0
        sample_bytes = W * m * es
        cpu_baseline = {"value": round(sample_bytes / t_cpu / 1e9, 6), "unit": "GB/s", "cores": threads, "kind": "oracle",
                        "sample": f"leading {m} of {B} elements of each of the {W} blocks of all {W} rank buffers "
                                  f"({sample_bytes / 2**20:.0f} MiB per rank), ring replayed in {t_cpu:.2f} s",
                        "seconds": round(t_cpu, 3),
                        "one_thread": {"value": round(W * m1 * es / t_one / 1e9, 6), "unit": "GB/s",
                                       "sample_MiB_per_rank": round(W * m1 * es / 2**20, 1), "seconds": round(t_one, 3)}}

    # ---- warm-up (the first run is also checked against the oracle sample) ----
    for i in range(max(1, args.warmup)):
        launches = hcl.allreduce_sim(send, recv, chunk_bytes=chunk_bytes, **opt)
        if i == 0:
            torch.cuda.synchronize()
            if cpu_baseline is not None:
                for r in range(W):
                    got = np.concatenate([wl.to_wire(recv[r][lo:hi]) for lo, hi in sample_idx])
                    if not wl.bits_equal_nan_aware(got, work[r], dtype).all():
                        raise SystemExit(f"bench.py: rank {r} differs from the CPU oracle on the sampled elements")
                cpu_baseline["parity"] = "bit-exact on the sample"
                del work
            if args.inplace:   # keep values bounded: refill before timing
                for r in range(W):
                    wl.fill_rank(send[r], wl.rank_seed(args.config, r), cfg["dist"])
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps ----
    K = args.steps
    phase_mode = not args.per_launch_events
    n_phases = 1 if args.sched == "fused" else 2
    per = (n_phases if phase_mode else launches) + 1
    ev = None if args.no_events else hcl.EventList(K * per)
    stream = torch.cuda.current_stream()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        o = dict(opt)
        if ev is not None:
            o["events"] = (ev, k * per, per)
            o["events_per_phase"] = phase_mode
        hcl.allreduce_sim(send, recv, chunk_bytes=chunk_bytes, stream=stream, **o)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0
    ms_per_step = t_total / K * 1e3

    # ---- average launch duration of the dominant kernel ----
    staged = xport == "host_staged"
    fuse = args.fuse_rs_ag and not staged
    if args.sched == "fused":
        kernel = f"ring_fused_vec<{dtype},W={W}>"
        bytes_per_launch = 2 * W * S          # every rank's vector read once, written once
        call_bytes = 2 * W * S
        n_dom = 1                              # launches of the dominant kernel per step
        dom = [0]                              # their indices among a step's launches
    else:
        # a Reduce-Scatter launch reads two blocks and writes one per rank: 3 * S bytes
        kernel = f"reduce_copy_vec<{dtype},NSRC=2,NDST=1>"
        bytes_per_launch = 3 * S
        call_bytes = 5 * (W - 1) * S - (S if fuse else 0)
        first_rs = 1 if staged else 0
        n_dom = W - 1
        dom = list(range(first_rs, first_rs + n_dom))
    roof = None
    if ev is not None:
        if phase_mode:
            # phase 0 holds the W-1 Reduce-Scatter launches (the fused last one, 4/3 of the bytes of a
            # plain one, and the staged pre-step are counted by their share of bytes)
            rs_ms = [ev.elapsed_ms(k * per, k * per + 1) for k in range(K)]
            if args.sched == "fused":
                units = 1.0
            else:
                units = (W - 1) + (1.0 / 3.0 if fuse else 0.0) + (2.0 / 3.0 if staged else 0.0)
            avg_ms = sum(rs_ms) / len(rs_ms) / units
            timed = K * n_dom
            how = "phase events: (time of the phase's launches, gaps included) / launches"
        else:
            durs = [ev.elapsed_ms(k * per + i, k * per + i + 1) for k in range(K) for i in dom]
            avg_ms = sum(durs) / len(durs)
            timed = len(durs)
            how = "one event pair per launch"
        achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": stored_traffic(kernel, cfg["name"]),
                "bytes_per_launch": bytes_per_launch, "avg_launch_ms": round(avg_ms, 5), "launches_timed": timed,
                "timing": how}
        if staged:
            roof["note"] = "staged transport: the link to host memory, not HBM, bounds this path"
        ev.close()

    value = S / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "ring all-reduce algorithm GB/s on 1 MI355X",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": cfg["name"], "W": W, "count_per_rank": count, "bytes_per_rank": S,
                   "chunk_bytes": chunk_bytes, "sched": args.sched, "xport": xport, "fuse_rs_ag": bool(args.fuse_rs_ag),
                   "inplace": bool(args.inplace), "launches_per_step": launches},
        "algbw_rank_equiv_GBps": round(W * value, 2),
        "call_hbm_GBps": round(call_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "call_hbm_frac_of_peak": round(call_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": roof, "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
