"""Seeded synthetic inputs for the ring-collective workloads.

This module is the only code shared by the CPU oracle's tests and the GPU
path's tests / benchmark.  It holds no arithmetic of the method itself: it
draws random buffers with torch's generators, casts them with torch's own
dtype conversion, and views tensors as numpy wire arrays.

The paper's collective benchmarks move 1 GB messages and sweep 1 KB - 1 GB
(Section 5.2 "Collective communication"; Appendix E.4), its training runs
exchange FP16 / BF16 gradients (Appendix D.3) through the All-Reduce,
All-Gather and Reduce-Scatter mix of the ZeRO stages (Appendix D.4).  None of
that data is available, so gradient-shaped random buffers of the same sizes
and dtypes stand in for it.
"""
import numpy as np
import torch

KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30

TORCH_DTYPE = {"fp32": torch.float32, "bf16": torch.bfloat16, "fp16": torch.float16, "int32": torch.int32,
               "fp64": torch.float64, "int64": torch.int64, "uint8": torch.uint8}
ESIZE = {"fp32": 4, "bf16": 2, "fp16": 2, "int32": 4, "fp64": 8, "int64": 8, "uint8": 1}
DTYPE_CODE = {"fp32": 0, "bf16": 1, "fp16": 2, "int32": 3, "fp64": 4, "int64": 5, "uint8": 6}

# The five workload families.  `count` is elements per rank buffer.
CONFIGS = {
    # small all-reduce, chunk = one block
    1: dict(name="cfg1_ar_w4_fp32_1MiB", op="allreduce", W=4, dtype="fp32", count=262144,
            dist=("uniform", -1.0, 1.0), chunk_bytes=262144 * 4 // 4),
    # headline bandwidth case: gradient-like bf16, 256 MiB per rank, 4 MiB chunks
    2: dict(name="cfg2_ar_w8_bf16_256MiB", op="allreduce", W=8, dtype="bf16", count=134217728,
            dist=("normal", 0.0, 1e-3), chunk_bytes=4 * MiB),
    # message-size sweep, fp16, W = 16, 8 KiB .. 1 GiB per rank
    3: dict(name="cfg3_sweep_w16_fp16", op="allreduce", W=16, dtype="fp16", count=None,
            sizes_bytes=[1 << k for k in range(13, 31)], dist=("normal", 0.0, 1.0), chunk_bytes=4 * MiB),
    # ZeRO-style split ops (reduce-scatter, then all-gather); shard = 2^30 bf16 elements
    4: dict(name="cfg4_rs_ag_w8_bf16_2GiB_shard", op="rs+ag", W=8, dtype="bf16", count=8 * (1 << 30),
            dist=("normal", 0.0, 1e-3), chunk_bytes=4 * MiB),
    # same bytes, int32 values for exact checking
    41: dict(name="cfg4_rs_ag_w8_int32_2GiB_shard", op="rs+ag", W=8, dtype="int32", count=8 * (1 << 29),
             dist=("randint", -1000, 1000), chunk_bytes=4 * MiB),
    # host-staged all-reduce, 512 MiB fp32 per rank
    5: dict(name="cfg5_ar_w8_fp32_512MiB_host_staged", op="allreduce", W=8, dtype="fp32", count=134217728,
            dist=("uniform", -1.0, 1.0), chunk_bytes=64 * MiB, xport="host_staged"),
}


def rank_seed(cfg_id, rank):
    return 1234 + 1000 * int(cfg_id) + int(rank)


def fill_rank(out, seed, dist, slab=1 << 24):
    """Fill the 1-D tensor `out` (any supported dtype, CPU or GPU) from `seed`.
    Values are drawn in fp32 (or int64) slabs with a generator on out's device
    and cast by torch into out's dtype."""
    gen = torch.Generator(device=out.device)
    gen.manual_seed(int(seed))
    n = out.numel()
    kind = dist[0]
    for lo in range(0, n, slab):
        m = min(slab, n - lo)
        if kind == "uniform":
            t = torch.empty(m, dtype=torch.float32, device=out.device).uniform_(dist[1], dist[2], generator=gen)
        elif kind == "normal":
            t = torch.empty(m, dtype=torch.float32, device=out.device).normal_(dist[1], dist[2], generator=gen)
        elif kind == "randint":
            t = torch.randint(int(dist[1]), int(dist[2]) + 1, (m,), generator=gen, device=out.device)
            if out.dtype == torch.uint8:
                t = t & 0xFF            # two's-complement wrap into the byte range
        elif kind == "bits":
            # uniformly random bit patterns: every exponent, subnormals, infinities, NaNs, both zeros
            width = out.element_size() * 8
            if width == 8:
                out[lo:lo + m].copy_(torch.randint(0, 256, (m,), generator=gen, device=out.device))
                continue
            top = (1 << (width - 1)) - (1 if width == 64 else 0)     # randint's bound must fit int64
            raw = torch.randint(-(1 << (width - 1)), top, (m,), generator=gen, device=out.device)
            out[lo:lo + m].view({16: torch.int16, 32: torch.int32, 64: torch.int64}[width]).copy_(raw)
            continue
        else:
            raise ValueError(kind)
        out[lo:lo + m].copy_(t)
    return out


def make_inputs(cfg_id, W, count, dtype, dist, device="cpu"):
    """W rank buffers of `count` elements, rank r seeded with rank_seed(cfg_id, r)."""
    bufs = []
    for r in range(W):
        t = torch.empty(count, dtype=TORCH_DTYPE[dtype], device=device)
        bufs.append(fill_rank(t, rank_seed(cfg_id, r), dist))
    return bufs


def to_wire(t):
    """torch tensor (CPU or GPU) -> contiguous numpy wire array: float32 / float64 / int32 /
    int64 / uint8 as is, bf16 / fp16 as uint16 bit patterns."""
    t = t.detach().contiguous().cpu()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def from_wire(a, dtype, device="cpu"):
    """numpy wire array -> torch tensor of the named dtype."""
    a = np.ascontiguousarray(a)
    if dtype in ("bf16", "fp16"):
        t = torch.from_numpy(a.view(np.int16).copy()).view(TORCH_DTYPE[dtype])
    else:
        t = torch.from_numpy(a.copy())
    return t.to(device)


def bits_equal_nan_aware(got, want, dtype):
    """Element-wise equality of wire arrays where any NaN equals any NaN."""
    got, want = np.asarray(got), np.asarray(want)
    eq = got == want
    if dtype == "fp32":
        eq = (got.view(np.uint32) == want.view(np.uint32)) | (np.isnan(got) & np.isnan(want))
    elif dtype == "fp64":
        eq = (got.view(np.uint64) == want.view(np.uint64)) | (np.isnan(got) & np.isnan(want))
    elif dtype == "bf16":
        isnan = lambda x: (x & 0x7FFF) > 0x7F80
        eq = eq | (isnan(got) & isnan(want))
    elif dtype == "fp16":
        isnan = lambda x: (x & 0x7FFF) > 0x7C00
        eq = eq | (isnan(got) & isnan(want))
    return eq
