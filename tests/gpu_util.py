"""Shared helpers of the GPU parity tests: run a collective through the C ABI
binding and compare every output element with the CPU oracle's bits."""
import numpy as np
import torch

import workloads as wl
from oracle import ring_oracle as orc
from paper_2601_22585_amd import hcl

CODE = wl.DTYPE_CODE


PAD = 256          # guard elements before and after every buffer the helpers allocate
GUARD_BYTE = 0xA5
_guarded = []      # (allocation, first data element, data elements) since the last check


def guarded(count, torch_dtype, misalign=0):
    """A `count`-element device buffer `misalign` elements past a 256-byte aligned address,
    with PAD guard elements on either side that check_guards() expects to find untouched."""
    base = torch.empty(PAD + misalign + count + PAD, dtype=torch_dtype, device="cuda")
    base.view(torch.uint8).fill_(GUARD_BYTE)
    _guarded.append((base, PAD + misalign, count))
    return base[PAD + misalign:PAD + misalign + count]


def check_guards():
    """No kernel may have written outside the buffers it was given (scalar tails, vectors that
    straddle the end of a misaligned buffer): every guard byte must still hold its pattern."""
    torch.cuda.synchronize()
    for base, lo, count in _guarded:
        b, es = base.view(torch.uint8), base.element_size()
        assert bool((b[:lo * es] == GUARD_BYTE).all()), "bytes before a buffer were overwritten"
        assert bool((b[(lo + count) * es:] == GUARD_BYTE).all()), "bytes after a buffer were overwritten"
    _guarded.clear()


def device_inputs(cfg_id, W, count, dtype, dist, misalign=0):
    """CPU-generated seeded inputs and their device copies.  misalign > 0 places
    every device buffer `misalign` elements past a 256-byte aligned address."""
    cpu = wl.make_inputs(cfg_id, W, count, dtype, dist)
    dev = []
    for t in cpu:
        d = guarded(count, t.dtype, misalign)
        d.copy_(t)
        dev.append(d)
    return cpu, dev


def fresh(W, count, dtype, misalign=0, fill=None):
    out = []
    for _ in range(W):
        d = guarded(count, wl.TORCH_DTYPE[dtype], misalign)
        if fill is not None:
            d.fill_(fill)
        out.append(d)
    return out


def assert_same_bits(got_t, want_np, dtype, what):
    got = wl.to_wire(got_t)
    eq = wl.bits_equal_nan_aware(got, want_np, dtype)
    if not eq.all():
        bad = np.flatnonzero(~eq)
        i = int(bad[0])
        raise AssertionError(f"{what}: {bad.size} of {got.size} elements differ; first at {i}: "
                             f"got {got[i]!r} want {want_np[i]!r}")


def pinned_stage(nbytes):
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, pin_memory=True)


def run_allreduce(cfg_id, W, count, dtype, dist, ring=None, chunk_bytes=0, inplace=False, misalign=0,
                  cpu_inputs=None, **opt):
    """Runs hcl_allreduce_sim and checks all W outputs against the oracle.  Returns launches."""
    if cpu_inputs is None:
        cpu, dev = device_inputs(cfg_id, W, count, dtype, dist, misalign)
    else:
        cpu = cpu_inputs
        dev = [_to_dev(t, misalign) for t in cpu]
    es = wl.ESIZE[dtype]
    want = orc.allreduce([wl.to_wire(t) for t in cpu], CODE[dtype], ring=ring,
                         chunk_elems=chunk_bytes // es)
    if opt.get("xport") == "host_staged":
        opt["host_stage"] = pinned_stage(hcl.host_stage_bytes(hcl.KIND_ALLREDUCE, W, count, CODE[dtype],
                                                              chunk_bytes, xport="host_staged"))
    recv = dev if inplace else fresh(W, count, dtype, misalign, fill=0)
    n = hcl.allreduce_sim(dev, recv, chunk_bytes=chunk_bytes, ring=ring, **opt)
    torch.cuda.synchronize()
    tag = f"allreduce W={W} count={count} {dtype} ring={ring} chunk={chunk_bytes} inplace={inplace} mis={misalign} {opt}"
    for r in range(W):
        assert_same_bits(recv[r], want[r], dtype, f"{tag} rank {r}")
        if not inplace:
            assert_same_bits(dev[r], wl.to_wire(cpu[r]), dtype, f"{tag} send[{r}] must stay untouched")
    check_guards()
    return n


def run_reduce_scatter(cfg_id, W, n, dtype, dist, ring=None, chunk_bytes=0, inplace=False, misalign=0, **opt):
    cpu, dev = device_inputs(cfg_id, W, W * n, dtype, dist, misalign)
    es = wl.ESIZE[dtype]
    want = orc.reduce_scatter([wl.to_wire(t) for t in cpu], CODE[dtype], ring=ring, chunk_elems=chunk_bytes // es)
    if opt.get("xport") == "host_staged":
        opt["host_stage"] = pinned_stage(hcl.host_stage_bytes(hcl.KIND_REDUCE_SCATTER, W, n, CODE[dtype],
                                                              chunk_bytes, xport="host_staged"))
    if inplace:
        recv = [dev[r][r * n:(r + 1) * n] for r in range(W)]
    else:
        recv = fresh(W, n, dtype, misalign, fill=0)
        wsb = hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, W, n, CODE[dtype], chunk_bytes,
                                  sched=opt.get("sched", "stepwise"), xport=opt.get("xport", "direct"))
        if wsb:
            opt["workspace"] = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    nl = hcl.reduce_scatter_sim(dev, recv, chunk_bytes=chunk_bytes, ring=ring, **opt)
    torch.cuda.synchronize()
    tag = f"reduce_scatter W={W} n={n} {dtype} ring={ring} chunk={chunk_bytes} inplace={inplace} mis={misalign} {opt.get('sched')} {opt.get('xport')}"
    for r in range(W):
        assert_same_bits(recv[r], want[r], dtype, f"{tag} rank {r}")
        if not inplace:
            assert_same_bits(dev[r], wl.to_wire(cpu[r]), dtype, f"{tag} send[{r}] must stay untouched")
    check_guards()
    return nl


def run_all_gather(cfg_id, W, n, dtype, dist, ring=None, chunk_bytes=0, inplace=False, misalign=0, **opt):
    cpu = wl.make_inputs(cfg_id, W, n, dtype, dist)
    es = wl.ESIZE[dtype]
    want = orc.all_gather([wl.to_wire(t) for t in cpu], CODE[dtype], ring=ring, chunk_elems=chunk_bytes // es)
    if opt.get("xport") == "host_staged":
        opt["host_stage"] = pinned_stage(hcl.host_stage_bytes(hcl.KIND_ALL_GATHER, W, n, CODE[dtype],
                                                              chunk_bytes, xport="host_staged"))
    recv = fresh(W, W * n, dtype, misalign, fill=0)
    if inplace:
        send = [recv[r][r * n:(r + 1) * n] for r in range(W)]
        for r in range(W):
            send[r].copy_(cpu[r])
    else:
        send = [_to_dev(t, misalign) for t in cpu]
    nl = hcl.all_gather_sim(send, recv, chunk_bytes=chunk_bytes, ring=ring, **opt)
    torch.cuda.synchronize()
    tag = f"all_gather W={W} n={n} {dtype} ring={ring} chunk={chunk_bytes} inplace={inplace} mis={misalign} {opt.get('sched')} {opt.get('xport')}"
    for r in range(W):
        assert_same_bits(recv[r], want[r], dtype, f"{tag} rank {r}")
    check_guards()
    return nl


def _to_dev(t, misalign=0):
    d = guarded(t.numel(), t.dtype, misalign)
    d.copy_(t)
    return d


def run_reduce(cfg_id, W, count, dtype, dist, root, ring=None, chunk_bytes=0, inplace=False, misalign=0, **opt):
    cpu = wl.make_inputs(cfg_id, W, count, dtype, dist)
    dev = [_to_dev(t, misalign) for t in cpu]
    want = orc.reduce([wl.to_wire(t) for t in cpu], CODE[dtype], root, ring=ring, chunk_elems=chunk_bytes // wl.ESIZE[dtype])
    wsb = hcl.workspace_bytes(hcl.KIND_REDUCE, W, count, CODE[dtype], chunk_bytes, sched=opt.get("sched", "stepwise"))
    if wsb:
        opt["workspace"] = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    recv = [None] * W
    recv[root] = dev[root] if inplace else fresh(1, count, dtype, misalign, fill=0)[0]
    n = hcl.reduce_sim(dev, recv, root, chunk_bytes=chunk_bytes, ring=ring, **opt)
    torch.cuda.synchronize()
    tag = f"reduce W={W} count={count} {dtype} root={root} ring={ring} chunk={chunk_bytes} inplace={inplace} mis={misalign} {opt.get('sched')}"
    assert_same_bits(recv[root], want, dtype, tag)
    for r in range(W):
        if not (inplace and r == root):
            assert_same_bits(dev[r], wl.to_wire(cpu[r]), dtype, f"{tag} send[{r}] must stay untouched")
    check_guards()
    return n


def run_broadcast(cfg_id, W, count, dtype, dist, root, ring=None, chunk_bytes=0, inplace=False, misalign=0, **opt):
    src = wl.make_inputs(cfg_id, 1, count, dtype, dist)[0]
    want = orc.broadcast(wl.to_wire(src), CODE[dtype], W, root, ring=ring)
    recv = fresh(W, count, dtype, misalign, fill=0)
    send = [None] * W
    if inplace:
        recv[root].copy_(src)
        send[root] = recv[root]
    else:
        send[root] = _to_dev(src, misalign)
    n = hcl.broadcast_sim(send, recv, root, chunk_bytes=chunk_bytes, ring=ring, **opt)
    torch.cuda.synchronize()
    tag = f"broadcast W={W} count={count} {dtype} root={root} ring={ring} chunk={chunk_bytes} inplace={inplace} mis={misalign} {opt.get('sched')}"
    for r in range(W):
        assert_same_bits(recv[r], want[r], dtype, f"{tag} rank {r}")
    check_guards()
    return n


def run_alltoall(cfg_id, W, n, dtype, dist, ring=None, chunk_bytes=0, misalign=0, **opt):
    cpu = wl.make_inputs(cfg_id, W, W * n, dtype, dist)
    dev = [_to_dev(t, misalign) for t in cpu]
    want = orc.alltoall([wl.to_wire(t) for t in cpu], CODE[dtype])
    recv = fresh(W, W * n, dtype, misalign, fill=0)
    nl = hcl.alltoall_sim(dev, recv, chunk_bytes=chunk_bytes, ring=ring, **opt)
    torch.cuda.synchronize()
    tag = f"alltoall W={W} n={n} {dtype} ring={ring} chunk={chunk_bytes} mis={misalign} {opt.get('sched')}"
    for r in range(W):
        assert_same_bits(recv[r], want[r], dtype, f"{tag} rank {r}")
        assert_same_bits(dev[r], wl.to_wire(cpu[r]), dtype, f"{tag} send[{r}] must stay untouched")
    check_guards()
    return nl
