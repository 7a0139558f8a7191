"""ctypes front end of the CPU oracle (ring_oracle.c) on numpy arrays.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark; never by the product package.  It shares no
code with the HIP path and does not import it.

Wire types are passed as numpy arrays: float32 / float64 / int32 / int64 /
uint8 as themselves and uint16 bit patterns for bf16 / fp16 (numpy has no
bfloat16, and bit patterns keep comparisons exact).
"""
import ctypes
import os
import subprocess

import numpy as np

FP32, BF16, FP16, INT32, FP64, INT64, UINT8 = 0, 1, 2, 3, 4, 5, 6
PHASE_RS, PHASE_AG = 0, 1
SUM, PROD, MAX, MIN = 0, 1, 2, 3
ORDER_RING, ORDER_TREE = 0, 1
ROUND_EACH, ROUND_ONCE = 0, 1
NP_WIRE = {FP32: np.float32, BF16: np.uint16, FP16: np.uint16, INT32: np.int32,
           FP64: np.float64, INT64: np.int64, UINT8: np.uint8}

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ring_oracle.c")
_LIB = os.path.join(_HERE, "libring_oracle.so")
GCC_FLAGS = ["-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared"]


def build(force=False):
    """Compile ring_oracle.c with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *GCC_FLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        vpp = ctypes.POINTER(ctypes.c_void_p)
        ip = ctypes.POINTER(ctypes.c_int)
        L.orc_ring_step.argtypes = [ctypes.c_int, ip, ctypes.c_int, ctypes.c_int, ctypes.c_int, ip, ip]
        L.orc_allreduce.argtypes = [vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ip, ctypes.c_size_t]
        L.orc_reduce_scatter.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ip, ctypes.c_size_t]
        L.orc_all_gather.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ip, ctypes.c_size_t]
        for name in ("orc_f32_to_bf16_n", "orc_f32_to_f16_n", "orc_bf16_to_f32_n", "orc_f16_to_f32_n"):
            getattr(L, name).argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t]
            getattr(L, name).restype = None
        L.orc_hop_n.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
        L.orc_hop_n.restype = None
        L.orc_reduce.argtypes = [vpp, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ip, ctypes.c_int, ctypes.c_size_t]
        L.orc_broadcast.argtypes = [ctypes.c_void_p, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ip, ctypes.c_int]
        L.orc_alltoall.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int]
        L.orc_allreduce_fp32acc.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ip]
        L.orc_reduce_scatter_fp32acc.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ip]
        L.orc_reduce_fp32acc.argtypes = [vpp, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ip, ctypes.c_int]
        L.orc_allreduce_op.argtypes = [vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ip, ctypes.c_size_t]
        L.orc_reduce_scatter_op.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ip, ctypes.c_size_t]
        L.orc_reduce_op.argtypes = [vpp, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ip, ctypes.c_int, ctypes.c_size_t]
        L.orc_allreduce_var.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ip, ctypes.c_int, ctypes.c_int]
        L.orc_reduce_scatter_var.argtypes = L.orc_allreduce_var.argtypes
        L.orc_reduce_var.argtypes = [vpp, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ip, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.orc_hop_op_n.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int]
        L.orc_hop_op_n.restype = None
        L.orc_set_threads.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def _ring_arg(ring, W):
    if ring is None:
        return None
    ring = [int(x) for x in ring]
    assert len(ring) == W
    return (ctypes.c_int * W)(*ring)


def _ptrs(arrays):
    return (ctypes.c_void_p * len(arrays))(*[a.ctypes.data for a in arrays])


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def _wire(a, dtype):
    a = np.ascontiguousarray(a)
    assert a.dtype == NP_WIRE[dtype] and a.ndim == 1, (a.dtype, dtype)
    return a


def set_threads(n):
    """Set the OpenMP thread count (0 keeps the default); returns the count in use."""
    return lib().orc_set_threads(int(n))


def ring_step(W, ring, phase, step, rank):
    """(send_block, recv_block) of `rank` at (phase, step)."""
    sb, rb = ctypes.c_int(-1), ctypes.c_int(-1)
    _check(lib().orc_ring_step(W, _ring_arg(ring, W), phase, step, rank, ctypes.byref(sb), ctypes.byref(rb)),
           "ring_step")
    return sb.value, rb.value


def allreduce(inputs, dtype, ring=None, chunk_elems=0, op=SUM):
    """Ring All-Reduce with operator `op`.  inputs: W arrays of `count` wire elements.
    Returns W new arrays; the inputs are left untouched."""
    W = len(inputs)
    work = [_wire(a, dtype).copy() for a in inputs]
    count = work[0].size
    assert all(w.size == count for w in work)
    if op == SUM:
        _check(lib().orc_allreduce(_ptrs(work), W, count, dtype, _ring_arg(ring, W), chunk_elems), "allreduce")
    else:
        _check(lib().orc_allreduce_op(_ptrs(work), W, count, dtype, op, _ring_arg(ring, W), chunk_elems), "allreduce_op")
    return work


def allreduce_inplace(work, dtype, ring=None, chunk_elems=0):
    """Ring All-Reduce replayed in place on the W arrays in `work` (no copies:
    this is the call the timing harness brackets)."""
    W = len(work)
    for w in work:
        assert w.dtype == NP_WIRE[dtype] and w.flags.c_contiguous and w.size == work[0].size
    _check(lib().orc_allreduce(_ptrs(work), W, work[0].size, dtype, _ring_arg(ring, W), chunk_elems), "allreduce")
    return work


def reduce_scatter(inputs, dtype, ring=None, chunk_elems=0, op=SUM):
    """Ring Reduce-Scatter with operator `op`.  inputs: W arrays of W*recvcount elements.
    Returns W arrays of recvcount elements (rank r gets block r)."""
    W = len(inputs)
    work = [_wire(a, dtype).copy() for a in inputs]
    total = work[0].size
    assert total % W == 0 and all(w.size == total for w in work)
    n = total // W
    out = [np.empty(n, dtype=NP_WIRE[dtype]) for _ in range(W)]
    if op == SUM:
        _check(lib().orc_reduce_scatter(_ptrs(work), _ptrs(out), W, n, dtype, _ring_arg(ring, W), chunk_elems),
               "reduce_scatter")
    else:
        _check(lib().orc_reduce_scatter_op(_ptrs(work), _ptrs(out), W, n, dtype, op, _ring_arg(ring, W), chunk_elems),
               "reduce_scatter_op")
    return out


def all_gather(inputs, dtype, ring=None, chunk_elems=0):
    """Ring All-Gather.  inputs: W arrays of sendcount elements.
    Returns W arrays of W*sendcount elements."""
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    n = src[0].size
    assert all(s.size == n for s in src)
    out = [np.zeros(W * n, dtype=NP_WIRE[dtype]) for _ in range(W)]
    _check(lib().orc_all_gather(_ptrs(src), _ptrs(out), W, n, dtype, _ring_arg(ring, W), chunk_elems),
           "all_gather")
    return out


def reduce(inputs, dtype, root, ring=None, chunk_elems=0, op=SUM):
    """Ring Reduce with operator `op` to `root`.  inputs: W arrays of count elements.  Returns the root's result."""
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    n = src[0].size
    assert all(s.size == n for s in src)
    out = np.zeros(n, dtype=NP_WIRE[dtype])
    if op == SUM:
        _check(lib().orc_reduce(_ptrs(src), out.ctypes.data, W, n, dtype, _ring_arg(ring, W), root, chunk_elems), "reduce")
    else:
        _check(lib().orc_reduce_op(_ptrs(src), out.ctypes.data, W, n, dtype, op, _ring_arg(ring, W), root, chunk_elems),
               "reduce_op")
    return out


def broadcast(root_input, dtype, W, root, ring=None):
    """Ring Broadcast from `root`.  Returns W arrays, each a copy of root_input."""
    src = _wire(root_input, dtype)
    out = [np.zeros(src.size, dtype=NP_WIRE[dtype]) for _ in range(W)]
    _check(lib().orc_broadcast(src.ctypes.data, _ptrs(out), W, src.size, dtype, _ring_arg(ring, W), root), "broadcast")
    return out


def alltoall(inputs, dtype):
    """All-to-All.  inputs: W arrays of W*n elements.  Returns W arrays of W*n elements."""
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    total = src[0].size
    assert total % W == 0 and all(s.size == total for s in src)
    out = [np.zeros(total, dtype=NP_WIRE[dtype]) for _ in range(W)]
    _check(lib().orc_alltoall(_ptrs(src), _ptrs(out), W, total // W, dtype), "alltoall")
    return out


def allreduce_fp32acc(inputs, dtype, ring=None):
    """All-Reduce with binary32 accumulation in ring order and one final rounding."""
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    n = src[0].size
    out = [np.zeros(n, dtype=NP_WIRE[dtype]) for _ in range(W)]
    _check(lib().orc_allreduce_fp32acc(_ptrs(src), _ptrs(out), W, n, dtype, _ring_arg(ring, W)), "allreduce_fp32acc")
    return out


def reduce_scatter_fp32acc(inputs, dtype, ring=None):
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    total = src[0].size
    assert total % W == 0
    out = [np.zeros(total // W, dtype=NP_WIRE[dtype]) for _ in range(W)]
    _check(lib().orc_reduce_scatter_fp32acc(_ptrs(src), _ptrs(out), W, total // W, dtype, _ring_arg(ring, W)),
           "reduce_scatter_fp32acc")
    return out


def reduce_fp32acc(inputs, dtype, root, ring=None):
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    out = np.zeros(src[0].size, dtype=NP_WIRE[dtype])
    _check(lib().orc_reduce_fp32acc(_ptrs(src), out.ctypes.data, W, src[0].size, dtype, _ring_arg(ring, W), root),
           "reduce_fp32acc")
    return out


def allreduce_var(inputs, dtype, op=SUM, ring=None, order=ORDER_RING, rounding=ROUND_EACH):
    """All-Reduce variant: operator, order (ring / tree) and rounding (every
    intermediate result / once at the end) chosen freely.  (RING, EACH) is the ring itself."""
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    n = src[0].size
    out = [np.zeros(n, dtype=NP_WIRE[dtype]) for _ in range(W)]
    _check(lib().orc_allreduce_var(_ptrs(src), _ptrs(out), W, n, dtype, op, _ring_arg(ring, W), order, rounding),
           "allreduce_var")
    return out


def reduce_scatter_var(inputs, dtype, op=SUM, ring=None, order=ORDER_RING, rounding=ROUND_EACH):
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    total = src[0].size
    assert total % W == 0
    out = [np.zeros(total // W, dtype=NP_WIRE[dtype]) for _ in range(W)]
    _check(lib().orc_reduce_scatter_var(_ptrs(src), _ptrs(out), W, total // W, dtype, op, _ring_arg(ring, W),
                                        order, rounding), "reduce_scatter_var")
    return out


def reduce_var(inputs, dtype, root, op=SUM, ring=None, order=ORDER_RING, rounding=ROUND_EACH):
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    out = np.zeros(src[0].size, dtype=NP_WIRE[dtype])
    _check(lib().orc_reduce_var(_ptrs(src), out.ctypes.data, W, src[0].size, dtype, op, _ring_arg(ring, W), root,
                                order, rounding), "reduce_var")
    return out


def hop_op(incoming, local, dtype, op):
    """Element-wise single hop with operator `op`."""
    a, b = _wire(incoming, dtype), _wire(local, dtype)
    assert a.size == b.size
    y = np.empty_like(a)
    lib().orc_hop_op_n(a.ctypes.data, b.ctypes.data, y.ctypes.data, a.size, dtype, op)
    return y


def hop(incoming, local, dtype):
    """Element-wise single hop: round_T(f32(incoming) + f32(local))."""
    a, b = _wire(incoming, dtype), _wire(local, dtype)
    assert a.size == b.size
    y = np.empty_like(a)
    lib().orc_hop_n(a.ctypes.data, b.ctypes.data, y.ctypes.data, a.size, dtype)
    return y


def f32_to_bf16(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    y = np.empty(x.shape, np.uint16)
    lib().orc_f32_to_bf16_n(x.ctypes.data, y.ctypes.data, x.size)
    return y


def f32_to_f16(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    y = np.empty(x.shape, np.uint16)
    lib().orc_f32_to_f16_n(x.ctypes.data, y.ctypes.data, x.size)
    return y


def bf16_to_f32(x):
    x = np.ascontiguousarray(x, dtype=np.uint16)
    y = np.empty(x.shape, np.float32)
    lib().orc_bf16_to_f32_n(x.ctypes.data, y.ctypes.data, x.size)
    return y


def f16_to_f32(x):
    x = np.ascontiguousarray(x, dtype=np.uint16)
    y = np.empty(x.shape, np.float32)
    lib().orc_f16_to_f32_n(x.ctypes.data, y.ctypes.data, x.size)
    return y


def replay_timed(kind, inputs, dtype, ring=None, chunk_elems=0, op=SUM, root=0, order=ORDER_RING,
                 rounding=ROUND_EACH, W=None):
    """One collective with the wall clock around the C replay only: working copies and
    output arrays are made, and their pages touched, before the clock starts.
    kind: "allreduce" | "reduce_scatter" | "all_gather" | "reduce" | "broadcast" | "alltoall";
    (order, rounding) other than (RING, EACH) selects the closed-form variant replay.
    Returns (result as the untimed functions give it, seconds)."""
    import time
    L = lib()
    variant = order != ORDER_RING or rounding != ROUND_EACH
    ra = _ring_arg(ring, len(inputs) if kind != "broadcast" else W)
    if kind == "broadcast":
        src = _wire(inputs[0], dtype)
        out = [np.zeros(src.size, dtype=NP_WIRE[dtype]) for _ in range(W)]
        po = _ptrs(out)
        t0 = time.perf_counter()
        rc = L.orc_broadcast(src.ctypes.data, po, W, src.size, dtype, ra, root)
        dt = time.perf_counter() - t0
        _check(rc, kind)
        return out, dt
    W = len(inputs)
    src = [_wire(a, dtype) for a in inputs]
    n = src[0].size
    if kind == "allreduce" and not variant:
        work = [a.copy() for a in src]
        pw = _ptrs(work)
        t0 = time.perf_counter()
        rc = (L.orc_allreduce(pw, W, n, dtype, ra, chunk_elems) if op == SUM
              else L.orc_allreduce_op(pw, W, n, dtype, op, ra, chunk_elems))
        dt = time.perf_counter() - t0
        _check(rc, kind)
        return work, dt
    if kind == "allreduce":
        out = [np.zeros(n, dtype=NP_WIRE[dtype]) for _ in range(W)]
        ps, po = _ptrs(src), _ptrs(out)
        t0 = time.perf_counter()
        rc = L.orc_allreduce_var(ps, po, W, n, dtype, op, ra, order, rounding)
        dt = time.perf_counter() - t0
        _check(rc, kind)
        return out, dt
    if kind == "reduce_scatter":
        assert n % W == 0
        out = [np.zeros(n // W, dtype=NP_WIRE[dtype]) for _ in range(W)]
        po = _ptrs(out)
        if variant:
            ps = _ptrs(src)
            t0 = time.perf_counter()
            rc = L.orc_reduce_scatter_var(ps, po, W, n // W, dtype, op, ra, order, rounding)
        else:
            work = [a.copy() for a in src]
            pw = _ptrs(work)
            t0 = time.perf_counter()
            rc = (L.orc_reduce_scatter(pw, po, W, n // W, dtype, ra, chunk_elems) if op == SUM
                  else L.orc_reduce_scatter_op(pw, po, W, n // W, dtype, op, ra, chunk_elems))
        dt = time.perf_counter() - t0
        _check(rc, kind)
        return out, dt
    if kind == "all_gather":
        out = [np.zeros(W * n, dtype=NP_WIRE[dtype]) for _ in range(W)]
        ps, po = _ptrs(src), _ptrs(out)
        t0 = time.perf_counter()
        rc = L.orc_all_gather(ps, po, W, n, dtype, ra, chunk_elems)
        dt = time.perf_counter() - t0
        _check(rc, kind)
        return out, dt
    if kind == "reduce":
        out = np.zeros(n, dtype=NP_WIRE[dtype])
        ps = _ptrs(src)
        t0 = time.perf_counter()
        if variant:
            rc = L.orc_reduce_var(ps, out.ctypes.data, W, n, dtype, op, ra, root, order, rounding)
        elif op == SUM:
            rc = L.orc_reduce(ps, out.ctypes.data, W, n, dtype, ra, root, chunk_elems)
        else:
            rc = L.orc_reduce_op(ps, out.ctypes.data, W, n, dtype, op, ra, root, chunk_elems)
        dt = time.perf_counter() - t0
        _check(rc, kind)
        return [out], dt
    if kind == "alltoall":
        assert n % W == 0
        out = [np.zeros(n, dtype=NP_WIRE[dtype]) for _ in range(W)]
        ps, po = _ptrs(src), _ptrs(out)
        t0 = time.perf_counter()
        rc = L.orc_alltoall(ps, po, W, n // W, dtype)
        dt = time.perf_counter() - t0
        _check(rc, kind)
        return out, dt
    raise ValueError(kind)
