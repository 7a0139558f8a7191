"""ctypes binding of libhcl (argument marshalling only; every step of a
collective runs in the library's HIP kernels).

torch is used for device memory and streams: the functions take lists of W
torch tensors (one per simulated rank) and pass their data pointers and the
current HIP stream through the C ABI declared in include/hcl.h.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhcl.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_ALIAS, ERR_WORKSPACE, ERR_HIP = range(6)
FP32, BF16, FP16, INT32, FP64, INT64, UINT8 = 0, 1, 2, 3, 4, 5, 6
SUM, PROD, MAX, MIN = 0, 1, 2, 3
OP = {"sum": SUM, "prod": PROD, "max": MAX, "min": MIN}
SCHED_STEPWISE, SCHED_FUSED = 0, 1
XPORT_DIRECT, XPORT_HOST_STAGED = 0, 1
KIND_ALLREDUCE, KIND_REDUCE_SCATTER, KIND_ALL_GATHER, KIND_REDUCE, KIND_BROADCAST, KIND_ALLTOALL = range(6)
PHASE_RS, PHASE_AG = 0, 1
MAX_RANKS = 16

DTYPE_OF_TORCH = {torch.float32: FP32, torch.bfloat16: BF16, torch.float16: FP16, torch.int32: INT32,
                  torch.float64: FP64, torch.int64: INT64, torch.uint8: UINT8}
SCHED = {"stepwise": SCHED_STEPWISE, "fused": SCHED_FUSED}
XPORT = {"direct": XPORT_DIRECT, "host_staged": XPORT_HOST_STAGED}
ACC_PER_HOP, ACC_FP32 = 0, 1
ACC = {"per_hop": ACC_PER_HOP, "fp32": ACC_FP32}
ORDER_RING, ORDER_TREE = 0, 1
ORDER = {"ring": ORDER_RING, "tree": ORDER_TREE}

EXPORTS = [
    "hcl_allreduce_sim", "hcl_reduce_scatter_sim", "hcl_all_gather_sim", "hcl_reduce_sim",
    "hcl_broadcast_sim", "hcl_alltoall_sim", "hcl_workspace_bytes",
    "hcl_host_stage_bytes", "hcl_ring_step", "hcl_schedule_items", "hcl_events_create",
    "hcl_events_destroy", "hcl_event_record", "hcl_event_elapsed_ms", "hcl_device_cu_count",
    "hcl_status_string", "hcl_last_error", "hcl_version",
    "hcl_reduce_scatter_sim_static", "hcl_static_scratch_bytes",
]


class HclError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{message} [{status}]")
        self.status = status


class Opts(ctypes.Structure):
    _fields_ = [
        ("ring", ctypes.POINTER(ctypes.c_int)),
        ("sched", ctypes.c_int),
        ("xport", ctypes.c_int),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
        ("host_stage", ctypes.c_void_p),
        ("host_stage_bytes", ctypes.c_size_t),
        ("threads", ctypes.c_int),
        ("blocks", ctypes.c_int),
        ("unroll", ctypes.c_int),
        ("nontemporal", ctypes.c_int),
        ("fuse_rs_ag", ctypes.c_int),
        ("events", ctypes.POINTER(ctypes.c_void_p)),
        ("n_events", ctypes.c_int),
        ("events_per_phase", ctypes.c_int),
        ("n_launches", ctypes.POINTER(ctypes.c_int)),
        ("accumulate", ctypes.c_int),
        ("order", ctypes.c_int),
        ("slab_bytes", ctypes.c_size_t),
        ("aux_stream", ctypes.c_void_p),
        ("aux_events", ctypes.POINTER(ctypes.c_void_p)),
    ]


class WorkItem(ctypes.Structure):
    _fields_ = [
        ("phase", ctypes.c_int), ("step", ctypes.c_int), ("rank", ctypes.c_int), ("from_rank", ctypes.c_int),
        ("block", ctypes.c_int), ("send_block", ctypes.c_int),
        ("chunk", ctypes.c_uint64), ("elem_offset", ctypes.c_uint64), ("elem_count", ctypes.c_uint64),
        ("vec_offset", ctypes.c_uint64),
    ]


_lib = None


def lib():
    """Loads libhcl.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_22585_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vpp = ctypes.POINTER(ctypes.c_void_p)
    ip = ctypes.POINTER(ctypes.c_int)
    op = ctypes.POINTER(Opts)
    L.hcl_allreduce_sim.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_size_t, op, ctypes.c_void_p]
    L.hcl_reduce_scatter_sim.argtypes = L.hcl_allreduce_sim.argtypes
    L.hcl_reduce_scatter_sim_static.argtypes = L.hcl_allreduce_sim.argtypes
    L.hcl_static_scratch_bytes.restype = ctypes.c_size_t
    L.hcl_all_gather_sim.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int,
                                     ctypes.c_size_t, op, ctypes.c_void_p]
    L.hcl_reduce_sim.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                 ctypes.c_size_t, op, ctypes.c_void_p]
    L.hcl_broadcast_sim.argtypes = [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_size_t, op, ctypes.c_void_p]
    L.hcl_alltoall_sim.argtypes = L.hcl_all_gather_sim.argtypes
    for f in ("hcl_workspace_bytes", "hcl_host_stage_bytes"):
        getattr(L, f).argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_size_t, op]
        getattr(L, f).restype = ctypes.c_size_t
    L.hcl_ring_step.argtypes = [ctypes.c_int, ip, ctypes.c_int, ctypes.c_int, ctypes.c_int, ip, ip]
    L.hcl_schedule_items.argtypes = [ctypes.c_int, ip, ctypes.c_size_t, ctypes.c_int, ctypes.c_size_t,
                                     ctypes.c_int, ctypes.c_int, ctypes.POINTER(WorkItem), ctypes.c_size_t,
                                     ctypes.POINTER(ctypes.c_size_t)]
    L.hcl_events_create.argtypes = [ctypes.c_int, vpp]
    L.hcl_events_destroy.argtypes = [ctypes.c_int, vpp]
    L.hcl_event_record.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    L.hcl_event_elapsed_ms.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_float)]
    L.hcl_status_string.argtypes = [ctypes.c_int]
    L.hcl_status_string.restype = ctypes.c_char_p
    L.hcl_last_error.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(status):
    if status != OK:
        L = lib()
        raise HclError(L.hcl_status_string(status).decode(), L.hcl_last_error().decode())


def _int_array(vals):
    return (ctypes.c_int * len(vals))(*[int(v) for v in vals])


def _ptr_array(ptrs):
    return (ctypes.c_void_p * len(ptrs))(*ptrs)


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class EventList:
    """HIP events owned by the library's helpers, for timing launches on their own stream."""

    def __init__(self, n):
        self.n = n
        self.arr = (ctypes.c_void_p * n)()
        _check(lib().hcl_events_create(n, self.arr))

    def record(self, i, stream=None):
        _check(lib().hcl_event_record(self.arr[i], _stream_handle(stream)))

    def elapsed_ms(self, i, j):
        ms = ctypes.c_float()
        _check(lib().hcl_event_elapsed_ms(self.arr[i], self.arr[j], ctypes.byref(ms)))
        return ms.value

    def close(self):
        if self.arr is not None:
            lib().hcl_events_destroy(self.n, self.arr)
            self.arr = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def make_opts(W, ring=None, sched="stepwise", xport="direct", workspace=None, host_stage=None,
              threads=0, blocks=0, unroll=0, nontemporal=0, fuse_rs_ag=False, events=None,
              events_per_phase=False, accumulate=0, order=0, aux_stream=None, aux_events=None, slab_bytes=0):
    """Builds the hcl_opts_t struct.  Returns (opts, keepalive): keep `keepalive`
    referenced until the call has returned."""
    o = Opts()
    keep = []
    if ring is not None:
        arr = _int_array(ring)
        keep.append(arr)
        o.ring = ctypes.cast(arr, ctypes.POINTER(ctypes.c_int))
    o.sched = SCHED[sched] if isinstance(sched, str) else int(sched)
    o.xport = XPORT[xport] if isinstance(xport, str) else int(xport)
    if workspace is not None:
        o.workspace = workspace.data_ptr()
        o.workspace_bytes = workspace.numel() * workspace.element_size()
        keep.append(workspace)
    if host_stage is not None:
        o.host_stage = host_stage.data_ptr()
        o.host_stage_bytes = host_stage.numel() * host_stage.element_size()
        keep.append(host_stage)
    o.threads, o.blocks, o.unroll, o.nontemporal = int(threads), int(blocks), int(unroll), int(nontemporal)
    o.fuse_rs_ag = 1 if fuse_rs_ag else 0
    o.accumulate = ACC[accumulate] if isinstance(accumulate, str) else int(accumulate)
    o.order = ORDER[order] if isinstance(order, str) else int(order)
    if events is not None:
        # an EventList, or (EventList, first, n) to use a slice of it
        ev, first, n = events if isinstance(events, tuple) else (events, 0, events.n)
        assert 0 <= first and first + n <= ev.n
        o.events = ctypes.cast(ctypes.byref(ev.arr, first * ctypes.sizeof(ctypes.c_void_p)),
                               ctypes.POINTER(ctypes.c_void_p))
        o.n_events = n
        o.events_per_phase = 1 if events_per_phase else 0
        keep.append(ev)
    o.slab_bytes = ctypes.c_size_t(-1).value if slab_bytes < 0 else int(slab_bytes)
    if aux_stream is not None:
        # a torch stream and an EventList of two events: the second dependency chain
        o.aux_stream = aux_stream.cuda_stream
        assert aux_events is not None and aux_events.n >= 2
        o.aux_events = ctypes.cast(aux_events.arr, ctypes.POINTER(ctypes.c_void_p))
        keep += [aux_stream, aux_events]
    nl = ctypes.c_int(0)
    o.n_launches = ctypes.pointer(nl)
    keep.append(nl)
    return o, keep


def _dtype_code(tensors, dtype):
    if dtype is not None:
        return int(dtype)
    return DTYPE_OF_TORCH[tensors[0].dtype]


def _op_code(op):
    return OP[op] if isinstance(op, str) else int(op)


def _ptrs(tensors):
    return _ptr_array([None if t is None else t.data_ptr() for t in tensors])


def allreduce_sim(send, recv, chunk_bytes=0, dtype=None, op=SUM, stream=None, count=None, **opt):
    """Ring All-Reduce (sum) over W = len(send) rank buffers.  Returns the number of launches."""
    W = len(send)
    o, keep = make_opts(W, **opt)
    n = send[0].numel() if count is None else count
    _check(lib().hcl_allreduce_sim(_ptrs(send), _ptrs(recv), W, n, _dtype_code(send, dtype), _op_code(op),
                                   chunk_bytes, ctypes.byref(o), _stream_handle(stream)))
    return o.n_launches.contents.value


def reduce_scatter_sim(send, recv, chunk_bytes=0, dtype=None, op=SUM, stream=None, recvcount=None, **opt):
    """Ring Reduce-Scatter (sum): send[r] has W * recvcount elements, recv[r] gets block r."""
    W = len(send)
    o, keep = make_opts(W, **opt)
    n = recv[0].numel() if recvcount is None else recvcount
    _check(lib().hcl_reduce_scatter_sim(_ptrs(send), _ptrs(recv), W, n, _dtype_code(send, dtype), _op_code(op),
                                        chunk_bytes, ctypes.byref(o), _stream_handle(stream)))
    return o.n_launches.contents.value


def reduce_scatter_sim_static(send, recv, chunk_bytes=0, dtype=None, op=SUM, stream=None, recvcount=None, **opt):
    """Reduce-Scatter whose partial sums live in the library's own fixed scratch array (no workspace)."""
    W = len(send)
    o, keep = make_opts(W, **opt)
    n = recv[0].numel() if recvcount is None else recvcount
    _check(lib().hcl_reduce_scatter_sim_static(_ptrs(send), _ptrs(recv), W, n, _dtype_code(send, dtype), _op_code(op),
                                               chunk_bytes, ctypes.byref(o), _stream_handle(stream)))
    return o.n_launches.contents.value


def static_scratch_bytes():
    return lib().hcl_static_scratch_bytes()


def all_gather_sim(send, recv, chunk_bytes=0, dtype=None, stream=None, sendcount=None, **opt):
    """Ring All-Gather: send[r] has sendcount elements, recv[r] gets all W blocks."""
    W = len(send)
    o, keep = make_opts(W, **opt)
    n = send[0].numel() if sendcount is None else sendcount
    _check(lib().hcl_all_gather_sim(_ptrs(send), _ptrs(recv), W, n, _dtype_code(send, dtype),
                                    chunk_bytes, ctypes.byref(o), _stream_handle(stream)))
    return o.n_launches.contents.value


def reduce_sim(send, recv, root, chunk_bytes=0, dtype=None, op=SUM, stream=None, count=None, **opt):
    """Ring Reduce (sum) to `root`: only recv[root] is written (other entries may be None)."""
    W = len(send)
    o, keep = make_opts(W, **opt)
    n = send[0].numel() if count is None else count
    _check(lib().hcl_reduce_sim(_ptrs(send), _ptrs(recv), W, n, _dtype_code(send, dtype), _op_code(op), root,
                                chunk_bytes, ctypes.byref(o), _stream_handle(stream)))
    return o.n_launches.contents.value


def broadcast_sim(send, recv, root, chunk_bytes=0, dtype=None, stream=None, count=None, **opt):
    """Ring Broadcast from `root`: only send[root] is read (other entries may be None)."""
    W = len(recv)
    o, keep = make_opts(W, **opt)
    n = recv[0].numel() if count is None else count
    _check(lib().hcl_broadcast_sim(_ptrs(send), _ptrs(recv), W, n, _dtype_code(recv, dtype), root,
                                   chunk_bytes, ctypes.byref(o), _stream_handle(stream)))
    return o.n_launches.contents.value


def alltoall_sim(send, recv, chunk_bytes=0, dtype=None, stream=None, count=None, **opt):
    """All-to-All: block q of recv[r] becomes block r of send[q]; count = elements per block."""
    W = len(send)
    o, keep = make_opts(W, **opt)
    n = send[0].numel() // W if count is None else count
    _check(lib().hcl_alltoall_sim(_ptrs(send), _ptrs(recv), W, n, _dtype_code(send, dtype),
                                  chunk_bytes, ctypes.byref(o), _stream_handle(stream)))
    return o.n_launches.contents.value


def workspace_bytes(kind, W, count, dtype, chunk_bytes=0, **opt):
    o, keep = make_opts(W, **opt)
    return lib().hcl_workspace_bytes(kind, W, count, dtype, chunk_bytes, ctypes.byref(o))


def host_stage_bytes(kind, W, count, dtype, chunk_bytes=0, **opt):
    o, keep = make_opts(W, **opt)
    return lib().hcl_host_stage_bytes(kind, W, count, dtype, chunk_bytes, ctypes.byref(o))


def ring_step(W, ring, phase, step, rank):
    sb, rb = ctypes.c_int(-1), ctypes.c_int(-1)
    arr = _int_array(ring) if ring is not None else None
    _check(lib().hcl_ring_step(W, arr, phase, step, rank, ctypes.byref(sb), ctypes.byref(rb)))
    return sb.value, rb.value


def schedule_items(W, ring, count, dtype, chunk_bytes, phase, step):
    """The work items of one ring step as a list of dicts."""
    arr = _int_array(ring) if ring is not None else None
    n = ctypes.c_size_t(0)
    _check(lib().hcl_schedule_items(W, arr, count, dtype, chunk_bytes, phase, step, None, 0, ctypes.byref(n)))
    items = (WorkItem * max(1, n.value))()
    _check(lib().hcl_schedule_items(W, arr, count, dtype, chunk_bytes, phase, step, items, n.value, ctypes.byref(n)))
    return [{f: getattr(items[i], f) for f, _ in WorkItem._fields_} for i in range(n.value)]


def device_cu_count():
    return lib().hcl_device_cu_count()


def version():
    return lib().hcl_version()
