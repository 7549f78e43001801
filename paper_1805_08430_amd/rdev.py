"""ctypes binding of librdev.so - argument marshalling only.

Function names equal the C ABI's (include/rdev.h).  Every step of the transfer
path runs inside the library; there is no Python or CPU fallback: if the shared
library has not been built, importing a symbol raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librdev.so")

MAX_DIMS = 8
META_BYTES = 128
DEFAULT_ALIGN = 256
ALL_TENSORS = 0xFFFFFFFF
HOST_ONLY = -1

OK, NOT_READY = 0, 1
E_INVAL, E_NOMEM, E_OVERLAP, E_ALIGN, E_RANGE, E_OVERFLOW, E_BUSY, E_HIP, E_STATE = range(-1, -10, -1)
_ERR_NAMES = {E_INVAL: "E_INVAL", E_NOMEM: "E_NOMEM", E_OVERLAP: "E_OVERLAP", E_ALIGN: "E_ALIGN",
              E_RANGE: "E_RANGE", E_OVERFLOW: "E_OVERFLOW", E_BUSY: "E_BUSY", E_HIP: "E_HIP", E_STATE: "E_STATE"}

U8, I8, I16, I32, I64, F16, BF16, F32, F64 = range(9)
DTYPE = {"u8": U8, "i8": I8, "i16": I16, "i32": I32, "i64": I64, "f16": F16, "bf16": BF16, "f32": F32, "f64": F64}
STATIC, DYNAMIC = 0, 1
ZEROCOPY, RPC2, RPC3, SENDERCOPY, DMA = 0, 1, 2, 3, 4
POLL_CONSUME, POLL_META, POLL_ARENA = 1, 2, 4
PLAN_CHECK_BUSY = 1


class Region(C.Structure):
    _fields_ = [("arena_id", C.c_uint32), ("_pad", C.c_uint32), ("offset", C.c_uint64), ("bytes", C.c_uint64)]


class TensorDesc(C.Structure):
    _fields_ = [("tensor_id", C.c_uint32), ("dtype", C.c_uint32), ("ndims", C.c_uint32),
                ("dst_arena", C.c_uint32), ("dims", C.c_int64 * MAX_DIMS)]


class Placement(C.Structure):
    _fields_ = [("tensor_id", C.c_uint32), ("kind", C.c_uint32), ("dst_arena", C.c_uint32), ("_pad", C.c_uint32),
                ("data_offset", C.c_uint64), ("bytes", C.c_uint64), ("flag_offset", C.c_uint64),
                ("meta_offset", C.c_uint64), ("region_bytes", C.c_uint64)]


class PlanOpts(C.Structure):
    _fields_ = [("align", C.c_uint64), ("max_static_bytes", C.c_uint64), ("dyn_heap_bytes", C.c_uint64),
                ("chunk_bytes", C.c_uint64), ("small_bytes", C.c_uint32), ("flags", C.c_uint32),
                ("rpc_frag_bytes", C.c_uint64), ("flag_groups", C.c_uint32), ("_reserved", C.c_uint32)]


class Meta(C.Structure):
    _fields_ = [("ndims", C.c_uint32), ("dtype", C.c_uint32), ("bytes", C.c_uint64), ("src_offset", C.c_uint64),
                ("dims", C.c_int64 * MAX_DIMS), ("dst_offset", C.c_uint64), ("src_arena", C.c_uint32),
                ("tensor_id", C.c_uint32), ("seq", C.c_uint32), ("reserved", C.c_uint32 * 3),
                ("data_flag", C.c_uint32), ("meta_flag", C.c_uint32)]


class Xfer(C.Structure):
    _fields_ = [("tensor_id", C.c_uint32), ("ndims", C.c_uint32), ("src", C.c_void_p), ("dtype", C.c_uint32),
                ("_pad", C.c_uint32), ("dims", C.c_int64 * MAX_DIMS), ("dim0_dev", C.c_void_p)]


class ConsumeResult(C.Structure):
    _fields_ = [("status", C.c_uint32), ("seen_flag", C.c_uint32), ("max", C.c_float), ("_arrivals", C.c_uint32),
                ("word_sum", C.c_uint64)]


class RdevError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{_ERR_NAMES.get(status, status)}: {msg}")
        self.status = status


_lib = None

# every symbol include/rdev.h declares: name -> (restype, argtypes)
_P = C.c_void_p
SYMBOLS = {
    "rdev_open": (C.c_int32, [C.POINTER(_P), C.c_int]),
    "rdev_close": (C.c_int32, [_P]),
    "rdev_last_error": (C.c_char_p, []),
    "rdev_abi_sizes": (None, [C.POINTER(C.c_uint32)]),
    "rdev_register_arena": (C.c_int32, [_P, _P, C.c_uint64, C.c_uint32, C.POINTER(C.c_uint32)]),
    "rdev_unregister_arena": (C.c_int32, [_P, C.c_uint32]),
    "rdev_alloc_region": (C.c_int32, [_P, C.c_uint32, C.c_uint64, C.c_uint64, C.POINTER(Region)]),
    "rdev_free_region": (C.c_int32, [_P, C.POINTER(Region)]),
    "rdev_plan": (C.c_int32, [_P, C.POINTER(TensorDesc), C.c_uint32, C.POINTER(PlanOpts), C.POINTER(_P)]),
    "rdev_plan_count": (C.c_int32, [_P, C.POINTER(C.c_uint32)]),
    "rdev_plan_get": (C.c_int32, [_P, C.c_uint32, C.POINTER(Placement)]),
    "rdev_plan_arena_info": (C.c_int32, [_P, C.c_uint32] + [C.POINTER(C.c_uint64)] * 4),
    "rdev_plan_bind_sources": (C.c_int32, [_P, C.POINTER(_P), C.c_uint32]),
    "rdev_plan_bind_buffers": (C.c_int32, [_P, C.POINTER(Region), C.POINTER(Region)]),
    "rdev_dyn_reset": (C.c_int32, [_P]),
    "rdev_plan_free": (C.c_int32, [_P]),
    "rdev_write_batch": (C.c_int32, [_P, _P, C.POINTER(Xfer), C.c_uint32, C.c_uint32, C.c_uint32, _P]),
    "rdev_write_batch_fixed_staging": (C.c_int32, [_P, _P, C.POINTER(Xfer), C.c_uint32, C.c_uint32, _P]),
    "rdev_read_batch": (C.c_int32, [_P, _P, C.POINTER(Xfer), C.c_uint32, C.c_uint32, _P]),
    "rdev_read_batch_device": (C.c_int32, [_P, _P, C.POINTER(Xfer), C.c_uint32, C.c_uint32, _P]),
    "rdev_recv_status": (C.c_int32, [_P, C.POINTER(C.c_int32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                     C.POINTER(C.c_uint32)]),
    "rdev_consume_batch": (C.c_int32, [_P, _P, C.POINTER(C.c_uint32), C.c_uint32, C.c_uint32, _P, _P]),
    "rdev_poll": (C.c_int32, [_P, _P, C.c_uint32, C.c_uint32, C.POINTER(Meta), _P]),
    "rdev_gather_unique_rows": (C.c_int32, [_P, _P, C.c_uint32, C.c_uint32, _P, C.c_uint32, _P, _P, _P, _P]),
    "rdev_consume_reduce_max": (C.c_int32, [_P, _P, C.c_uint32, C.c_uint32, _P, _P]),
    "rdev_recv_polling_async": (C.c_int32, [_P, _P, C.POINTER(C.c_uint32), C.c_uint32, _P, _P, _P, C.c_uint64,
                                            C.POINTER(C.c_uint64)]),
    "rdev_graph_open": (C.c_int32, [C.POINTER(_P)]),
    "rdev_graph_close": (C.c_int32, [_P]),
    "rdev_graph_input": (C.c_int32, [_P, C.c_uint32, C.c_uint32, C.POINTER(C.c_int64), C.c_uint32, C.POINTER(C.c_uint32)]),
    "rdev_graph_node": (C.c_int32, [_P, C.c_uint32, C.POINTER(C.c_uint32), C.c_uint32, C.POINTER(C.c_int64), C.c_uint32,
                                    C.c_uint32, C.POINTER(C.c_uint32)]),
    "rdev_graph_infer": (C.c_int32, [_P]),
    "rdev_graph_value": (C.c_int32, [_P, C.c_uint32, C.POINTER(TensorDesc)]),
    "rdev_graph_transfers": (C.c_int32, [_P, C.POINTER(C.c_uint32), C.c_uint32, C.POINTER(TensorDesc),
                                         C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.c_uint32, C.POINTER(C.c_uint32)]),
    "rdev_tracer_open": (C.c_int32, [_P, _P, C.c_uint64, C.c_uint32, C.POINTER(_P)]),
    "rdev_tracer_close": (C.c_int32, [_P]),
    "rdev_tracer_begin_iteration": (C.c_int32, [_P]),
    "rdev_tracer_alloc": (C.c_int32, [_P, C.c_uint32, C.c_uint64, C.POINTER(_P), C.POINTER(C.c_uint32),
                                      C.POINTER(C.c_uint32)]),
    "rdev_tracer_free": (C.c_int32, [_P, _P]),
    "rdev_tracer_mark_sent": (C.c_int32, [_P, _P, C.POINTER(C.c_uint32)]),
    "rdev_tracer_send": (C.c_int32, [_P, _P, C.c_uint32, _P, C.c_uint32, _P, C.POINTER(C.c_uint32)]),
    "rdev_tracer_set_size": (C.c_int32, [_P, C.POINTER(C.c_uint32)]),
    "rdev_tracer_set_get": (C.c_int32, [_P, C.c_uint32, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]),
    "rdev_device_info": (C.c_int32, [_P, C.POINTER(C.c_uint64)]),
    "rdev_plan_profile": (C.c_int32, [_P, C.c_uint32, C.c_uint32]),
    "rdev_plan_profile_read": (C.c_int32, [_P, C.POINTER(C.c_float), C.c_uint32, C.POINTER(C.c_uint32)]),
}


def lib() -> C.CDLL:
    """Load librdev.so (once).  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RdevError(E_HIP, f"{LIB_PATH} is missing: run `python -m paper_1805_08430_amd.build` "
                                   "(there is no fallback path)")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        sizes = (C.c_uint32 * 6)()
        l.rdev_abi_sizes(sizes)
        want = [C.sizeof(TensorDesc), C.sizeof(Placement), C.sizeof(PlanOpts), C.sizeof(Meta), C.sizeof(Xfer),
                C.sizeof(Region)]
        if list(sizes) != want:
            raise RdevError(E_INVAL, f"ABI struct sizes differ: library {list(sizes)}, binding {want}")
        _lib = l
    return _lib


def _check(st: int) -> int:
    if st < 0:
        raise RdevError(st, (lib().rdev_last_error() or b"").decode())
    return st


def rdev_last_error() -> str:
    return (lib().rdev_last_error() or b"").decode()


def rdev_open(hip_device: int = 0) -> int:
    h = _P()
    _check(lib().rdev_open(C.byref(h), hip_device))
    return h.value


def rdev_close(dev: int) -> None:
    _check(lib().rdev_close(dev))


def rdev_register_arena(dev: int, base: int, nbytes: int, arena_flags: int = 0) -> int:
    out = C.c_uint32()
    _check(lib().rdev_register_arena(dev, base, nbytes, arena_flags, C.byref(out)))
    return out.value


def rdev_unregister_arena(dev: int, arena_id: int) -> None:
    _check(lib().rdev_unregister_arena(dev, arena_id))


def rdev_alloc_region(dev: int, arena_id: int, nbytes: int, align: int = DEFAULT_ALIGN) -> Region:
    r = Region()
    _check(lib().rdev_alloc_region(dev, arena_id, nbytes, align, C.byref(r)))
    return r


def rdev_free_region(dev: int, region: Region) -> None:
    _check(lib().rdev_free_region(dev, C.byref(region)))


def make_desc(tensor_id: int, dtype: int, dims: Sequence[int], dst_arena: int) -> TensorDesc:
    d = TensorDesc()
    d.tensor_id, d.dtype, d.ndims, d.dst_arena = tensor_id, dtype, len(dims), dst_arena
    for i, v in enumerate(dims[:MAX_DIMS]):
        d.dims[i] = v
    return d


def rdev_plan(dev: int, descs: Sequence[TensorDesc], align: int = 0, max_static_bytes: int = 0,
              dyn_heap_bytes: int = 0, chunk_bytes: int = 0, small_bytes: int = 0, flags: int = 0,
              rpc_frag_bytes: int = 0, flag_groups: int = 0) -> int:
    arr = (TensorDesc * max(len(descs), 1))(*descs)
    o = PlanOpts(align, max_static_bytes, dyn_heap_bytes, chunk_bytes, small_bytes, flags, rpc_frag_bytes,
                 flag_groups, 0)
    h = _P()
    _check(lib().rdev_plan(dev, arr, len(descs), C.byref(o), C.byref(h)))
    return h.value


def rdev_plan_count(plan: int) -> int:
    n = C.c_uint32()
    _check(lib().rdev_plan_count(plan, C.byref(n)))
    return n.value


def rdev_plan_get(plan: int, i: int) -> Placement:
    p = Placement()
    _check(lib().rdev_plan_get(plan, i, C.byref(p)))
    return p


def rdev_plan_arena_info(plan: int, arena_id: int) -> dict:
    v = [C.c_uint64() for _ in range(4)]
    _check(lib().rdev_plan_arena_info(plan, arena_id, *[C.byref(x) for x in v]))
    return dict(base=v[0].value, static_bytes=v[1].value, heap_offset=v[2].value, heap_bytes=v[3].value)


def rdev_plan_bind_sources(plan: int, src_ptrs: Sequence[Optional[int]]) -> None:
    arr = (_P * max(len(src_ptrs), 1))(*[p if p else None for p in src_ptrs])
    _check(lib().rdev_plan_bind_sources(plan, arr, len(src_ptrs)))


def rdev_plan_bind_buffers(plan: int, send_buf: Region, recv_buf: Optional[Region] = None) -> None:
    _check(lib().rdev_plan_bind_buffers(plan, C.byref(send_buf), C.byref(recv_buf) if recv_buf is not None else None))


def rdev_dyn_reset(plan: int) -> None:
    _check(lib().rdev_dyn_reset(plan))


def rdev_plan_free(plan: int) -> None:
    _check(lib().rdev_plan_free(plan))


def make_xfer(tensor_id: int, src: Optional[int] = None, dtype: int = 0, dims: Sequence[int] = (),
              dim0_dev: Optional[int] = None) -> Xfer:
    x = Xfer()
    x.tensor_id, x.ndims, x.src, x.dtype, x.dim0_dev = tensor_id, len(dims), src, dtype, dim0_dev
    for i, v in enumerate(dims[:MAX_DIMS]):
        x.dims[i] = v
    return x


class XferArray:
    """A batch marshalled once (a C array of rdev_xfer) for callers that send the same batch every iteration."""
    __slots__ = ("arr", "n")

    def __init__(self, xs: Sequence[Xfer]):
        self.arr, self.n = (Xfer * len(xs))(*xs), len(xs)


def _xfers(x):
    if not x:
        return None, 0
    if isinstance(x, XferArray):
        return x.arr, x.n
    return (Xfer * len(x))(*x), len(x)


def rdev_write_batch(dev: int, plan: int, x: Optional[Sequence[Xfer]] = None, mode: int = ZEROCOPY, seq: int = 1,
                     stream: int = 0) -> None:
    arr, n = _xfers(x)
    _check(lib().rdev_write_batch(dev, plan, arr, n, mode, seq, stream or None))


FIXED_STAGING_BYTES = 16 << 20


def rdev_write_batch_fixed_staging(dev: int, plan: int, x: Optional[Sequence[Xfer]] = None, seq: int = 1,
                                   stream: int = 0) -> None:
    arr, n = _xfers(x)
    _check(lib().rdev_write_batch_fixed_staging(dev, plan, arr, n, seq, stream or None))


def rdev_read_batch(dev: int, plan: int, x: Optional[Sequence[Xfer]] = None, seq: int = 1, stream: int = 0) -> None:
    arr, n = _xfers(x)
    _check(lib().rdev_read_batch(dev, plan, arr, n, seq, stream or None))


def rdev_read_batch_device(dev: int, plan: int, x: Sequence[Xfer], seq: int = 1, stream: int = 0) -> None:
    arr, n = _xfers(x)
    _check(lib().rdev_read_batch_device(dev, plan, arr, n, seq, stream or None))


def rdev_recv_status(plan: int) -> dict:
    st, ent, done, made = C.c_int32(), C.c_uint32(), C.c_uint32(), C.c_uint32()
    _check(lib().rdev_recv_status(plan, C.byref(st), C.byref(ent), C.byref(done), C.byref(made)))
    return dict(status=st.value, entry=ent.value, calls_done=done.value, calls_made=made.value)


def rdev_consume_batch(dev: int, plan: int, tensor_ids: Sequence[int], max_spins: int, out_ptr: int, stream: int = 0) -> None:
    arr = (C.c_uint32 * max(len(tensor_ids), 1))(*tensor_ids)
    _check(lib().rdev_consume_batch(dev, plan, arr, len(tensor_ids), max_spins, out_ptr, stream or None))


def rdev_poll(dev: int, plan: int, tensor_id: int = ALL_TENSORS, poll_flags: int = 0, stream: int = 0,
              want_meta: bool = False):
    """Returns True/False (ready or not); with want_meta=True returns (ready, Meta-or-None)."""
    m = Meta()
    st = _check(lib().rdev_poll(dev, plan, tensor_id, poll_flags, C.byref(m) if want_meta else None, stream or None))
    ready = st == OK
    if want_meta:
        return ready, (m if ready else None)
    return ready


def rdev_gather_unique_rows(dev: int, ids_ptr: int, n_ids: int, vocab: int, table_ptr: int, row_bytes: int,
                            out_ids_ptr: int, out_rows_ptr: int, count_ptr: int, stream: int = 0) -> None:
    _check(lib().rdev_gather_unique_rows(dev, ids_ptr, n_ids, vocab, table_ptr, row_bytes, out_ids_ptr, out_rows_ptr,
                                         count_ptr, stream or None))


def rdev_consume_reduce_max(dev: int, plan: int, tensor_id: int, max_spins: int, out_ptr: int, stream: int = 0) -> None:
    _check(lib().rdev_consume_reduce_max(dev, plan, tensor_id, max_spins, out_ptr, stream or None))


def rdev_recv_polling_async(dev: int, plan: int, tensor_ids: Sequence[int], out_ptr: int, flag_stream: int = 0,
                            consumer_stream: int = 0, max_polls: int = 1 << 40):
    """Returns (all_received, polls made)."""
    arr = (C.c_uint32 * max(len(tensor_ids), 1))(*tensor_ids)
    polls = C.c_uint64()
    st = _check(lib().rdev_recv_polling_async(dev, plan, arr, len(tensor_ids), out_ptr, flag_stream or None,
                                              consumer_stream or None, max_polls, C.byref(polls)))
    return st == OK, polls.value


OP_UNARY, OP_BINARY, OP_MATMUL, OP_TRANSPOSE, OP_RESHAPE, OP_CONCAT, OP_REDUCE, OP_GATHER, OP_UNIQUE, OP_CONV2D, \
    OP_GRAD, OP_CAST = range(12)


def rdev_graph_open() -> int:
    h = _P()
    _check(lib().rdev_graph_open(C.byref(h)))
    return h.value


def rdev_graph_close(g: int) -> None:
    _check(lib().rdev_graph_close(g))


def rdev_graph_input(g: int, dtype: int, dims: Sequence[int], partition: int) -> int:
    arr = (C.c_int64 * max(len(dims), 1))(*dims)
    v = C.c_uint32()
    _check(lib().rdev_graph_input(g, dtype, len(dims), arr, partition, C.byref(v)))
    return v.value


def rdev_graph_node(g: int, op: int, inputs: Sequence[int], attrs: Sequence[int], partition: int) -> int:
    ins = (C.c_uint32 * max(len(inputs), 1))(*inputs)
    at = (C.c_int64 * max(len(attrs), 1))(*attrs)
    v = C.c_uint32()
    _check(lib().rdev_graph_node(g, op, ins, len(inputs), at, len(attrs), partition, C.byref(v)))
    return v.value


def rdev_graph_infer(g: int) -> None:
    _check(lib().rdev_graph_infer(g))


def rdev_graph_value(g: int, value: int) -> TensorDesc:
    d = TensorDesc()
    _check(lib().rdev_graph_value(g, value, C.byref(d)))
    return d


def rdev_graph_transfers(g: int, partition_to_arena: Sequence[int]):
    """Returns (descs, values, destination partitions)."""
    p2a = (C.c_uint32 * max(len(partition_to_arena), 1))(*partition_to_arena)
    n = C.c_uint32()
    st = lib().rdev_graph_transfers(g, p2a, len(partition_to_arena), None, None, None, 0, C.byref(n))
    if st not in (OK, E_NOMEM):
        _check(st)
    cap = max(n.value, 1)
    descs, vals, parts = (TensorDesc * cap)(), (C.c_uint32 * cap)(), (C.c_uint32 * cap)()
    _check(lib().rdev_graph_transfers(g, p2a, len(partition_to_arena), descs, vals, parts, cap, C.byref(n)))
    return list(descs[:n.value]), list(vals[:n.value]), list(parts[:n.value])


def rdev_tracer_open(dev: int, pool_base: int, pool_bytes: int, arena_id: int) -> int:
    h = _P()
    _check(lib().rdev_tracer_open(dev, pool_base, pool_bytes, arena_id, C.byref(h)))
    return h.value


def rdev_tracer_close(tr: int) -> None:
    _check(lib().rdev_tracer_close(tr))


def rdev_tracer_begin_iteration(tr: int) -> None:
    _check(lib().rdev_tracer_begin_iteration(tr))


def rdev_tracer_alloc(tr: int, node_id: int, nbytes: int):
    """Returns (device pointer, allocation index, in_arena)."""
    p, idx, ar = _P(), C.c_uint32(), C.c_uint32()
    _check(lib().rdev_tracer_alloc(tr, node_id, nbytes, C.byref(p), C.byref(idx), C.byref(ar)))
    return p.value, idx.value, bool(ar.value)


def rdev_tracer_free(tr: int, ptr: int) -> None:
    _check(lib().rdev_tracer_free(tr, ptr))


def rdev_tracer_mark_sent(tr: int, ptr: int) -> bool:
    """Returns True when the buffer lies in registered memory."""
    r = C.c_uint32()
    _check(lib().rdev_tracer_mark_sent(tr, ptr, C.byref(r)))
    return bool(r.value)


def rdev_tracer_send(tr: int, plan: int, tensor_id: int, ptr: int, seq: int = 1, stream: int = 0) -> bool:
    """Returns True when the tensor was staged (copied) before the write."""
    c = C.c_uint32()
    _check(lib().rdev_tracer_send(tr, plan, tensor_id, ptr, seq, stream or None, C.byref(c)))
    return bool(c.value)


def rdev_tracer_set(tr: int):
    n = C.c_uint32()
    _check(lib().rdev_tracer_set_size(tr, C.byref(n)))
    out = []
    for i in range(n.value):
        a, b = C.c_uint32(), C.c_uint32()
        _check(lib().rdev_tracer_set_get(tr, i, C.byref(a), C.byref(b)))
        out.append((a.value, b.value))
    return out


def rdev_device_info(dev: int) -> dict:
    v = (C.c_uint64 * 4)()
    _check(lib().rdev_device_info(dev, v))
    return dict(memory_clock_khz=v[0], memory_bus_bits=v[1], compute_units=v[2], l2_bytes=v[3])


def rdev_plan_profile(plan: int, max_samples: int, every: int = 1) -> None:
    _check(lib().rdev_plan_profile(plan, max_samples, every))


def rdev_plan_profile_read(plan: int, cap: int) -> List[float]:
    buf = (C.c_float * max(cap, 1))()
    n = C.c_uint32()
    _check(lib().rdev_plan_profile_read(plan, buf, cap, C.byref(n)))
    return [buf[i] for i in range(n.value)]


def placements(plan: int) -> List[Placement]:
    return [rdev_plan_get(plan, i) for i in range(rdev_plan_count(plan))]
