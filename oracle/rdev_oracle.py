"""CPU checker for tensor transfer through a memory-region "device" interface.

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct model of
what the transfer path computes, written from the paper's prose (the paper has
no equations or listings for this path).  Only tests, the smoke check and the
CPU-baseline leg of the benchmark may use it; the GPU library neither imports
nor links anything from here, and this file imports nothing from the library.

What is modelled (section numbers are the paper's):

* section 3.1  a *device* exposes allocate / free of remotely accessible memory
               regions and a memory copy between a local and a remote region.
* section 3.4  one large registered buffer (an *arena*) with a sub-allocator on
               top; before the computation the analyzer pre-allocates receiver
               data buffers for tensors whose shape never changes, or metadata
               buffers otherwise, and hands the addresses to the sender.
* section 3.2  static placement: the sender writes the tensor into the fixed
               receiver region, a flag at the tail of the region becomes set
               only after the whole tensor; the receiver polls, clears, goes on.
* section 3.3  dynamic allocation: rank is fixed so the metadata record has a
               fixed size (ndims, dims, element type, sender address); sender
               writes metadata + flag; receiver polls, clears, allocates
               storage, pulls the payload with a one-sided read.
* section 2.2 / 5.1  the RPC-style path that is being replaced: header +
               payload copied into a message buffer, (copied once more to a
               receive buffer,) parsed and copied into a fresh allocation; and
               the sender-side staging copy variant.

Readings where the paper is silent are fixed here: alignment 256, a 4-byte flag
word holding the iteration number, a 128-byte little-endian record, a
deterministic bump heap, placement in input order.

The result is exact: after a transfer every receiver region holds the byte
string of its source tensor at the planned place and nothing else changed.
Arenas are numpy uint8 arrays; every store is also appended to an event log so
that ordering properties (no flag before its payload) can be checked.

Pins (tests, CPU only): plan invariants + closed-form prefix sums + brute-force
pairwise disjointness; byte-at-a-time movers on exhaustive tiny inputs; the
one-aligned-tensor case against numpy slice assignment; RPC modes against the
zero-copy result and against message, fragment and staging buffers rebuilt one
byte at a time; the place a poll names after an RPC delivery and after a later
zero-copy delivery; metadata bytes against a hand-assembled fixture; gather
against nested Python loops.  No function here is unpinned.
"""
from __future__ import annotations

import struct
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

U64_MAX = (1 << 64) - 1
MAX_DIMS = 8
META_BYTES = 128
DEFAULT_ALIGN = 256
FLAG_BYTES = 4

# element type codes of the metadata record (own enumeration; section 3.3 only
# lists the element type among the record's fields)
DTYPE_CODE = {"u8": 0, "i8": 1, "i16": 2, "i32": 3, "i64": 4, "f16": 5, "bf16": 6, "f32": 7, "f64": 8}
DTYPE_SIZE = {0: 1, 1: 1, 2: 2, 3: 4, 4: 8, 5: 2, 6: 2, 7: 4, 8: 8}

STATIC, DYNAMIC = 0, 1
MODE_ZEROCOPY, MODE_RPC2, MODE_RPC3, MODE_SENDERCOPY = 0, 1, 2, 3


class OracleError(Exception):
    """kind is one of: inval, nomem, overlap, align, range, overflow, busy, state."""

    def __init__(self, kind: str, msg: str = ""):
        super().__init__(f"{kind}: {msg}")
        self.kind = kind


def round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


def tensor_nbytes(dtype_code: int, dims: Sequence[int]) -> int:
    """bytes = itemsize * product of dims; rank 0 is a scalar (one element)."""
    if dtype_code not in DTYPE_SIZE:
        raise OracleError("inval", f"unknown dtype {dtype_code}")
    if len(dims) > MAX_DIMS:
        raise OracleError("inval", "rank too large")
    n = DTYPE_SIZE[dtype_code]
    for d in dims:
        if d < 0:
            raise OracleError("inval", "unknown dim in a size computation")
        n *= d
    if n > U64_MAX:
        raise OracleError("overflow", "tensor bytes exceed 64 bits")
    return n


# ---------------------------------------------------------------------------
# section 3.4: registered arena + sub-allocator (section 3.1: alloc / free region)
# ---------------------------------------------------------------------------
class RegionAllocator:
    """First fit from the lowest address inside one arena; free blocks are kept
    sorted and merged with their neighbours when a region is returned."""

    def __init__(self, nbytes: int):
        self.nbytes = nbytes
        self.free: List[Tuple[int, int]] = [(0, nbytes)] if nbytes else []   # (offset, bytes)
        self.used: Dict[int, int] = {}                                        # offset -> bytes

    def alloc(self, nbytes: int, align: int) -> int:
        if nbytes <= 0:
            raise OracleError("inval", "region bytes must be positive")
        if align <= 0 or align & (align - 1):
            raise OracleError("align", "alignment must be a power of two")
        for i, (off, sz) in enumerate(self.free):
            start = round_up(off, align)
            if start + nbytes <= off + sz:
                pieces = []
                if start > off:
                    pieces.append((off, start - off))
                if start + nbytes < off + sz:
                    pieces.append((start + nbytes, off + sz - start - nbytes))
                self.free[i:i + 1] = pieces
                self.used[start] = nbytes
                return start
        raise OracleError("nomem", "no free block fits")

    def release(self, offset: int, nbytes: int) -> None:
        if self.used.get(offset) != nbytes:
            raise OracleError("inval", "not an allocated region")
        del self.used[offset]
        self.free.append((offset, nbytes))
        self.free.sort()
        merged: List[Tuple[int, int]] = []
        for off, sz in self.free:
            if merged and merged[-1][0] + merged[-1][1] == off:
                merged[-1] = (merged[-1][0], merged[-1][1] + sz)
            else:
                merged.append((off, sz))
        self.free = merged


@dataclass
class Arena:
    mem: np.ndarray                 # uint8 image
    alloc: RegionAllocator


class Device:
    """Holds the arenas of both ends (one process stands in for sender and
    receiver) and the event log."""

    def __init__(self):
        self.arenas: List[Arena] = []
        self.log: List[Tuple[str, int, int, int, int]] = []   # (kind, tensor, arena, lo, hi)

    def register_arena(self, image: np.ndarray) -> int:
        assert image.dtype == np.uint8 and image.ndim == 1
        self.arenas.append(Arena(image, RegionAllocator(image.size)))
        return len(self.arenas) - 1

    def alloc_region(self, arena: int, nbytes: int, align: int = DEFAULT_ALIGN) -> Tuple[int, int, int]:
        a = self._arena(arena)
        off = a.alloc.alloc(nbytes, align)
        return (arena, off, nbytes)

    def free_region(self, region: Tuple[int, int, int]) -> None:
        self._arena(region[0]).alloc.release(region[1], region[2])

    def _arena(self, arena: int) -> Arena:
        if not 0 <= arena < len(self.arenas):
            raise OracleError("inval", f"unknown arena {arena}")
        return self.arenas[arena]

    # raw stores, all logged
    def _store(self, kind: str, tensor: int, arena: int, lo: int, data: np.ndarray) -> None:
        mem = self._arena(arena).mem
        hi = lo + data.size
        if hi > mem.size:
            raise OracleError("range", "store outside arena")
        mem[lo:hi] = data
        self.log.append((kind, tensor, arena, lo, hi))

    def _store_u32(self, kind: str, tensor: int, arena: int, off: int, value: int) -> None:
        self._store(kind, tensor, arena, off, np.frombuffer(struct.pack("<I", value), dtype=np.uint8))

    def _load_u32(self, arena: int, off: int) -> int:
        return struct.unpack_from("<I", self._arena(arena).mem, off)[0]


# ---------------------------------------------------------------------------
# sections 3.2-3.4: classification and placement (the static plan)
# ---------------------------------------------------------------------------
@dataclass
class TensorDesc:
    tensor_id: int
    dtype: int
    dims: Tuple[int, ...]           # -1 = unknown at plan time
    dst_arena: int


@dataclass
class Placement:
    tensor_id: int
    kind: int
    dst_arena: int
    data_offset: int = 0            # static: payload start
    nbytes: int = 0                 # static: payload bytes
    flag_offset: int = 0            # static: completion flag; dynamic: metadata flag
    meta_offset: int = 0            # dynamic: start of the metadata record
    region_bytes: int = 0


@dataclass
class ArenaPlan:
    base: int = 0                   # offset of the plan's block inside the arena
    static_bytes: int = 0           # regions + metadata slots
    heap_offset: int = 0
    heap_bytes: int = 0
    heap_ptr: int = 0               # bump pointer, relative to heap_offset

    @property
    def total_bytes(self) -> int:
        return self.static_bytes + self.heap_bytes


@dataclass
class Plan:
    align: int
    placements: List[Placement]
    arenas: Dict[int, ArenaPlan]
    by_id: Dict[int, int] = field(default_factory=dict)
    descs: Dict[int, TensorDesc] = field(default_factory=dict)
    rpc_offsets: Dict[int, int] = field(default_factory=dict)   # tensor -> heap offset of the last RPC delivery
    dyn_meta: Dict[int, bytes] = field(default_factory=dict)    # tensor -> record seen by the last metadata poll

    def get(self, tensor_id: int) -> Placement:
        if tensor_id not in self.by_id:
            raise OracleError("inval", f"unknown tensor {tensor_id}")
        return self.placements[self.by_id[tensor_id]]


def classify(desc: TensorDesc, max_static_bytes: int = 0) -> int:
    """Static iff every dim is known before the computation starts (section 3.4);
    the rank is always known (section 3.3).  A known-size tensor larger than
    max_static_bytes (when non-zero) is sent dynamically to save footprint
    (introduction, item (ii))."""
    if len(desc.dims) > MAX_DIMS:
        raise OracleError("inval", "rank too large")
    if desc.dtype not in DTYPE_SIZE:
        raise OracleError("inval", "unknown dtype")
    if any(d < -1 for d in desc.dims):
        raise OracleError("inval", "negative dim")
    if any(d == -1 for d in desc.dims):
        return DYNAMIC
    nb = tensor_nbytes(desc.dtype, desc.dims)
    if max_static_bytes and nb > max_static_bytes:
        return DYNAMIC
    return STATIC


def place(descs: Sequence[TensorDesc], align: int = DEFAULT_ALIGN, max_static_bytes: int = 0,
          dyn_heap_bytes: int = 0):
    """Offsets relative to each arena's plan block.  Per arena, in input order:
    a static tensor gets [payload | pad to 16 | 4-byte flag | pad to align];
    a dynamic tensor gets one metadata slot (its last word is the metadata flag,
    the word before it the payload-complete flag); the dynamic heap follows."""
    if align < 16 or align & (align - 1):
        raise OracleError("align", "alignment must be a power of two >= 16")
    seen = set()
    ptr: Dict[int, int] = {}
    out: List[Placement] = []
    for d in descs:
        if d.tensor_id in seen:
            raise OracleError("inval", "duplicate tensor id")
        seen.add(d.tensor_id)
        kind = classify(d, max_static_bytes)
        p = ptr.setdefault(d.dst_arena, 0)
        if kind == STATIC:
            nb = tensor_nbytes(d.dtype, d.dims)
            padded = round_up(nb, 16)
            region = round_up(padded + 16, align)
            pl = Placement(d.tensor_id, STATIC, d.dst_arena, data_offset=p, nbytes=nb,
                           flag_offset=p + padded, region_bytes=region)
        else:
            region = round_up(META_BYTES, align)
            pl = Placement(d.tensor_id, DYNAMIC, d.dst_arena, meta_offset=p,
                           flag_offset=p + META_BYTES - 4, region_bytes=region)
        if p + region > U64_MAX:
            raise OracleError("overflow", "arena offsets exceed 64 bits")
        ptr[d.dst_arena] = p + region
        out.append(pl)
    heap = round_up(dyn_heap_bytes, align)
    arenas = {a: ArenaPlan(0, p, p, heap, 0) for a, p in ptr.items()}
    for ap in arenas.values():
        if ap.static_bytes + ap.heap_bytes > U64_MAX:
            raise OracleError("overflow", "arena bytes exceed 64 bits")
    return out, arenas


def plan(dev: Device, descs: Sequence[TensorDesc], align: int = DEFAULT_ALIGN,
         max_static_bytes: int = 0, dyn_heap_bytes: int = 0) -> Plan:
    """Pre-allocate the receiver side: one block per destination arena taken
    from that arena's sub-allocator, regions inside it by prefix sums."""
    placements, arenas = place(descs, align, max_static_bytes, dyn_heap_bytes)
    for a in arenas:
        dev._arena(a)
    done = []
    try:
        for a in sorted(arenas):
            ap = arenas[a]
            if ap.total_bytes == 0:
                continue
            _, base, _ = dev.alloc_region(a, ap.total_bytes, align)
            done.append((a, base, ap.total_bytes))
            ap.base = base
            ap.heap_offset += base
    except OracleError:
        for r in done:
            dev.free_region(r)
        raise
    for pl in placements:
        b = arenas[pl.dst_arena].base
        pl.data_offset += b if pl.kind == STATIC else 0
        pl.meta_offset += b if pl.kind == DYNAMIC else 0
        pl.flag_offset += b
    # a flag must read "not set" before the first transfer: the pre-allocation
    # step clears each static region's flag word and each metadata slot
    for pl in placements:
        if dev.arenas[pl.dst_arena].mem.size == 0:
            continue                # layout-only arena (no backing bytes)
        if pl.kind == STATIC:
            dev._store_u32("init", pl.tensor_id, pl.dst_arena, pl.flag_offset, 0)
        else:
            dev._store("init", pl.tensor_id, pl.dst_arena, pl.meta_offset, np.zeros(META_BYTES, dtype=np.uint8))
    p = Plan(align, placements, arenas)
    p.by_id = {pl.tensor_id: i for i, pl in enumerate(placements)}
    p.descs = {d.tensor_id: d for d in descs}
    return p


# ---------------------------------------------------------------------------
# section 3.3: the metadata record
# ---------------------------------------------------------------------------
# byte offsets: ndims 0, dtype 4, bytes 8, src_offset 16, dims 24, dst_offset 88,
# src_arena 96, tensor_id 100, seq 104, reserved 108..119, data_flag 120, meta_flag 124
_META = struct.Struct("<IIQQ8qQIII3III")
assert _META.size == META_BYTES


def encode_meta(ndims: int, dtype: int, nbytes: int, src_arena: int, src_offset: int,
                dims: Sequence[int], tensor_id: int, seq: int, dst_offset: int = 0,
                data_flag: int = 0, meta_flag: int = 0) -> bytes:
    d = list(dims) + [0] * (MAX_DIMS - len(dims))
    return _META.pack(ndims, dtype, nbytes, src_offset, *d, dst_offset, src_arena, tensor_id, seq,
                      0, 0, 0, data_flag, meta_flag)


def decode_meta(rec: bytes) -> dict:
    f = _META.unpack(bytes(rec))
    return dict(ndims=f[0], dtype=f[1], nbytes=f[2], src_offset=f[3], dims=tuple(f[4:12]),
                dst_offset=f[12], src_arena=f[13], tensor_id=f[14], seq=f[15],
                data_flag=f[19], meta_flag=f[20])


# ---------------------------------------------------------------------------
# section 3.2: static transfer, flag, poll
# ---------------------------------------------------------------------------
def _check_src(dev: Device, src: Tuple[int, int], nbytes: int) -> None:
    a = dev._arena(src[0])
    if src[1] < 0 or src[1] + nbytes > a.mem.size:
        raise OracleError("range", "source outside its arena")


def _check_disjoint(src: Tuple[int, int], dst: Tuple[int, int], nbytes: int) -> None:
    if nbytes and src[0] == dst[0] and src[1] < dst[1] + nbytes and dst[1] < src[1] + nbytes:
        raise OracleError("overlap", "source and destination ranges overlap")


def static_write(dev: Device, pl: Plan, sources: Dict[int, Tuple[int, int]], seq: int,
                 tensor_ids: Optional[Sequence[int]] = None) -> None:
    """One-sided write of each static tensor into its pre-allocated region, then
    its flag.  sources: tensor_id -> (sender arena, offset).  A batch is
    validated as a whole before anything moves."""
    if seq < 1:
        raise OracleError("inval", "seq must be >= 1")
    ids = [p.tensor_id for p in pl.placements if p.kind == STATIC] if tensor_ids is None else list(tensor_ids)
    for t in ids:
        p = pl.get(t)
        if p.kind != STATIC:
            raise OracleError("inval", "not a static tensor")
        if t not in sources:
            raise OracleError("inval", "no source bound")
        _check_src(dev, sources[t], p.nbytes)
        _check_disjoint(sources[t], (p.dst_arena, p.data_offset), p.nbytes)
    for t in ids:
        p = pl.get(t)
        sa, so = sources[t]
        data = dev.arenas[sa].mem[so:so + p.nbytes].copy()
        dev._store("payload", t, p.dst_arena, p.data_offset, data)
        dev._store_u32("flag_set", t, p.dst_arena, p.flag_offset, seq)
        pl.rpc_offsets.pop(t, None)         # the tensor now sits in its static region again


POLL_META, POLL_DATA = 0, 1


def poll(dev: Device, pl: Plan, tensor_id: int, consume: bool = False, which: int = POLL_DATA):
    """Non-blocking completion test (section 3.2: the receiver polls the flag and
    clears it on success).  Static tensor: the region's flag.  Dynamic tensor:
    which=POLL_META tests the metadata flag and returns the record,
    which=POLL_DATA tests the payload-complete flag.
    Returns (ready, record-or-None)."""
    p = pl.get(tensor_id)
    if p.kind == STATIC:
        ready = dev._load_u32(p.dst_arena, p.flag_offset) != 0
        if ready and consume:
            dev._store_u32("flag_clear", tensor_id, p.dst_arena, p.flag_offset, 0)
        meta = None
        if ready and tensor_id in pl.rpc_offsets:
            meta = {"dst_offset": pl.rpc_offsets[tensor_id]}
        return ready, meta
    off = p.meta_offset + (124 if which == POLL_META else 120)
    ready = dev._load_u32(p.dst_arena, off) != 0
    rec = None
    if ready:
        rec = bytes(dev.arenas[p.dst_arena].mem[p.meta_offset:p.meta_offset + META_BYTES])
        if which == POLL_META:
            pl.dyn_meta[tensor_id] = rec
        if consume:
            dev._store_u32("flag_clear", tensor_id, p.dst_arena, off, 0)
    return ready, (decode_meta(rec) if rec is not None else None)


# ---------------------------------------------------------------------------
# section 3.3: dynamic transfer
# ---------------------------------------------------------------------------
def dyn_reset(pl: Plan) -> None:
    """Start of an iteration: the receiver's dynamic heaps are empty again."""
    for ap in pl.arenas.values():
        ap.heap_ptr = 0


def _heap_alloc(pl: Plan, arena: int, nbytes: int) -> int:
    ap = pl.arenas[arena]
    need = round_up(nbytes, pl.align)
    if ap.heap_ptr + need > ap.heap_bytes:
        raise OracleError("nomem", "dynamic heap exhausted")
    off = ap.heap_offset + ap.heap_ptr
    ap.heap_ptr += need
    return off


def dyn_send(dev: Device, pl: Plan, tensor_id: int, src: Tuple[int, int], dtype: int,
             dims: Sequence[int], seq: int) -> None:
    """Sender: write the metadata record (flags zero) into the receiver's slot
    except for its last word, then that last word = seq (the metadata flag).
    The payload-complete word (offset 120) is left as the receiver keeps it."""
    p = pl.get(tensor_id)
    if p.kind != DYNAMIC:
        raise OracleError("inval", "not a dynamic tensor")
    if seq < 1:
        raise OracleError("inval", "seq must be >= 1")
    nb = tensor_nbytes(dtype, dims)
    _check_src(dev, src, nb)
    rec = encode_meta(len(dims), dtype, nb, src[0], src[1], dims, tensor_id, seq)
    dev._store("meta", tensor_id, p.dst_arena, p.meta_offset,
               np.frombuffer(rec[:120], dtype=np.uint8))
    dev._store_u32("flag_set", tensor_id, p.dst_arena, p.meta_offset + 124, seq)


def dyn_recv(dev: Device, pl: Plan, tensor_id: int, seq: int) -> int:
    """Receiver, after a successful metadata poll: allocate storage in the
    arena's dynamic heap, record the chosen offset in the slot, pull the payload
    from the sender's address, then set the payload-complete flag.
    Returns the destination offset."""
    p = pl.get(tensor_id)
    if p.kind != DYNAMIC:
        raise OracleError("inval", "not a dynamic tensor")
    if tensor_id not in pl.dyn_meta:
        raise OracleError("state", "metadata has not been polled")
    m = decode_meta(pl.dyn_meta.pop(tensor_id))
    nb = m["nbytes"]
    src = (m["src_arena"], m["src_offset"])
    _check_src(dev, src, nb)
    dst = _heap_alloc(pl, p.dst_arena, nb)
    _check_disjoint(src, (p.dst_arena, dst), nb)
    dev._store("meta", tensor_id, p.dst_arena, p.meta_offset + 88,
               np.frombuffer(struct.pack("<Q", dst), dtype=np.uint8))
    data = dev.arenas[src[0]].mem[src[1]:src[1] + nb].copy()
    dev._store("payload", tensor_id, p.dst_arena, dst, data)
    dev._store_u32("flag_set", tensor_id, p.dst_arena, p.meta_offset + 120, seq)
    return dst


# ---------------------------------------------------------------------------
# sections 2.2, 5.1: RPC-style copy path and the sender staging copy
# ---------------------------------------------------------------------------
FRAG_HEADER_BYTES = 32
_FRAG = struct.Struct("<IIIIQII")      # tensor_id, seq, frag_index, frag_count, offset, bytes, reserved
assert _FRAG.size == FRAG_HEADER_BYTES


def rpc_message_bytes(nbytes: int, frag_bytes: int = 0) -> int:
    """header || payload || pad to 16; or, fragmented (section 2.2): header, then
    per fragment a 32-byte fragment header || piece || pad to 16."""
    if not frag_bytes:
        return META_BYTES + round_up(nbytes, 16)
    total = META_BYTES
    for off in range(0, nbytes, frag_bytes):
        total += FRAG_HEADER_BYTES + round_up(min(frag_bytes, nbytes - off), 16)
    return total


def _header(pl: Plan, tensor_id: int, src_arena: int, src_offset: int, seq: int) -> bytes:
    """Message header of a static tensor: the same record as the dynamic path's
    metadata, filled from the plan-time description."""
    d = pl.descs[tensor_id]
    nb = tensor_nbytes(d.dtype, d.dims)
    return encode_meta(len(d.dims), d.dtype, nb, src_arena, src_offset, d.dims, tensor_id, seq)


def copy_write(dev: Device, pl: Plan, sources: Dict[int, Tuple[int, int]], mode: int, seq: int,
               send_buf: Tuple[int, int, int], recv_buf: Optional[Tuple[int, int, int]] = None,
               tensor_ids: Optional[Sequence[int]] = None, frag_bytes: int = 0) -> None:
    """The copying alternatives for a batch of static tensors.

    RPC2: pack header||payload||zero pad into send_buf back to back; unpack:
          parse each header, allocate fresh storage in the receiver's dynamic
          heap, copy the payload out, set the tensor's flag.
    RPC3: as RPC2 with the packed bytes copied send_buf -> recv_buf in between
          and unpacked from recv_buf.
    SENDERCOPY: copy each source into send_buf (align-spaced, no header), then
          the zero-copy write from there into the static region + flag."""
    if seq < 1:
        raise OracleError("inval", "seq must be >= 1")
    ids = [p.tensor_id for p in pl.placements if p.kind == STATIC] if tensor_ids is None else list(tensor_ids)
    for t in ids:
        p = pl.get(t)
        if p.kind != STATIC:
            raise OracleError("inval", "not a static tensor")
        if t not in sources:
            raise OracleError("inval", "no source bound")
        _check_src(dev, sources[t], p.nbytes)
    sb_arena, sb_off, sb_bytes = send_buf
    if mode == MODE_SENDERCOPY:
        ptr = 0
        staged = {}
        for t in ids:
            p = pl.get(t)
            if ptr + p.nbytes > sb_bytes:
                raise OracleError("nomem", "staging buffer too small")
            staged[t] = (sb_arena, sb_off + ptr)
            ptr += round_up(p.nbytes, pl.align)
        for t in ids:
            p = pl.get(t)
            sa, so = sources[t]
            dev._store("stage", t, sb_arena, staged[t][1], dev.arenas[sa].mem[so:so + p.nbytes].copy())
        static_write(dev, pl, staged, seq, ids)
        return
    if mode not in (MODE_RPC2, MODE_RPC3):
        raise OracleError("inval", "unknown mode")
    if frag_bytes % 16:
        raise OracleError("inval", "fragment size must be a multiple of 16")
    total = sum(rpc_message_bytes(pl.get(t).nbytes, frag_bytes) for t in ids)
    if total > sb_bytes or (mode == MODE_RPC3 and (recv_buf is None or total > recv_buf[2])):
        raise OracleError("nomem", "message buffer too small")
    # heap space is claimed for the whole batch before anything moves
    need: Dict[int, int] = {}
    for t in ids:
        p = pl.get(t)
        need[p.dst_arena] = need.get(p.dst_arena, 0) + round_up(p.nbytes, pl.align)
    for a, n in need.items():
        ap = pl.arenas[a]
        if ap.heap_ptr + n > ap.heap_bytes:
            raise OracleError("nomem", "dynamic heap exhausted")
    # pack
    ptr = 0
    offs = []
    for t in ids:
        p = pl.get(t)
        sa, so = sources[t]
        rec = _header(pl, t, sa, so, seq)
        msg = np.zeros(rpc_message_bytes(p.nbytes, frag_bytes), dtype=np.uint8)
        msg[:META_BYTES] = np.frombuffer(rec, dtype=np.uint8)
        if not frag_bytes:
            msg[META_BYTES:META_BYTES + p.nbytes] = dev.arenas[sa].mem[so:so + p.nbytes]
        else:
            nfrag = -(-p.nbytes // frag_bytes)
            cur = META_BYTES
            for k in range(nfrag):
                off = k * frag_bytes
                fb = min(frag_bytes, p.nbytes - off)
                msg[cur:cur + FRAG_HEADER_BYTES] = np.frombuffer(_FRAG.pack(t, seq, k, nfrag, off, fb, 0), dtype=np.uint8)
                msg[cur + FRAG_HEADER_BYTES:cur + FRAG_HEADER_BYTES + fb] = dev.arenas[sa].mem[so + off:so + off + fb]
                cur += FRAG_HEADER_BYTES + round_up(fb, 16)
        dev._store("pack", t, sb_arena, sb_off + ptr, msg)
        offs.append(ptr)
        ptr += msg.size
    buf_arena, buf_off = sb_arena, sb_off
    if mode == MODE_RPC3:
        dev._store("wire", -1, recv_buf[0], recv_buf[1], dev.arenas[sb_arena].mem[sb_off:sb_off + total].copy())
        buf_arena, buf_off = recv_buf[0], recv_buf[1]
    # unpack: everything is taken from the buffer bytes
    mem = dev.arenas[buf_arena].mem
    cur = 0
    for _ in ids:
        m = decode_meta(bytes(mem[buf_off + cur:buf_off + cur + META_BYTES]))
        t, nb = m["tensor_id"], m["nbytes"]
        p = pl.get(t)
        dst = _heap_alloc(pl, p.dst_arena, nb)
        if not frag_bytes:
            data = mem[buf_off + cur + META_BYTES:buf_off + cur + META_BYTES + nb].copy()
            dev._store("payload", t, p.dst_arena, dst, data)
            cur += rpc_message_bytes(nb)
        else:
            # re-assembly: walk the fragment headers until the whole tensor has arrived
            cur += META_BYTES
            got = 0
            while got < nb:
                ft, fseq, fk, fn, foff, fb, _ = _FRAG.unpack(bytes(mem[buf_off + cur:buf_off + cur + FRAG_HEADER_BYTES]))
                if ft != t or fseq != m["seq"] or foff + fb > nb:
                    raise OracleError("state", "fragment does not belong to this message")
                piece = mem[buf_off + cur + FRAG_HEADER_BYTES:buf_off + cur + FRAG_HEADER_BYTES + fb].copy()
                dev._store("payload", t, p.dst_arena, dst + foff, piece)
                got += fb
                cur += FRAG_HEADER_BYTES + round_up(fb, 16)
        dev._store_u32("flag_set", t, p.dst_arena, p.flag_offset, m["seq"])
        pl.rpc_offsets[t] = dst


# ---------------------------------------------------------------------------
# workload side of the sparse-gradient case (section 3.3 motivation: shapes that
# depend on the mini-batch)
# ---------------------------------------------------------------------------
def gather_unique_rows(ids: np.ndarray, table: np.ndarray):
    """Rows of `table` touched by the mini-batch's token ids, ascending id, each once."""
    u = np.unique(np.asarray(ids).reshape(-1))
    return u.astype(np.int64), table[u]


# ---------------------------------------------------------------------------
# section 3.4: sender-side allocation-site tracing
# ---------------------------------------------------------------------------
class Tracer:
    """The instrumented allocator of the sender's runtime.

    First mini-batch: every allocation is recorded as address -> (node id, index
    of the allocation within that node's execution); an allocation that reuses an
    address replaces the older entry.  When a tensor is sent, its buffer address
    is looked up and the allocation site found goes into the set S.  Later
    mini-batches: an allocation whose site is in S is served from the registered
    arena, all others from the ordinary (unregistered) pool.  A tensor sent from
    the pool is first copied into a freshly allocated registered staging buffer.
    """

    def __init__(self, dev: Device, pool: np.ndarray, arena: int):
        dev._arena(arena)
        self.dev, self.pool, self.arena = dev, pool, arena
        self.pool_alloc = RegionAllocator(pool.size)
        self.iteration = 0
        self.next_index: Dict[int, int] = {}
        self.site_of: Dict[Tuple[str, int], Tuple[int, int]] = {}    # address -> allocation site
        self.S: List[Tuple[int, int]] = []
        self.live: Dict[Tuple[str, int], int] = {}                    # address -> bytes
        self.staging: List[Tuple[int, int, int]] = []

    def _release_all(self) -> None:
        for (where, off), nb in self.live.items():
            (self.dev.arenas[self.arena].alloc if where == "arena" else self.pool_alloc).release(off, nb)
        self.live.clear()
        for r in self.staging:
            self.dev.free_region(r)
        self.staging.clear()

    def begin_iteration(self) -> None:
        self._release_all()
        self.next_index.clear()
        self.iteration += 1

    def alloc(self, node: int, nbytes: int) -> Tuple[str, int, int]:
        """Returns (where, offset, allocation index)."""
        if self.iteration == 0:
            raise OracleError("state", "no iteration begun")
        idx = self.next_index.get(node, 0)
        where = "arena" if self.iteration > 1 and (node, idx) in self.S else "pool"
        a = self.dev.arenas[self.arena].alloc if where == "arena" else self.pool_alloc
        off = a.alloc(nbytes, 256)
        self.next_index[node] = idx + 1
        self.live[(where, off)] = nbytes
        if self.iteration == 1:
            self.site_of[(where, off)] = (node, idx)
        return where, off, idx

    def free(self, where: str, off: int) -> None:
        nb = self.live.pop((where, off), None)
        if nb is None:
            raise OracleError("inval", "not a live buffer")
        (self.dev.arenas[self.arena].alloc if where == "arena" else self.pool_alloc).release(off, nb)

    def buffer(self, where: str, off: int, nbytes: int) -> np.ndarray:
        mem = self.dev.arenas[self.arena].mem if where == "arena" else self.pool
        return mem[off:off + nbytes]

    def send(self, pl: Plan, tensor_id: int, where: str, off: int, seq: int) -> bool:
        """Returns True when the tensor had to be staged (copied)."""
        p = pl.get(tensor_id)
        if p.kind != STATIC:
            raise OracleError("inval", "not a static tensor")
        if (where, off) not in self.live:
            raise OracleError("inval", "not a live buffer")
        if self.live[(where, off)] < p.nbytes:
            raise OracleError("range", "buffer smaller than the tensor")
        copied = where != "arena"
        src = (self.arena, off)
        stage = None
        if copied:
            if p.nbytes:
                stage = self.dev.alloc_region(self.arena, p.nbytes, 256)
                src = (self.arena, stage[1])
            else:
                src = (self.arena, 0)
        try:
            _check_src(self.dev, src, p.nbytes)
            _check_disjoint(src, (p.dst_arena, p.data_offset), p.nbytes)
        except OracleError:
            if stage:
                self.dev.free_region(stage)
            raise
        if self.iteration == 1:
            site = self.site_of.get((where, off))
            if site is not None and site not in self.S:
                self.S.append(site)
        if copied and p.nbytes:
            self.staging.append(stage)
            self.dev._store("stage", tensor_id, self.arena, stage[1], self.pool[off:off + p.nbytes].copy())
        static_write(self.dev, pl, {tensor_id: src}, seq, [tensor_id])
        return copied


# ---------------------------------------------------------------------------
# section 5.1: the receiver's light consumer (reduce_max) of the micro-benchmark
# ---------------------------------------------------------------------------
def consume_reduce_max(dev: Device, pl: Plan, tensor_id: int, from_offset: Optional[int] = None):
    """(max, word_sum) of a delivered static tensor read as 32-bit words:
    max over the fp32 values that are not NaN, with -0 below +0, -inf when
    nothing is left; word_sum = sum of the words modulo 2^64."""
    p = pl.get(tensor_id)
    if p.kind != STATIC or p.nbytes % 4:
        raise OracleError("inval", "consumer takes static tensors of 32-bit elements")
    off = p.data_offset if from_offset is None else from_offset
    words = dev.arenas[p.dst_arena].mem[off:off + p.nbytes].copy().view("<u4")
    word_sum = 0
    for chunk in np.array_split(words, max(1, words.size // (1 << 20))):
        word_sum = (word_sum + int(chunk.astype(np.uint64).sum(dtype=np.uint64))) % (1 << 64)
    vals = words.view(np.float32)
    vals = vals[~np.isnan(vals)]
    if vals.size == 0:
        return np.float32(-np.inf), word_sum
    mx = vals.max()
    if mx == 0:
        plus_zero = bool((vals.view("<u4") == 0).any())
        mx = np.float32(0.0) if plus_zero else np.float32(-0.0)
    return np.float32(mx), word_sum
