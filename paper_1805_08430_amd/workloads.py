"""Seeded synthetic tensor sets shaped like the paper's CNN / RNN workloads.

This module only *describes inputs*: which tensors cross the partition (name,
element type, dims, receiving arena), where each source tensor sits in its
sender arena, and the bytes the sender holds.  It contains no placement,
transfer, flag or metadata logic; the CPU checker and the GPU library each
receive these inputs and compute everything else on their own.

The sets follow the evaluation section's workload description (Table 1 and the
tensor-size CCDF remark in section 5): parameter / gradient tensors of
AlexNet-, VGG-16-, Inception-v3- and LSTM-shaped models placed round-robin on
parameter-server arenas, fp32, synthetic random contents.

Everything is drawn from ``numpy.random.Generator(PCG64(seed))`` with
``seed = SEED_BASE + config index`` so that two callers get identical bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

SEED_BASE = 18050843

_ITEMSIZE = {"u8": 1, "i8": 1, "i16": 2, "i32": 4, "i64": 8,
             "f16": 2, "bf16": 2, "f32": 4, "f64": 8}


def itemsize(dtype: str) -> int:
    return _ITEMSIZE[dtype]


@dataclass
class TensorSpec:
    """One tensor crossing the partition.

    dims: plan-time dims, -1 where a dim is unknown until run time.
    dst_arena: index into the workload's receiver arenas (0-based).
    src_arena: index into the workload's sender arenas (0-based).
    src_offset: byte offset of the source tensor in its sender arena
                (None for dynamic tensors whose source is produced per iteration).
    """
    name: str
    dtype: str
    dims: Tuple[int, ...]
    dst_arena: int = 0
    src_arena: int = 0
    src_offset: Optional[int] = None

    @property
    def is_static(self) -> bool:
        return all(d >= 0 for d in self.dims)

    @property
    def nbytes(self) -> int:
        assert self.is_static
        n = _ITEMSIZE[self.dtype]
        for d in self.dims:
            n *= d
        return n


@dataclass
class Workload:
    name: str
    seed: int
    tensors: List[TensorSpec]
    n_sender_arenas: int
    n_receiver_arenas: int
    sender_bytes: List[int]           # bytes needed per sender arena for static sources
    fill: str                         # "bits" (uniform 32-bit patterns) or "normal" (N(0, 0.01))
    notes: str = ""
    extra: Dict[str, object] = field(default_factory=dict)

    @property
    def static_tensors(self) -> List[TensorSpec]:
        return [t for t in self.tensors if t.is_static]

    @property
    def payload_bytes(self) -> int:
        return sum(t.nbytes for t in self.static_tensors)


def _round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


def _pack_sources(tensors: Sequence[TensorSpec], n_sender: int, gran: int) -> List[int]:
    """Lay the static source tensors out back to back in their sender arenas."""
    ptr = [0] * n_sender
    for t in tensors:
        if not t.is_static:
            continue
        ptr[t.src_arena] = _round_up(ptr[t.src_arena], gran)
        t.src_offset = ptr[t.src_arena]
        ptr[t.src_arena] += t.nbytes
    return [_round_up(p, 256) + 256 for p in ptr]


def poison(nbytes: int, seed: int) -> np.ndarray:
    """Seeded background pattern for an arena: whatever the transfer does not
    write must still hold these bytes afterwards."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x5EED))
    # a short random period repeated: cheap for GB-sized arenas, still not
    # something a stray write could reproduce by accident.
    period = rng.integers(0, 256, size=65521, dtype=np.uint8)  # prime length
    reps = nbytes // period.size + 1
    return np.tile(period, reps)[:nbytes].copy()


def fill_sources(wl: Workload, variant: int = 0) -> List[np.ndarray]:
    """Sender-arena images (uint8) holding every static source tensor.

    variant: different contents for the same layout (iteration number, or
    worker number for the multi-worker set)."""
    rng = np.random.Generator(np.random.PCG64(wl.seed * 1000003 + variant))
    arenas = [poison(n, wl.seed + 77 + 131 * variant + i) for i, n in enumerate(wl.sender_bytes)]
    for t in wl.static_tensors:
        nb = t.nbytes
        if nb == 0:
            continue
        dst = arenas[t.src_arena][t.src_offset:t.src_offset + nb]
        if wl.fill == "bits" or t.dtype not in ("f32",):
            dst[:] = rng.integers(0, 256, size=nb, dtype=np.uint8)
        else:
            n = nb // 4
            out = np.empty(n, dtype=np.float32)
            step = 1 << 22
            for lo in range(0, n, step):
                hi = min(n, lo + step)
                out[lo:hi] = rng.normal(0.0, 0.01, size=hi - lo).astype(np.float32)
            dst[:] = out.view(np.uint8)
    return arenas


# --------------------------------------------------------------------------
# config 0: tiny
# --------------------------------------------------------------------------
def tiny() -> Workload:
    """16 static fp32 tensors, element counts log-uniform in [1024, 262144)
    (4 KB - 1 MB), random bit patterns, packed at 4-byte granularity so that
    source and destination are mutually misaligned; plus 2 dynamic [rows, 256]
    fp32 tensors whose row count is drawn per iteration."""
    seed = SEED_BASE + 0
    rng = np.random.Generator(np.random.PCG64(seed))
    tensors = []
    for i in range(16):
        n = int(np.floor(np.exp(rng.uniform(np.log(1024.0), np.log(262144.0)))))
        tensors.append(TensorSpec(f"s{i}", "f32", (n,), 0, 0))
    tensors.append(TensorSpec("d0", "f32", (-1, 256), 0, 0))
    tensors.append(TensorSpec("d1", "f32", (-1, 256), 0, 0))
    sb = _pack_sources(tensors, 1, 4)
    return Workload("tiny", seed, tensors, 1, 1, sb, "bits",
                    "16 static + 2 dynamic, 1 sender arena -> 1 receiver arena")


def tiny_dynamic_rows(iteration: int) -> Tuple[int, int]:
    rng = np.random.Generator(np.random.PCG64((SEED_BASE + 0) * 7919 + iteration))
    r = rng.integers(1, 513, size=2)
    return int(r[0]), int(r[1])


def dynamic_payload(nbytes: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, 256, size=nbytes, dtype=np.uint8)


# --------------------------------------------------------------------------
# config 1 / 2: AlexNet- and VGG-16-shaped parameter sets
# --------------------------------------------------------------------------
def _wb_list(layers: Sequence[Tuple[str, Tuple[int, ...]]], n_recv: int) -> List[TensorSpec]:
    out = []
    for name, shape in layers:
        out.append(TensorSpec(name + ".W", "f32", tuple(shape), len(out) % n_recv, 0))
        out.append(TensorSpec(name + ".b", "f32", (shape[0],), len(out) % n_recv, 0))
    return out


def alexnet() -> Workload:
    seed = SEED_BASE + 1
    layers = [("conv1", (96, 3, 11, 11)), ("conv2", (256, 96, 5, 5)), ("conv3", (384, 256, 3, 3)),
              ("conv4", (384, 384, 3, 3)), ("conv5", (256, 384, 3, 3)), ("fc6", (4096, 9216)),
              ("fc7", (4096, 4096)), ("fc8", (1000, 4096))]
    tensors = _wb_list(layers, 1)
    sb = _pack_sources(tensors, 1, 256)
    return Workload("alexnet", seed, tensors, 1, 1, sb, "normal",
                    "8 weight + 8 bias tensors, ungrouped shapes as listed")


def vgg16(misalign=False) -> Workload:
    """misalign=True: the same tensors, but source k starts k mod 16 bytes off a 16-byte boundary, so that every
    alignment class of the copy routine (16-byte, 4-byte, byte) is exercised on full-size tensors.
    misalign=n (1..15): every source starts n bytes off a 16-byte boundary."""
    seed = SEED_BASE + 2
    chans = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256),
             (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
    layers = [(f"conv{i + 1}", (co, ci, 3, 3)) for i, (ci, co) in enumerate(chans)]
    layers += [("fc14", (4096, 25088)), ("fc15", (4096, 4096)), ("fc16", (1000, 4096))]
    tensors = _wb_list(layers, 8)
    sb = _pack_sources(tensors, 1, 256)
    if misalign:
        shift = 0
        for k, t in enumerate(tensors):
            shift += 16
            # keeps the sources apart; walks through all 16 offsets, or applies the one that was asked for
            t.src_offset += shift + ((k % 16) if misalign is True else int(misalign) % 16)
        sb = [sb[0] + shift + 64]
    return Workload("vgg16", seed, tensors, 1, 8, sb, "normal",
                    "16 weight + 16 bias tensors, tensor i -> receiver arena i mod 8")


# --------------------------------------------------------------------------
# config 3: 2-layer LSTM language model
# --------------------------------------------------------------------------
LSTM_VOCAB = 40000
LSTM_WIDTH = 1024
LSTM_BATCH = 64
LSTM_SEQ = 35


def lstm() -> Workload:
    """Dense gradients (two 4096x2048 LSTM matrices, 40000x1024 softmax) are
    static; the embedding gradient is sparse: the rows touched by the token ids
    of one mini-batch, so its first dim is unknown at plan time."""
    seed = SEED_BASE + 3
    tensors = [TensorSpec("lstm0.W", "f32", (4096, 2048), 0, 0),
               TensorSpec("lstm1.W", "f32", (4096, 2048), 0, 0),
               TensorSpec("softmax.W", "f32", (LSTM_VOCAB, LSTM_WIDTH), 0, 0),
               TensorSpec("emb.ids", "i64", (-1,), 0, 0),
               TensorSpec("emb.rows", "f32", (-1, LSTM_WIDTH), 0, 0)]
    sb = _pack_sources(tensors, 1, 256)
    return Workload("lstm", seed, tensors, 1, 1, sb, "normal",
                    "3 dense static grads + sparse embedding grad (ids, rows) dynamic")


def zipf_pmf(n: int, s: float) -> np.ndarray:
    k = np.arange(1, n + 1, dtype=np.float64)
    p = k ** (-s)
    return p / p.sum()


def lstm_token_ids(iteration: int) -> np.ndarray:
    """batch x seq token ids, finite Zipf(s=1.1) over the vocabulary, id = rank-1."""
    rng = np.random.Generator(np.random.PCG64((SEED_BASE + 3) * 7919 + iteration))
    pmf = zipf_pmf(LSTM_VOCAB, 1.1)
    ids = rng.choice(LSTM_VOCAB, size=(LSTM_BATCH, LSTM_SEQ), p=pmf)
    return ids.astype(np.int64)


def lstm_embedding_table(rows: int = LSTM_VOCAB) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64((SEED_BASE + 3) * 104729))
    out = np.empty((rows, LSTM_WIDTH), dtype=np.float32)
    step = 4096
    for lo in range(0, rows, step):
        hi = min(rows, lo + step)
        out[lo:hi] = rng.normal(0.0, 0.01, size=(hi - lo, LSTM_WIDTH)).astype(np.float32)
    return out


# --------------------------------------------------------------------------
# config 4: Inception-v3-shaped list, several workers -> one server arena
# --------------------------------------------------------------------------
INCEPTION_WORKERS = 10


def inception(n_workers: int = INCEPTION_WORKERS) -> Workload:
    """Structural stand-in for an Inception-v3 parameter list: 94 conv layers,
    each a weight [kh, kw, Cin, Cout] with batch-norm gamma[Cout] and
    beta[Cout] (128 B - 8 KB), plus two fully connected weight/bias pairs;
    about 24 M fp32 parameters in 286 tensors.  Channel widths are drawn, then
    rescaled until the total lands in [23.2 M, 24.5 M].  The list is replicated
    per worker: worker w's tensors sit in sender arena w and go to slot w of the
    single receiver arena."""
    seed = SEED_BASE + 4
    rng = np.random.Generator(np.random.PCG64(seed))
    widths = np.array([32, 48, 64, 80, 96, 128, 160, 192, 224, 256, 320, 384, 448, 512,
                       768, 1024, 1280, 2048])
    kshapes = [(1, 1), (3, 3), (5, 5), (1, 7), (7, 1), (1, 3), (3, 1)]
    kprob = np.array([0.42, 0.22, 0.04, 0.10, 0.10, 0.06, 0.06])
    n_conv = 94
    # widths grow with depth, with jitter, as in a real CNN
    depth = np.linspace(0.0, 1.0, n_conv)
    base_idx = 1 + depth * 9.5 + rng.normal(0.0, 1.8, size=n_conv)
    ks = rng.choice(len(kshapes), size=n_conv, p=kprob)
    extreme = rng.choice(n_conv, size=4, replace=False)

    def build(scale: float):
        idx = np.clip(np.round(base_idx + scale), 0, len(widths) - 1).astype(int)
        idx[extreme[:2]] = 0                    # a few 32-channel layers: 128 B gamma/beta
        idx[extreme[2:]] = len(widths) - 1      # and 2048-channel ones: 8 KB
        couts = widths[idx]
        cin = 3
        layers = []
        for l in range(n_conv):
            kh, kw = kshapes[ks[l]]
            layers.append((kh, kw, cin, int(couts[l])))
            cin = int(couts[l])
        total = sum(kh * kw * ci * co + 2 * co for kh, kw, ci, co in layers)
        total += 2048 * 1000 + 1000 + 768 * 1000 + 1000
        return layers, total

    lo_s, hi_s = -8.0, 8.0
    layers, total = build(0.0)
    for _ in range(60):
        if 23_200_000 <= total <= 24_500_000:
            break
        mid = 0.5 * (lo_s + hi_s)
        layers, total = build(mid)
        if total > 24_500_000:
            hi_s = mid
        elif total < 23_200_000:
            lo_s = mid
    if not (23_200_000 <= total <= 24_500_000):
        raise RuntimeError(f"inception-shaped generator did not converge: {total}")

    one = []
    for l, (kh, kw, ci, co) in enumerate(layers):
        one.append((f"conv{l}.W", (kh, kw, ci, co)))
        one.append((f"conv{l}.gamma", (co,)))
        one.append((f"conv{l}.beta", (co,)))
    one += [("fc.W", (2048, 1000)), ("fc.b", (1000,)), ("aux_fc.W", (768, 1000)), ("aux_fc.b", (1000,))]

    tensors = []
    for w in range(n_workers):
        for name, shape in one:
            tensors.append(TensorSpec(f"w{w}.{name}", "f32", tuple(shape), 0, w))
    sb = _pack_sources(tensors, n_workers, 256)
    return Workload("inception", seed, tensors, n_workers, 1, sb, "normal",
                    f"{len(one)} tensors x {n_workers} workers -> one server arena",
                    extra={"tensors_per_worker": len(one), "params_per_worker": total})


def small_mixed(seed: int, n: int = 12, max_bytes: int = 5000, n_recv: int = 2,
                dtypes: Sequence[str] = ("u8", "i16", "f32", "f64"), gran: int = 1,
                n_dynamic: int = 0) -> Workload:
    """Small randomised set for CPU-side tests: odd sizes, mixed element types,
    byte-granular source packing, a few zero-size and rank-0 tensors."""
    rng = np.random.Generator(np.random.PCG64(seed))
    tensors = []
    for i in range(n):
        dt = dtypes[int(rng.integers(0, len(dtypes)))]
        kind = int(rng.integers(0, 10))
        if kind == 0:
            dims: Tuple[int, ...] = ()
        elif kind == 1:
            dims = (int(rng.integers(1, 5)), 0)
        else:
            nel = max(1, int(rng.integers(1, max_bytes)) // _ITEMSIZE[dt])
            a = int(rng.integers(1, min(nel, 7) + 1))
            dims = (a, max(1, nel // a))
        tensors.append(TensorSpec(f"t{i}", dt, dims, int(rng.integers(0, n_recv)), 0))
    for i in range(n_dynamic):
        tensors.append(TensorSpec(f"dyn{i}", "f32", (-1, 8), int(rng.integers(0, n_recv)), 0))
    sb = _pack_sources(tensors, 1, gran)
    return Workload(f"mixed{seed}", seed, tensors, 1, n_recv, sb, "bits")


# --------------------------------------------------------------------------
# two more sets shaped after the paper's Table 1
# --------------------------------------------------------------------------
def fcn5() -> Workload:
    """FCN-5-shaped: 784 -> 4096 -> 4096 -> 4096 -> 4096 -> 10, five weight/bias
    pairs = 10 tensors, 53 601 290 fp32 parameters = 204.47 MiB (the size the
    paper's Table 1 lists for its FCN-5), round-robin over 2 receiver arenas."""
    seed = SEED_BASE + 5
    dims = [784, 4096, 4096, 4096, 4096, 10]
    layers = [(f"fc{i + 1}", (dims[i + 1], dims[i])) for i in range(5)]
    tensors = _wb_list(layers, 2)
    sb = _pack_sources(tensors, 1, 256)
    return Workload("fcn5", seed, tensors, 1, 2, sb, "normal", "5 weight + 5 bias tensors")


def gru() -> Workload:
    """GRU-shaped, hidden size 1024, one layer: gate kernel [2048, 2048] + bias,
    candidate kernel [2048, 1024] + bias, output projection [1024, 1000] + bias:
    7 319 528 fp32 parameters = 27.92 MiB (Table 1's size for its GRU)."""
    seed = SEED_BASE + 6
    tensors = [TensorSpec("gru.gates.W", "f32", (2048, 2048), 0, 0), TensorSpec("gru.gates.b", "f32", (2048,), 0, 0),
               TensorSpec("gru.cand.W", "f32", (2048, 1024), 0, 0), TensorSpec("gru.cand.b", "f32", (1024,), 0, 0),
               TensorSpec("proj.W", "f32", (1024, 1000), 0, 0), TensorSpec("proj.b", "f32", (1000,), 0, 0)]
    sb = _pack_sources(tensors, 1, 256)
    return Workload("gru", seed, tensors, 1, 1, sb, "normal", "6 tensors")


def flat(nbytes: int = 553430176, n_recv: int = 1, pieces: int = 1) -> Workload:
    """One sender arena, `pieces` equal fp32 tensors of `nbytes` in total dealt round-robin to `n_recv` receiver
    arenas: the plain large copy, to tell what a tensor set's structure costs on top of it."""
    seed = SEED_BASE + 7
    per = nbytes // pieces // 4
    tensors = [TensorSpec(f"flat{i}", "f32", (per,), i % n_recv, 0) for i in range(pieces)]
    sb = _pack_sources(tensors, 1, 256)
    return Workload("flat", seed, tensors, 1, n_recv, sb, "normal", f"{pieces} tensor(s), {n_recv} receiver arena(s)")


EXTRA_CONFIGS = {"fcn5": fcn5, "gru": gru, "flat": flat}

CONFIGS = {"tiny": tiny, "alexnet": alexnet, "vgg16": vgg16, "lstm": lstm, "inception": inception}
