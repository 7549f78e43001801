"""Pins for the checker's allocator, classifier and planner (CPU only)."""
import os

import numpy as np
import pytest

from oracle import rdev_oracle as O
from paper_1805_08430_amd import workloads as W
import invariants as I
from helpers import GOLDEN, OracleRun, placement_dict, receiver_bytes


def _golden_plan():
    rows = []
    for line in open(os.path.join(GOLDEN, "plan_small.txt")):
        if line.startswith("#") or not line.strip():
            continue
        rows.append([int(x) for x in line.split()])
    return rows


def test_plan_matches_hand_computed_example():
    descs = [O.TensorDesc(0, O.DTYPE_CODE["f32"], (3,), 0),
             O.TensorDesc(1, O.DTYPE_CODE["u8"], (300,), 0),
             O.TensorDesc(2, O.DTYPE_CODE["f32"], (-1, 4), 0),
             O.TensorDesc(3, O.DTYPE_CODE["f64"], (32, 31), 1),
             O.TensorDesc(4, O.DTYPE_CODE["i16"], (0,), 0)]
    pls, arenas = O.place(descs, 256)
    got = [[p.tensor_id, p.kind, p.dst_arena, p.data_offset, p.nbytes, p.flag_offset, p.meta_offset,
            p.region_bytes] for p in pls]
    assert got == _golden_plan()
    assert arenas[0].static_bytes == 1280 and arenas[1].static_bytes == 8192


def test_tensor_nbytes_cases():
    assert O.tensor_nbytes(O.DTYPE_CODE["f32"], ()) == 4            # rank 0 = one element
    assert O.tensor_nbytes(O.DTYPE_CODE["f64"], (3, 0, 5)) == 0
    assert O.tensor_nbytes(O.DTYPE_CODE["bf16"], (7, 3)) == 42
    assert O.tensor_nbytes(O.DTYPE_CODE["u8"], (1 << 32, 1 << 31)) == 1 << 63
    with pytest.raises(O.OracleError) as e:
        O.tensor_nbytes(O.DTYPE_CODE["i64"], (1 << 31, 1 << 31))   # 2^65
    assert e.value.kind == "overflow"
    with pytest.raises(O.OracleError):
        O.tensor_nbytes(99, (1,))
    with pytest.raises(O.OracleError):
        O.tensor_nbytes(0, (1,) * 9)
    # itemsizes against numpy's
    for name, npdt in [("u8", np.uint8), ("i8", np.int8), ("i16", np.int16), ("i32", np.int32),
                       ("i64", np.int64), ("f16", np.float16), ("f32", np.float32), ("f64", np.float64)]:
        assert O.DTYPE_SIZE[O.DTYPE_CODE[name]] == np.dtype(npdt).itemsize
    assert O.DTYPE_SIZE[O.DTYPE_CODE["bf16"]] == 2


def test_classify():
    f32 = O.DTYPE_CODE["f32"]
    assert O.classify(O.TensorDesc(0, f32, (4, 5), 0)) == O.STATIC
    assert O.classify(O.TensorDesc(0, f32, (-1, 5), 0)) == O.DYNAMIC
    assert O.classify(O.TensorDesc(0, f32, (), 0)) == O.STATIC
    assert O.classify(O.TensorDesc(0, f32, (100,), 0), max_static_bytes=400) == O.STATIC
    assert O.classify(O.TensorDesc(0, f32, (101,), 0), max_static_bytes=400) == O.DYNAMIC
    with pytest.raises(O.OracleError):
        O.classify(O.TensorDesc(0, f32, (-2,), 0))


@pytest.mark.parametrize("name", ["tiny", "alexnet", "vgg16", "lstm", "inception"])
@pytest.mark.parametrize("align", [256, 4096])
def test_plan_invariants_on_the_five_configs(name, align):
    wl = W.CONFIGS[name]()
    sizes = receiver_bytes(wl, align, heap=1 << 20)
    dev = O.Device()
    for n in sizes:
        dev.arenas.append(O.Arena(np.zeros(0, dtype=np.uint8), O.RegionAllocator(n)))   # layout only
    descs = [O.TensorDesc(i, O.DTYPE_CODE[t.dtype], tuple(t.dims), t.dst_arena) for i, t in enumerate(wl.tensors)]
    pl = O.plan(dev, descs, align, 0, 1 << 20)
    I.check_plan([placement_dict(p) for p in pl.placements], dict(enumerate(sizes)), align,
                 bases={a: 0 for a in range(len(sizes))})
    # closed form: static bytes of an arena = sum over its tensors of the region formula
    for a, ap in pl.arenas.items():
        want = 0
        for t in wl.tensors:
            if t.dst_arena != a:
                continue
            if t.is_static:
                want += -(-(-(-t.nbytes // 16) * 16 + 16) // align) * align
            else:
                want += -(-128 // align) * align
        assert ap.static_bytes == want
        assert ap.heap_offset == want and ap.heap_bytes == 1 << 20
    # a pure function of its input
    dev2 = O.Device()
    for n in sizes:
        dev2.arenas.append(O.Arena(np.zeros(0, dtype=np.uint8), O.RegionAllocator(n)))
    pl2 = O.plan(dev2, descs, align, 0, 1 << 20)
    assert [placement_dict(p) for p in pl.placements] == [placement_dict(p) for p in pl2.placements]


def test_vgg_round_robin_arena_loads():
    """Payload bytes per receiver arena for the 32 VGG-16-shaped tensors sent
    round-robin (W, b, W, b, ...) to 8 arenas; the figures are sums of the
    listed shapes."""
    wl = W.vgg16()
    loads = [0] * 8
    for t in wl.tensors:
        loads[t.dst_arena] += t.nbytes
    assert loads == [20060928, 5376, 422985728, 19712, 79200256, 19968, 31129600, 8608]
    assert sum(loads) == 553430176 and len(wl.tensors) == 32
    assert W.alexnet().payload_bytes == 249513376
    assert W.lstm().payload_bytes == 230948864


def test_table1_shaped_extra_sets():
    """FCN-5- and GRU-shaped sets reproduce the sizes the paper's Table 1 lists (in MiB)."""
    f, g = W.fcn5(), W.gru()
    assert len(f.tensors) == 10 and round(f.payload_bytes / 2 ** 20, 2) == 204.47
    assert round(g.payload_bytes / 2 ** 20, 2) == 27.92


def test_plan_random_mixed_sets():
    for seed in range(40):
        wl = W.small_mixed(seed, n=14, n_recv=3, n_dynamic=seed % 3)
        for align in (16, 64, 256):
            r = OracleRun(wl, align=align, heap=4096)
            sizes = {rid: s for rid, s in zip(r.recv_ids, r.recv_sizes)}
            I.check_plan([placement_dict(p) for p in r.plan.placements], sizes, align)


def test_plan_errors():
    dev = O.Device()
    dev.register_arena(np.zeros(1024, dtype=np.uint8))
    f32 = O.DTYPE_CODE["f32"]
    with pytest.raises(O.OracleError) as e:
        O.plan(dev, [O.TensorDesc(0, f32, (1000,), 0)], 256)        # 4000 B do not fit in 1024
    assert e.value.kind == "nomem"
    assert dev.arenas[0].alloc.free == [(0, 1024)]                    # nothing leaked
    with pytest.raises(O.OracleError) as e:
        O.plan(dev, [O.TensorDesc(0, f32, (1,), 0)], 24)
    assert e.value.kind == "align"
    with pytest.raises(O.OracleError) as e:
        O.plan(dev, [O.TensorDesc(0, f32, (1,), 0)], 8)
    assert e.value.kind == "align"
    with pytest.raises(O.OracleError) as e:
        O.plan(dev, [O.TensorDesc(0, f32, (1,), 3)], 256)
    assert e.value.kind == "inval"
    with pytest.raises(O.OracleError) as e:
        O.plan(dev, [O.TensorDesc(0, f32, (1,), 0), O.TensorDesc(0, f32, (1,), 0)], 256)
    assert e.value.kind == "inval"
    with pytest.raises(O.OracleError) as e:
        O.plan(dev, [O.TensorDesc(0, O.DTYPE_CODE["i64"], (1 << 31, 1 << 31), 0)], 256)
    assert e.value.kind == "overflow"


def test_allocator_first_fit_and_merge():
    a = O.RegionAllocator(4096)
    r0 = a.alloc(100, 256)
    r1 = a.alloc(300, 256)
    r2 = a.alloc(10, 16)
    assert (r0, r1) == (0, 256)
    assert r2 == 112            # first fit: the gap after r0, 16-aligned
    a.release(r1, 300)
    assert a.alloc(200, 64) == 128    # lowest address that fits with this alignment
    with pytest.raises(O.OracleError):
        a.release(5, 1)
    with pytest.raises(O.OracleError):
        a.alloc(0, 16)
    with pytest.raises(O.OracleError):
        a.alloc(16, 48)
    with pytest.raises(O.OracleError) as e:
        a.alloc(1 << 20, 16)
    assert e.value.kind == "nomem"


def test_allocator_random_against_bitmap_model():
    """Brute force: a byte bitmap of the arena gives the lowest aligned offset
    where `n` free bytes start; the allocator must return exactly that, and
    after any sequence of frees the free list must equal the bitmap's runs."""
    rng = np.random.Generator(np.random.PCG64(7))
    for trial in range(30):
        size = int(rng.integers(200, 1500))
        a = O.RegionAllocator(size)
        used = np.zeros(size, dtype=bool)
        live = []
        for step in range(60):
            if live and rng.random() < 0.4:
                off, n = live.pop(int(rng.integers(0, len(live))))
                a.release(off, n)
                used[off:off + n] = False
            else:
                n = int(rng.integers(1, 200))
                align = 1 << int(rng.integers(0, 7))
                want = None
                for off in range(0, size - n + 1, align):
                    if not used[off:off + n].any():
                        want = off
                        break
                if want is None:
                    with pytest.raises(O.OracleError):
                        a.alloc(n, align)
                else:
                    assert a.alloc(n, align) == want
                    used[want:want + n] = True
                    live.append((want, n))
            runs = []
            i = 0
            while i < size:
                if not used[i]:
                    j = i
                    while j < size and not used[j]:
                        j += 1
                    runs.append((i, j - i))
                    i = j
                else:
                    i += 1
            assert a.free == runs
