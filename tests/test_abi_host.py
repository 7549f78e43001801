"""CPU-only checks of the C-ABI library: it loads, exports every declared
symbol, and its host logic (sub-allocator, classifier, planner, error paths)
agrees with the CPU checker.  No byte is moved here: a host-only device refuses
transfers."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import rdev_oracle as O
from paper_1805_08430_amd import rdev as R
from paper_1805_08430_amd import workloads as W
import invariants as I
from helpers import placement_dict, receiver_bytes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def lib_placement_dict(p):
    return dict(tensor_id=p.tensor_id, kind=p.kind, dst_arena=p.dst_arena, data_offset=p.data_offset,
                nbytes=p.bytes, flag_offset=p.flag_offset, meta_offset=p.meta_offset, region_bytes=p.region_bytes)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "rdev.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(rdev_[a-z_0-9]+)\s*\(", hdr))
    assert {"rdev_alloc_region", "rdev_plan", "rdev_write_batch", "rdev_read_batch", "rdev_poll"} <= declared
    l = ctypes.CDLL(R.LIB_PATH)
    for name in declared:
        assert hasattr(l, name), name
    assert declared == set(R.SYMBOLS), declared ^ set(R.SYMBOLS)
    R.lib()      # also checks the struct sizes against the library's


def _fake_base(i):
    return 0x7000_0000_0000 + i * (1 << 40)


def _open_with_arenas(sizes):
    dev = R.rdev_open(R.HOST_ONLY)
    ids = [R.rdev_register_arena(dev, _fake_base(i), n) for i, n in enumerate(sizes)]
    return dev, ids


@pytest.mark.parametrize("name", ["tiny", "alexnet", "vgg16", "lstm", "inception"])
@pytest.mark.parametrize("align,heap,max_static", [(256, 0, 0), (4096, 1 << 20, 0), (64, 4096, 1 << 20)])
def test_planner_equals_checker_on_the_five_configs(name, align, heap, max_static):
    wl = W.CONFIGS[name]()
    sizes = receiver_bytes(wl, align, heap)
    dev, ids = _open_with_arenas(sizes)
    odev = O.Device()
    for n in sizes:
        odev.arenas.append(O.Arena(np.zeros(0, dtype=np.uint8), O.RegionAllocator(n)))
    descs = [R.make_desc(i, R.DTYPE[t.dtype], t.dims, ids[t.dst_arena]) for i, t in enumerate(wl.tensors)]
    odescs = [O.TensorDesc(i, O.DTYPE_CODE[t.dtype], tuple(t.dims), t.dst_arena) for i, t in enumerate(wl.tensors)]
    plan = R.rdev_plan(dev, descs, align=align, dyn_heap_bytes=heap, max_static_bytes=max_static)
    opl = O.plan(odev, odescs, align, max_static, heap)
    got = [lib_placement_dict(p) for p in R.placements(plan)]
    assert got == [placement_dict(p) for p in opl.placements]
    I.check_plan(got, dict(zip(ids, sizes)), align)
    for a, ap in opl.arenas.items():
        info = R.rdev_plan_arena_info(plan, a)
        assert info == dict(base=ap.base, static_bytes=ap.static_bytes, heap_offset=ap.heap_offset,
                            heap_bytes=ap.heap_bytes)
    R.rdev_plan_free(plan)
    R.rdev_close(dev)


def test_planner_equals_checker_random_sets_with_busy_arenas():
    """Arenas that already hold regions: the plan's block goes to the first fit."""
    rng = np.random.Generator(np.random.PCG64(5))
    for seed in range(25):
        wl = W.small_mixed(100 + seed, n=12, n_recv=3, n_dynamic=seed % 3)
        sizes = [s + 8192 for s in receiver_bytes(wl, 256, 2048)]
        dev, ids = _open_with_arenas(sizes)
        odev = O.Device()
        for n in sizes:
            odev.arenas.append(O.Arena(np.zeros(0, dtype=np.uint8), O.RegionAllocator(n)))
        for a in range(3):        # pre-existing regions, some freed again
            held = []
            for _ in range(4):
                nb, al = int(rng.integers(1, 900)), 1 << int(rng.integers(0, 9))
                r = R.rdev_alloc_region(dev, ids[a], nb, al)
                assert (r.arena_id, r.offset, r.bytes) == odev.alloc_region(a, nb, al)
                held.append(r)
            for r in held[::2]:
                R.rdev_free_region(dev, r)
                odev.free_region((a, r.offset, r.bytes))
        descs = [R.make_desc(i, R.DTYPE[t.dtype], t.dims, ids[t.dst_arena]) for i, t in enumerate(wl.tensors)]
        odescs = [O.TensorDesc(i, O.DTYPE_CODE[t.dtype], tuple(t.dims), t.dst_arena) for i, t in enumerate(wl.tensors)]
        plan = R.rdev_plan(dev, descs, align=256, dyn_heap_bytes=2048)
        opl = O.plan(odev, odescs, 256, 0, 2048)
        assert [lib_placement_dict(p) for p in R.placements(plan)] == [placement_dict(p) for p in opl.placements]
        # freeing the plan returns its blocks: the same request fits again at the same place
        R.rdev_plan_free(plan)
        plan2 = R.rdev_plan(dev, descs, align=256, dyn_heap_bytes=2048)
        assert [lib_placement_dict(p) for p in R.placements(plan2)] == [placement_dict(p) for p in opl.placements]
        R.rdev_plan_free(plan2)
        R.rdev_close(dev)


def test_allocator_random_equals_checker():
    rng = np.random.Generator(np.random.PCG64(8))
    for trial in range(20):
        size = int(rng.integers(500, 5000))
        dev, ids = _open_with_arenas([size])
        oa = O.RegionAllocator(size)
        live = []
        for _ in range(80):
            if live and rng.random() < 0.45:
                r = live.pop(int(rng.integers(0, len(live))))
                R.rdev_free_region(dev, r)
                oa.release(r.offset, r.bytes)
            else:
                nb, al = int(rng.integers(1, 600)), 1 << int(rng.integers(0, 8))
                try:
                    want = oa.alloc(nb, al)
                except O.OracleError as e:
                    with pytest.raises(R.RdevError) as ge:
                        R.rdev_alloc_region(dev, ids[0], nb, al)
                    assert ge.value.status == R.E_NOMEM and e.kind == "nomem"
                    continue
                r = R.rdev_alloc_region(dev, ids[0], nb, al)
                assert r.offset == want and r.bytes == nb
                live.append(r)
        R.rdev_close(dev)


def _status(fn, *a, **k):
    with pytest.raises(R.RdevError) as e:
        fn(*a, **k)
    assert R.rdev_last_error()
    return e.value.status


def test_error_paths():
    dev, ids = _open_with_arenas([4096, 4096])
    f32 = R.F32
    assert _status(R.rdev_register_arena, dev, _fake_base(0) + 256, 1024) == R.E_OVERLAP
    assert _status(R.rdev_register_arena, dev, _fake_base(9) + 8, 1024) == R.E_ALIGN
    assert _status(R.rdev_register_arena, dev, _fake_base(9), 0) == R.E_INVAL
    assert _status(R.rdev_alloc_region, dev, 7, 16, 16) == R.E_INVAL
    assert _status(R.rdev_alloc_region, dev, ids[0], 16, 24) == R.E_ALIGN
    assert _status(R.rdev_alloc_region, dev, ids[0], 0, 16) == R.E_INVAL
    assert _status(R.rdev_alloc_region, dev, ids[0], 8192, 16) == R.E_NOMEM
    bogus = R.Region(ids[0], 0, 64, 64)
    assert _status(R.rdev_free_region, dev, bogus) == R.E_INVAL
    assert _status(R.rdev_plan, dev, [R.make_desc(0, f32, (2000,), ids[0])]) == R.E_NOMEM
    # nothing stays allocated after a failed plan: the whole arena is still free
    r = R.rdev_alloc_region(dev, ids[0], 4096, 256)
    R.rdev_free_region(dev, r)
    two = [R.make_desc(0, f32, (100,), ids[0]), R.make_desc(1, f32, (2000,), ids[1])]
    assert _status(R.rdev_plan, dev, two) == R.E_NOMEM            # arena 1 fails after arena 0 succeeded
    r = R.rdev_alloc_region(dev, ids[0], 4096, 256)
    R.rdev_free_region(dev, r)
    assert _status(R.rdev_plan, dev, [R.make_desc(0, f32, (1,), ids[0])], align=24) == R.E_ALIGN
    assert _status(R.rdev_plan, dev, [R.make_desc(0, f32, (1,), ids[0])], align=8) == R.E_ALIGN
    assert _status(R.rdev_plan, dev, [R.make_desc(0, f32, (1,), 5)]) == R.E_INVAL
    assert _status(R.rdev_plan, dev, [R.make_desc(0, 42, (1,), ids[0])]) == R.E_INVAL
    assert _status(R.rdev_plan, dev, [R.make_desc(0, f32, (-2,), ids[0])]) == R.E_INVAL
    assert _status(R.rdev_plan, dev, [R.make_desc(0, f32, (1,), ids[0]), R.make_desc(0, f32, (1,), ids[0])]) == R.E_INVAL
    assert _status(R.rdev_plan, dev, [R.make_desc(0, R.I64, (1 << 31, 1 << 31), ids[0])]) == R.E_OVERFLOW
    d9 = R.make_desc(0, f32, (1,) * 8, ids[0])
    d9.ndims = 9
    assert _status(R.rdev_plan, dev, [d9]) == R.E_INVAL
    assert _status(R.rdev_plan, dev, [R.make_desc(0, f32, (1,), ids[0])], chunk_bytes=1000) == R.E_INVAL
    assert _status(R.rdev_plan, dev, [R.make_desc(0, f32, (1,), ids[0])], rpc_frag_bytes=100) == R.E_INVAL
    assert _status(R.rdev_plan, dev, [R.make_desc(0, f32, (1,), ids[0])], flag_groups=5000) == R.E_INVAL
    # zero-size and scalar tensors are legal
    plan = R.rdev_plan(dev, [R.make_desc(0, f32, (), ids[0]), R.make_desc(1, f32, (4, 0), ids[0]),
                             R.make_desc(2, R.U8, (1 << 40, 0, 1 << 40), ids[0])])
    pl = R.placements(plan)
    assert [p.bytes for p in pl] == [4, 0, 0] and [p.region_bytes for p in pl] == [256, 256, 256]
    # a host-only device cannot transfer
    assert _status(R.rdev_write_batch, dev, plan) == R.E_HIP
    assert _status(R.rdev_poll, dev, plan, 0) == R.E_HIP
    assert _status(R.rdev_close, dev) == R.E_BUSY          # plan still alive
    # bind: a source must lie in a registered arena and must not overlap its destination
    assert _status(R.rdev_plan_bind_sources, plan, [0x1000, None, None]) == R.E_RANGE
    assert _status(R.rdev_plan_bind_sources, plan, [_fake_base(0) + pl[0].data_offset + 2, None, None]) == R.E_OVERLAP
    assert _status(R.rdev_plan_bind_sources, plan, [None]) == R.E_INVAL
    R.rdev_plan_bind_sources(plan, [_fake_base(1), _fake_base(1) + 8, _fake_base(1) + 4096])
    assert _status(R.rdev_unregister_arena, dev, ids[0]) == R.E_BUSY     # the plan's block lives there
    R.rdev_plan_free(plan)
    R.rdev_unregister_arena(dev, ids[0])
    assert _status(R.rdev_alloc_region, dev, ids[0], 16, 16) == R.E_INVAL
    assert _status(R.rdev_unregister_arena, dev, ids[0]) == R.E_INVAL
    assert R.rdev_register_arena(dev, _fake_base(0), 4096) == 2          # same memory again, new id
    R.rdev_close(dev)


def test_header_is_plain_c_and_usable_from_c(tmp_path):
    """include/rdev.h compiles as C99 with gcc, and a C program linked against the
    library reproduces the hand-computed placement."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    exe = str(tmp_path / "c_abi_check")
    libdir = os.path.dirname(R.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_abi_check.c"), "-o", exe, "-L", libdir, "-lrdev",
                    "-Wl,-rpath," + libdir], check=True, capture_output=True, text=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0 and "c abi ok" in r.stdout, r.stdout + r.stderr


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(R, "_lib", None)
    monkeypatch.setattr(R, "LIB_PATH", "/nonexistent/librdev.so")
    with pytest.raises(R.RdevError):
        R.rdev_open(R.HOST_ONLY)
