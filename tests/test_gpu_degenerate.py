"""GPU parity on degenerate inputs: empty plans, plans of only empty tensors,
rank-8 and 2-byte-element dynamic tensors, many tiny tensors in one launch."""
import numpy as np
import pytest
import torch

from oracle import rdev_oracle as O
from paper_1805_08430_amd import rdev as R
from paper_1805_08430_amd import workloads as W
from helpers import OracleRun
from test_gpu_static import _compare_all, _run_static

pytestmark = pytest.mark.gpu


def _wl(name, tensors, sender_bytes):
    return W.Workload(name, 990 + len(tensors), tensors, 1, 1, [sender_bytes], "bits")


def test_empty_plan():
    from gpu_harness import GpuRun
    wl = _wl("empty", [], 512)
    g, o = GpuRun(wl), OracleRun(wl)
    R.rdev_write_batch(g.dev, g.plan, None, R.ZEROCOPY, 1, g.s)          # nothing to move, nothing to flag
    g.stream.synchronize()
    assert R.rdev_poll(g.dev, g.plan, R.ALL_TENSORS, R.POLL_CONSUME, g.s)  # vacuously ready
    assert R.rdev_plan_count(g.plan) == 0
    _compare_all(g, o, "empty plan")
    g.close()


def test_only_empty_and_scalar_tensors():
    tensors = [W.TensorSpec("z0", "f32", (0,), 0, 0, 0), W.TensorSpec("z1", "f64", (4, 0, 3), 0, 0, 0),
               W.TensorSpec("s0", "i8", (), 0, 0, 5), W.TensorSpec("s1", "f64", (), 0, 0, 9),
               W.TensorSpec("z2", "u8", (0,), 0, 0, 300)]
    _run_static(_wl("degenerate", tensors, 512), iters=2)


def test_many_tiny_tensors_one_launch():
    rng = np.random.Generator(np.random.PCG64(3))
    tensors, off = [], 0
    for i in range(3000):
        n = int(rng.integers(0, 300))
        tensors.append(W.TensorSpec(f"t{i}", "u8", (n,), 0, 0, off))
        off += n + int(rng.integers(0, 7))
    _run_static(_wl("tiny3000", tensors, off + 512), iters=1)


def test_dynamic_rank8_and_two_byte_types():
    from gpu_harness import GpuRun
    tensors = [W.TensorSpec("a", "bf16", (-1, 2, 1, 3, 1, 2, 1, 2), 0, 0), W.TensorSpec("b", "f16", (3, -1), 0, 0),
               W.TensorSpec("c", "u8", (-1,), 0, 0), W.TensorSpec("d", "i16", (-1, -1), 0, 0)]
    wl = _wl("dyn_only", tensors, 512)
    g = GpuRun(wl, heap=1 << 16, extra_arenas=(1 << 16,))
    o = OracleRun(wl, heap=1 << 16, extra_arenas=(1 << 16,))
    src_t, src_id = g.extra_t[0], o.extra_ids[0]
    for it, shapes in enumerate([[(5, 2, 1, 3, 1, 2, 1, 2), (3, 7), (0,), (2, 9)],
                                 [(1, 2, 1, 3, 1, 2, 1, 2), (3, 0), (4099,), (0, 0)]], start=1):
        R.rdev_dyn_reset(g.plan)
        O.dyn_reset(o.plan)
        off, xs = 0, []
        for t, (spec, dims) in enumerate(zip(tensors, shapes)):
            nb = W.itemsize(spec.dtype) * int(np.prod(dims))
            payload = W.dynamic_payload(nb, 31 * it + t)
            off = O.round_up(off, 16) + 2                               # 2-byte aligned sources
            src_t[off:off + nb].copy_(torch.from_numpy(payload))
            o.image(src_id)[off:off + nb] = payload
            xs.append((t, spec.dtype, dims, off))
            off += nb
        torch.cuda.synchronize()
        R.rdev_write_batch(g.dev, g.plan, [R.make_xfer(t, src_t.data_ptr() + so, R.DTYPE[dt], dims)
                                           for t, dt, dims, so in xs], R.ZEROCOPY, it, g.s)
        for t, dt, dims, so in xs:
            O.dyn_send(o.dev, o.plan, t, (src_id, so), O.DTYPE_CODE[dt], dims, it)
        for t, *_ in xs:
            g.wait(t, R.POLL_META | R.POLL_CONSUME)
            assert O.poll(o.dev, o.plan, t, True, O.POLL_META)[0]
        R.rdev_read_batch(g.dev, g.plan, [R.make_xfer(t) for t, *_ in xs], it, g.s)
        for t, *_ in xs:
            O.dyn_recv(o.dev, o.plan, t, it)
        for t, *_ in xs:
            ok, m = g.wait(t, R.POLL_CONSUME, want_meta=True)
            ok2, m2 = O.poll(o.dev, o.plan, t, consume=True, which=O.POLL_DATA)
            assert ok2 and tuple(m.dims) == m2["dims"] and m.bytes == m2["nbytes"] and m.dst_offset == m2["dst_offset"]
        _compare_all(g, o, f"round {it}")
    # whole-plan calls on a plan without static tensors are no-ops
    R.rdev_write_batch(g.dev, g.plan, None, R.ZEROCOPY, 9, g.s)
    assert R.rdev_poll(g.dev, g.plan, R.ALL_TENSORS)
    _compare_all(g, o, "no static tensors")
    g.close()
