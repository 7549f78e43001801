"""Sender-side allocation-site tracing (paper section 3.4): pins for the CPU
checker's tracer, the library's host logic against it (CPU), and GPU parity of
a traced mini-batch loop."""
import numpy as np
import pytest

from oracle import rdev_oracle as O
from paper_1805_08430_amd import rdev as R
from paper_1805_08430_amd import workloads as W

POOL_BASE = 0x7100_0000_0000
ARENA_BASE = 0x7200_0000_0000
RECV_BASE = 0x7300_0000_0000


def _oracle_setup(pool_bytes=1 << 16, arena_bytes=1 << 16, sizes=(1000, 2000)):
    dev = O.Device()
    a = dev.register_arena(np.zeros(arena_bytes, dtype=np.uint8))
    r = dev.register_arena(np.zeros(1 << 16, dtype=np.uint8))
    pl = O.plan(dev, [O.TensorDesc(i, 0, (n,), r) for i, n in enumerate(sizes)])
    tr = O.Tracer(dev, np.zeros(pool_bytes, dtype=np.uint8), a)
    return dev, pl, tr, a, r


def test_paper_scenario_by_hand():
    """GenGrad (node 1) allocates a temporary, then the gradient; an in-place
    node (2) passes the gradient through; node 3 sends it.  The sent buffer's
    allocation site is (node 1, second allocation): S = {(1, 1)}.  In the next
    mini-batch exactly that allocation comes from the registered arena."""
    dev, pl, tr, a, r = _oracle_setup()
    tr.begin_iteration()
    w_t, o_t, i_t = tr.alloc(1, 512)
    w_g, o_g, i_g = tr.alloc(1, 1000)
    assert (w_t, i_t, w_g, i_g) == ("pool", 0, "pool", 1)
    tr.free(w_t, o_t)
    tr.buffer(w_g, o_g, 1000)[:] = np.arange(1000) % 251
    assert tr.send(pl, 0, w_g, o_g, 1) is True                     # staged: the buffer is not registered
    assert tr.S == [(1, 1)]
    assert len(tr.staging) == 1
    p = pl.get(0)
    assert (dev.arenas[r].mem[p.data_offset:p.data_offset + 1000] == np.arange(1000) % 251).all()
    tr.begin_iteration()
    assert dev.arenas[a].alloc.used == {}                           # staging released
    assert tr.alloc(1, 512)[0] == "pool"
    w_g, o_g, i_g = tr.alloc(1, 1000)
    assert (w_g, i_g) == ("arena", 1)
    tr.buffer(w_g, o_g, 1000)[:] = 7
    O.poll(dev, pl, 0, consume=True)
    assert tr.send(pl, 0, w_g, o_g, 2) is False                    # zero-copy now
    assert tr.staging == [] and tr.S == [(1, 1)]
    assert (dev.arenas[r].mem[p.data_offset:p.data_offset + 1000] == 7).all()


def test_address_reuse_last_writer_wins_and_tracing_only_first_iteration():
    dev, pl, tr, a, r = _oracle_setup()
    tr.begin_iteration()
    w4, o4, _ = tr.alloc(4, 2000)
    tr.free(w4, o4)
    w5, o5, _ = tr.alloc(5, 2000)
    assert (w5, o5) == (w4, o4)                                     # same address handed out again
    tr.send(pl, 1, w5, o5, 1)
    assert tr.S == [(5, 0)]                                         # not (4, 0)
    tr.begin_iteration()
    assert tr.alloc(4, 2000)[0] == "pool" and tr.alloc(5, 2000)[0] == "arena"
    w9, o9, _ = tr.alloc(9, 1000)
    O.poll(dev, pl, 0, consume=True)
    assert tr.send(pl, 0, w9, o9, 2) is True                        # never seen in the tracing iteration: copied
    assert tr.S == [(5, 0)]                                         # and S no longer grows
    tr.begin_iteration()
    assert tr.alloc(9, 1000)[0] == "pool"


def _fake_dev():
    dev = R.rdev_open(R.HOST_ONLY)
    a = R.rdev_register_arena(dev, ARENA_BASE, 1 << 20)
    return dev, a


def test_library_tracer_host_logic_equals_checker_random():
    rng = np.random.Generator(np.random.PCG64(17))
    for trial in range(20):
        dev, a = _fake_dev()
        tr = R.rdev_tracer_open(dev, POOL_BASE, 1 << 20, a)
        odev = O.Device()
        oa = odev.register_arena(np.zeros(1 << 20, dtype=np.uint8))
        otr = O.Tracer(odev, np.zeros(1 << 20, dtype=np.uint8), oa)
        for it in range(3):
            R.rdev_tracer_begin_iteration(tr)
            otr.begin_iteration()
            live = []
            for step in range(60):
                op = rng.random()
                if op < 0.55 or not live:
                    node, nb = int(rng.integers(0, 6)), int(rng.integers(1, 5000))
                    ptr, idx, in_arena = R.rdev_tracer_alloc(tr, node, nb)
                    w, off, oidx = otr.alloc(node, nb)
                    assert (idx, in_arena) == (oidx, w == "arena")
                    assert ptr == (ARENA_BASE if in_arena else POOL_BASE) + off
                    live.append((ptr, w, off))
                elif op < 0.8:
                    ptr, w, off = live.pop(int(rng.integers(0, len(live))))
                    R.rdev_tracer_free(tr, ptr)
                    otr.free(w, off)
                else:
                    ptr, w, off = live[int(rng.integers(0, len(live)))]
                    assert R.rdev_tracer_mark_sent(tr, ptr) == (w == "arena")
                    if otr.iteration == 1:
                        site = otr.site_of.get((w, off))
                        if site is not None and site not in otr.S:
                            otr.S.append(site)
            assert R.rdev_tracer_set(tr) == otr.S
        R.rdev_tracer_close(tr)
        R.rdev_close(dev)


def test_library_tracer_errors():
    dev, a = _fake_dev()
    with pytest.raises(R.RdevError) as e:
        R.rdev_tracer_open(dev, ARENA_BASE + 4096, 4096, a)        # the pool must not be registered memory
    assert e.value.status == R.E_OVERLAP
    with pytest.raises(R.RdevError) as e:
        R.rdev_tracer_open(dev, POOL_BASE, 4096, 9)
    assert e.value.status == R.E_INVAL
    tr = R.rdev_tracer_open(dev, POOL_BASE, 4096, a)
    with pytest.raises(R.RdevError) as e:
        R.rdev_tracer_alloc(tr, 0, 16)                             # no iteration begun
    assert e.value.status == R.E_STATE
    R.rdev_tracer_begin_iteration(tr)
    with pytest.raises(R.RdevError) as e:
        R.rdev_tracer_alloc(tr, 0, 8192)
    assert e.value.status == R.E_NOMEM
    with pytest.raises(R.RdevError) as e:
        R.rdev_tracer_free(tr, POOL_BASE + 64)
    assert e.value.status == R.E_INVAL
    p, _, _ = R.rdev_tracer_alloc(tr, 0, 100)
    R.rdev_tracer_close(tr)                                         # releases what is still held
    R.rdev_close(dev)


@pytest.mark.gpu
def test_traced_minibatch_loop_on_gpu():
    """A small sender graph run for three mini-batches through the library's
    tracer and through the checker's: same decisions, same S, and the same
    bytes in the registered arena (staging included) and the receiver arena."""
    import torch
    wl = W.small_mixed(44, n=10, max_bytes=40000, n_recv=1, dtypes=("f32",), gran=256)
    sizes = [max(t.nbytes, 4) for t in wl.tensors]
    dev = R.rdev_open(0)
    arena_t = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    recv_t = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    pool_t = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    a = R.rdev_register_arena(dev, arena_t.data_ptr(), arena_t.numel())
    r = R.rdev_register_arena(dev, recv_t.data_ptr(), recv_t.numel())
    plan = R.rdev_plan(dev, [R.make_desc(i, R.U8, (n,), r) for i, n in enumerate(sizes)])
    tr = R.rdev_tracer_open(dev, pool_t.data_ptr(), pool_t.numel(), a)
    odev = O.Device()
    oa = odev.register_arena(np.zeros(1 << 20, dtype=np.uint8))
    orr = odev.register_arena(np.zeros(1 << 20, dtype=np.uint8))
    opl = O.plan(odev, [O.TensorDesc(i, 0, (n,), orr) for i, n in enumerate(sizes)])
    otr = O.Tracer(odev, np.zeros(1 << 20, dtype=np.uint8), oa)
    stream = torch.cuda.Stream()
    copies = []
    for it in range(1, 4):
        torch.cuda.synchronize()
        R.rdev_tracer_begin_iteration(tr)
        otr.begin_iteration()
        for i, n in enumerate(sizes):
            node = 100 + i
            tptr, _, _ = R.rdev_tracer_alloc(tr, node, 777)                  # a temporary
            tw, toff, _ = otr.alloc(node, 777)
            gptr, gidx, g_in = R.rdev_tracer_alloc(tr, node, n)              # the gradient
            gw, goff, oidx = otr.alloc(node, n)
            assert (gidx, g_in) == (oidx, gw == "arena")
            if i % 3 == 0:                                                   # some temporaries die early
                R.rdev_tracer_free(tr, tptr)
                otr.free(tw, toff)
            data = W.dynamic_payload(n, 1000 * it + i)
            base_t = arena_t if g_in else pool_t
            off = gptr - base_t.data_ptr()
            assert off == goff
            base_t[off:off + n].copy_(torch.from_numpy(data))
            otr.buffer(gw, goff, n)[:] = data
            torch.cuda.synchronize()
            if i == 7 and it > 1:
                continue                                                     # this one is not sent every time
            copied = R.rdev_tracer_send(tr, plan, i, gptr, it, stream.cuda_stream)
            assert copied == otr.send(opl, i, gw, goff, it)
            copies.append((it, i, copied))
        stream.synchronize()
        assert R.rdev_tracer_set(tr) == otr.S
        assert np.array_equal(arena_t.cpu().numpy(), odev.arenas[oa].mem)
        assert np.array_equal(recv_t.cpu().numpy(), odev.arenas[orr].mem)
        for i in range(len(sizes)):
            if R.rdev_poll(dev, plan, i):
                assert R.rdev_poll(dev, plan, i, R.POLL_CONSUME, stream.cuda_stream)
                assert O.poll(odev, opl, i, consume=True)[0]
    assert all(c for it, i, c in copies if it == 1)              # tracing iteration: everything staged
    assert not any(c for it, i, c in copies if it > 1)           # afterwards: nothing
    torch.cuda.synchronize()
    R.rdev_tracer_close(tr)
    R.rdev_plan_free(plan)
    R.rdev_close(dev)
