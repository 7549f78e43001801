"""GPU parity of the sparse-gradient producer (distinct ids ascending + their
rows) and its hand-over to the dynamic transfer path."""
import numpy as np
import pytest
import torch

from oracle import rdev_oracle as O
from paper_1805_08430_amd import rdev as R
from paper_1805_08430_amd import workloads as W
from helpers import OracleRun
from test_gpu_static import _compare_all
from test_gpu_dynamic import _meta_dict

pytestmark = pytest.mark.gpu


def _gather(dev, ids_np, table_np, stream=0):
    ids = torch.from_numpy(ids_np.reshape(-1).astype(np.int64)).to("cuda:0")
    table = torch.from_numpy(table_np).to("cuda:0")
    cap = max(1, min(ids.numel(), table_np.shape[0]))
    row_bytes = table_np.shape[1] * table_np.itemsize
    out_ids = torch.full((cap,), -7, dtype=torch.int64, device="cuda:0")
    out_rows = torch.zeros(cap * row_bytes, dtype=torch.uint8, device="cuda:0")
    count = torch.zeros(2, dtype=torch.int32, device="cuda:0")
    R.rdev_gather_unique_rows(dev, ids.data_ptr(), ids.numel(), table_np.shape[0], table.data_ptr(), row_bytes,
                              out_ids.data_ptr(), out_rows.data_ptr(), count.data_ptr(), stream)
    torch.cuda.synchronize()
    c = count.cpu().numpy()
    return int(c[0]), int(c[1]), out_ids.cpu().numpy(), out_rows.cpu().numpy()


def test_gather_equals_checker():
    dev = R.rdev_open(0)
    rng = np.random.Generator(np.random.PCG64(6))
    cases = [(W.lstm_token_ids(1), W.lstm_embedding_table(40000)[:, :1024])]
    for vocab, n, width in [(1, 5, 4), (33, 200, 8), (1000, 1, 12), (262144, 5000, 4), (4097, 4097, 4), (50, 0, 4)]:
        cases.append((rng.integers(0, vocab, size=n), rng.normal(size=(vocab, width)).astype(np.float32)))
    cases.append((np.full(300, 17), rng.normal(size=(64, 4)).astype(np.float32)))            # one id repeated
    cases.append((np.arange(999, -1, -1), rng.normal(size=(1000, 4)).astype(np.float32)))     # every id, descending
    for ids, table in cases:
        cnt, bad, got_ids, got_rows = _gather(dev, np.asarray(ids), table)
        want_ids, want_rows = O.gather_unique_rows(np.asarray(ids, dtype=np.int64), table) if np.asarray(ids).size else \
            (np.zeros(0, np.int64), table[:0])
        assert (cnt, bad) == (want_ids.size, 0)
        assert np.array_equal(got_ids[:cnt], want_ids)
        assert np.array_equal(got_rows[:cnt * table.shape[1] * 4], np.ascontiguousarray(want_rows).view(np.uint8).reshape(-1))
        assert (got_ids[cnt:] == -7).all() and (got_rows[cnt * table.shape[1] * 4:] == 0).all()   # nothing beyond
    # ids outside the vocabulary are counted and ignored
    ids = np.array([3, -1, 70, 5, 3, 1 << 40])
    table = rng.normal(size=(64, 4)).astype(np.float32)
    cnt, bad, got_ids, _ = _gather(dev, ids, table)
    assert (cnt, bad, got_ids[:2].tolist()) == (2, 3, [3, 5])
    with pytest.raises(R.RdevError):
        R.rdev_gather_unique_rows(dev, 256, 1, 1 << 20, 256, 16, 256, 256, 256)
    R.rdev_close(dev)


def test_lstm_sparse_gradient_end_to_end_on_gpu():
    """ids -> (device) distinct ids + rows, produced straight into the registered
    sender arena -> dynamic transfer; the checker does the same with numpy."""
    from gpu_harness import GpuRun
    wl = W.lstm()
    table_np = W.lstm_embedding_table()
    heap = 8 << 20
    g = GpuRun(wl, heap=heap, extra_arenas=(16 << 20,))
    o = OracleRun(wl, heap=heap, extra_arenas=(16 << 20,))
    table = torch.from_numpy(table_np).to("cuda:0")
    count = torch.zeros(2, dtype=torch.int32, device="cuda:0")
    src_t, src_id = g.extra_t[0], o.extra_ids[0]
    ids_off, rows_off = 4096, 65536
    for it in range(1, 3):
        ids_np = W.lstm_token_ids(it)
        ids = torch.from_numpy(ids_np.reshape(-1)).to("cuda:0")
        R.rdev_gather_unique_rows(g.dev, ids.data_ptr(), ids.numel(), W.LSTM_VOCAB, table.data_ptr(), 4096,
                                  src_t.data_ptr() + ids_off, src_t.data_ptr() + rows_off, count.data_ptr(), g.s)
        g.stream.synchronize()
        u = int(count.cpu()[0])
        want_ids, want_rows = O.gather_unique_rows(ids_np, table_np)
        assert u == want_ids.size
        o.image(src_id)[ids_off:ids_off + 8 * u] = want_ids.view(np.uint8)
        o.image(src_id)[rows_off:rows_off + 4096 * u] = np.ascontiguousarray(want_rows).view(np.uint8).reshape(-1)
        _compare_all(g, o, "gathered into the sender arena")
        R.rdev_dyn_reset(g.plan)
        O.dyn_reset(o.plan)
        R.rdev_write_batch(g.dev, g.plan, [R.make_xfer(3, src_t.data_ptr() + ids_off, R.I64, (u,)),
                                           R.make_xfer(4, src_t.data_ptr() + rows_off, R.F32, (u, 1024))],
                           R.ZEROCOPY, it, g.s)
        O.dyn_send(o.dev, o.plan, 3, (src_id, ids_off), O.DTYPE_CODE["i64"], (u,), it)
        O.dyn_send(o.dev, o.plan, 4, (src_id, rows_off), O.DTYPE_CODE["f32"], (u, 1024), it)
        for t in (3, 4):
            ok, m = g.wait(t, R.POLL_META | R.POLL_CONSUME, want_meta=True)
            assert _meta_dict(m) == O.poll(o.dev, o.plan, t, consume=True, which=O.POLL_META)[1]
        R.rdev_read_batch(g.dev, g.plan, [R.make_xfer(3), R.make_xfer(4)], it, g.s)
        for t in (3, 4):
            O.dyn_recv(o.dev, o.plan, t, it)
            g.wait(t, R.POLL_CONSUME)
            assert O.poll(o.dev, o.plan, t, consume=True, which=O.POLL_DATA)[0]
        _compare_all(g, o, f"iteration {it}")
    # the same without the host ever learning the count before it sends: the metadata kernel reads it on the device
    for it in range(3, 6):
        ids_np = W.lstm_token_ids(it)
        ids = torch.from_numpy(ids_np.reshape(-1)).to("cuda:0")
        want_ids, want_rows = O.gather_unique_rows(ids_np, table_np)
        u = want_ids.size
        bound = ids.numel() if it != 5 else u - 10                    # round 5: a bound below the count cuts it
        sent = min(u, bound)
        R.rdev_dyn_reset(g.plan)
        O.dyn_reset(o.plan)
        R.rdev_gather_unique_rows(g.dev, ids.data_ptr(), ids.numel(), W.LSTM_VOCAB, table.data_ptr(), 4096,
                                  src_t.data_ptr() + ids_off, src_t.data_ptr() + rows_off, count.data_ptr(), g.s)
        R.rdev_write_batch(g.dev, g.plan,
                           [R.make_xfer(3, src_t.data_ptr() + ids_off, R.I64, (bound,), count.data_ptr()),
                            R.make_xfer(4, src_t.data_ptr() + rows_off, R.F32, (bound, 1024), count.data_ptr())],
                           R.ZEROCOPY, it, g.s)
        o.image(src_id)[ids_off:ids_off + 8 * u] = want_ids.view(np.uint8)
        o.image(src_id)[rows_off:rows_off + 4096 * u] = np.ascontiguousarray(want_rows).view(np.uint8).reshape(-1)
        O.dyn_send(o.dev, o.plan, 3, (src_id, ids_off), O.DTYPE_CODE["i64"], (sent,), it)
        O.dyn_send(o.dev, o.plan, 4, (src_id, rows_off), O.DTYPE_CODE["f32"], (sent, 1024), it)
        for t in (3, 4):
            ok, m = g.wait(t, R.POLL_META | R.POLL_CONSUME, want_meta=True)
            assert _meta_dict(m) == O.poll(o.dev, o.plan, t, consume=True, which=O.POLL_META)[1]
            assert m.dims[0] == sent
        R.rdev_read_batch(g.dev, g.plan, [R.make_xfer(3), R.make_xfer(4)], it, g.s)
        for t in (3, 4):
            O.dyn_recv(o.dev, o.plan, t, it)
            g.wait(t, R.POLL_CONSUME)
            assert O.poll(o.dev, o.plan, t, consume=True, which=O.POLL_DATA)[0]
        _compare_all(g, o, f"device-sized iteration {it}")
    g.close()
