"""Pins for the checker's byte movers, flags, metadata and copy baselines (CPU only)."""
import os
import struct

import numpy as np
import pytest

from oracle import rdev_oracle as O
from paper_1805_08430_amd import workloads as W
import invariants as I
from helpers import GOLDEN, OracleRun, placement_dict


def _le32(v):
    return [v & 255, (v >> 8) & 255, (v >> 16) & 255, (v >> 24) & 255]


def test_exhaustive_tiny_static_against_byte_loops():
    """sizes 0..67 B x source misalignment 0..15 x 1..3 tensors; the expected
    arena image is built one byte at a time."""
    rng = np.random.Generator(np.random.PCG64(11))
    u8 = O.DTYPE_CODE["u8"]
    for ntens in (1, 2, 3):
        for size in range(0, 68):
            for mis in range(16):
                if ntens > 1 and (size * 16 + mis) % 5:      # thin out the larger products
                    continue
                dev = O.Device()
                src = rng.integers(0, 256, size=1024, dtype=np.uint8)
                s_id = dev.register_arena(src.copy())
                poison = W.poison(2048, size * 16 + mis)
                r_id = dev.register_arena(poison.copy())
                sizes = [size] + [int(x) for x in rng.integers(0, 68, size=ntens - 1)]
                descs = [O.TensorDesc(i, u8, (n,), r_id) for i, n in enumerate(sizes)]
                pl = O.plan(dev, descs, 16)
                sources, off = {}, 64 + mis
                for i, n in enumerate(sizes):
                    sources[i] = (s_id, off)
                    off += n + 3
                O.static_write(dev, pl, sources, 7)
                want = [int(b) for b in poison]
                for i, n in enumerate(sizes):
                    p = pl.get(i)
                    for k in range(n):
                        want[p.data_offset + k] = int(src[sources[i][1] + k])
                    want[p.flag_offset:p.flag_offset + 4] = _le32(7)
                assert dev.arenas[r_id].mem.tolist() == want
                assert (dev.arenas[s_id].mem == src).all()


def test_single_aligned_tensor_is_a_slice_assignment():
    n = 1 << 20
    rng = np.random.Generator(np.random.PCG64(3))
    src = rng.integers(0, 256, size=n, dtype=np.uint8)
    dev = O.Device()
    s = dev.register_arena(src.copy())
    r = dev.register_arena(np.zeros(n + 512, dtype=np.uint8))
    pl = O.plan(dev, [O.TensorDesc(0, O.DTYPE_CODE["f32"], (n // 4,), r)], 256)
    O.static_write(dev, pl, {0: (s, 0)}, 1)
    want = np.zeros(n + 512, dtype=np.uint8)
    want[0:n] = src
    want[n:n + 4] = _le32(1)
    assert (dev.arenas[r].mem == want).all()


@pytest.mark.parametrize("seed", range(6))
def test_static_write_invariants_mixed(seed):
    wl = W.small_mixed(seed, n=16, n_recv=3, gran=1)
    r = OracleRun(wl)
    O.static_write(r.dev, r.plan, r.sources, 5)
    for k, rid in enumerate(r.recv_ids):
        ranges = []
        for p in r.plan.placements:
            if p.dst_arena != rid:
                continue
            t = wl.tensors[p.tensor_id]
            got = r.image(rid)[p.data_offset:p.data_offset + p.nbytes]
            sent = r.src_images[t.src_arena][t.src_offset:t.src_offset + t.nbytes]
            assert (got == sent).all()                                    # I4
            assert struct.unpack_from("<I", r.image(rid), p.flag_offset)[0] == 5
            ranges += [(p.data_offset, p.data_offset + p.nbytes), (p.flag_offset, p.flag_offset + 4)]
        I.check_untouched(r.image(rid), r.recv_poison[k], ranges)         # I5
    for k, sid in enumerate(r.send_ids):
        assert (r.image(sid) == r.src_images[k]).all()                    # sources never change
    I.check_flag_order(r.dev.log)                                         # I7


def test_flag_order_checker_catches_planted_mistake():
    good = [("payload", 0, 1, 0, 8), ("flag_set", 0, 1, 16, 20)]
    I.check_flag_order(good)
    with pytest.raises(AssertionError):
        I.check_flag_order([("flag_set", 0, 1, 16, 20), ("payload", 0, 1, 0, 8)])
    with pytest.raises(AssertionError):
        I.check_flag_order(good + [("flag_set", 0, 1, 16, 20)])


def test_poll_consume_and_reuse_over_iterations():
    wl = W.tiny()
    r = OracleRun(wl, heap=1 << 20)
    ids = [i for i, t in enumerate(wl.tensors) if t.is_static]
    for it in range(1, 4):
        imgs = W.fill_sources(wl, variant=it)
        for sid, img in zip(r.send_ids, imgs):
            r.image(sid)[:] = img
        for t in ids:
            assert O.poll(r.dev, r.plan, t)[0] is False         # cleared at plan time / last iteration
        O.static_write(r.dev, r.plan, r.sources, it)
        for t in ids:
            p = r.plan.get(t)
            assert O.poll(r.dev, r.plan, t)[0] is True                       # non-consuming poll
            assert struct.unpack_from("<I", r.image(p.dst_arena), p.flag_offset)[0] == it
            assert O.poll(r.dev, r.plan, t, consume=True)[0] is True
            assert O.poll(r.dev, r.plan, t, consume=True)[0] is False        # I9
            ts = wl.tensors[t]
            assert (r.image(p.dst_arena)[p.data_offset:p.data_offset + p.nbytes] ==
                    imgs[0][ts.src_offset:ts.src_offset + ts.nbytes]).all()
    I.check_flag_order(r.dev.log)


def test_subset_and_errors():
    wl = W.small_mixed(2, n=6, n_recv=1)
    r = OracleRun(wl)
    O.static_write(r.dev, r.plan, r.sources, 1, tensor_ids=[3, 1])
    assert [e[1] for e in r.dev.log if e[0] == "payload"] == [3, 1]         # batch order
    assert O.poll(r.dev, r.plan, 0)[0] is False
    with pytest.raises(O.OracleError) as e:
        O.static_write(r.dev, r.plan, r.sources, 0)
    assert e.value.kind == "inval"
    with pytest.raises(O.OracleError) as e:
        O.static_write(r.dev, r.plan, {k: (v[0], v[1] + (1 << 30)) for k, v in r.sources.items()}, 1)
    assert e.value.kind == "range"
    # a source inside its own destination range
    big = next(p for p in r.plan.placements if p.nbytes > 8)
    bad = dict(r.sources)
    bad[big.tensor_id] = (big.dst_arena, big.data_offset + 4)
    before = [a.mem.copy() for a in r.dev.arenas]
    with pytest.raises(O.OracleError) as e:
        O.static_write(r.dev, r.plan, bad, 2)
    assert e.value.kind == "overlap"
    for a, b in zip(r.dev.arenas, before):                                    # validated before moving
        assert (a.mem == b).all()


def test_meta_record_matches_hand_assembled_bytes():
    want = bytearray(128)
    for line in open(os.path.join(GOLDEN, "meta_record.txt")):
        if line.startswith("#") or not line.strip():
            continue
        off, hx = line.split()[:2]
        b = bytes.fromhex(hx)
        want[int(off):int(off) + len(b)] = b
    got = O.encode_meta(2, O.DTYPE_CODE["f32"], 24, 1, 0x1234, (2, 3), 9, 5, dst_offset=0x400, meta_flag=5)
    assert got == bytes(want)
    m = O.decode_meta(got)
    assert (m["ndims"], m["dtype"], m["nbytes"], m["src_offset"], m["dims"][:3], m["dst_offset"],
            m["src_arena"], m["tensor_id"], m["seq"], m["data_flag"], m["meta_flag"]) == \
        (2, 7, 24, 0x1234, (2, 3, 0), 0x400, 1, 9, 5, 0, 5)


def test_dynamic_protocol_tiny_config():
    wl = W.tiny()
    heap = 2 << 20
    r = OracleRun(wl, heap=heap, extra_arenas=(1 << 20,))
    dyn_src_arena = r.extra_ids[0]
    dyn_ids = [i for i, t in enumerate(wl.tensors) if not t.is_static]
    f32 = O.DTYPE_CODE["f32"]
    rid = r.recv_ids[0]
    ap = r.plan.arenas[rid]
    for it in range(1, 4):
        O.dyn_reset(r.plan)
        rows = W.tiny_dynamic_rows(it)
        off = 0
        sent = {}
        for t, nrows in zip(dyn_ids, rows):
            nb = nrows * 256 * 4
            payload = W.dynamic_payload(nb, 100 * it + t)
            off = O.round_up(off, 16) + 4                       # deliberately 4-byte, not 16-byte aligned
            r.image(dyn_src_arena)[off:off + nb] = payload
            sent[t] = (off, nrows, payload)
            off += nb
        for t in dyn_ids:
            assert O.poll(r.dev, r.plan, t, which=O.POLL_META)[0] is False
            with pytest.raises(O.OracleError):
                O.dyn_recv(r.dev, r.plan, t, it)                 # nothing polled yet
            O.dyn_send(r.dev, r.plan, t, (dyn_src_arena, sent[t][0]), f32, (sent[t][1], 256), it)
        prev_end = ap.heap_offset
        for t in dyn_ids:
            assert O.poll(r.dev, r.plan, t, which=O.POLL_DATA)[0] is False
            ok, m = O.poll(r.dev, r.plan, t, consume=True, which=O.POLL_META)
            assert ok
            off, nrows, payload = sent[t]
            # I6: the record describes the tensor that was sent
            assert m["ndims"] == 2 and m["dims"][:2] == (nrows, 256) and m["dtype"] == f32
            assert m["nbytes"] == nrows * 1024 == 4 * m["dims"][0] * m["dims"][1]
            assert (m["src_arena"], m["src_offset"], m["tensor_id"], m["seq"]) == (dyn_src_arena, off, t, it)
            assert O.poll(r.dev, r.plan, t, which=O.POLL_META)[0] is False      # cleared
            dst = O.dyn_recv(r.dev, r.plan, t, it)
            # I8: inside the heap, after the previous allocation, aligned
            assert dst == prev_end and dst % 256 == 0
            assert ap.heap_offset <= dst and dst + len(payload) <= ap.heap_offset + ap.heap_bytes
            prev_end = dst + O.round_up(len(payload), 256)
            assert (r.image(rid)[dst:dst + len(payload)] == payload).all()       # I4
            ok, m2 = O.poll(r.dev, r.plan, t, consume=True, which=O.POLL_DATA)
            assert ok and m2["dst_offset"] == dst
            assert O.poll(r.dev, r.plan, t, which=O.POLL_DATA)[0] is False
    I.check_flag_order(r.dev.log)
    # static regions were never touched by the dynamic traffic
    for p in r.plan.placements:
        if p.kind == O.STATIC:
            got = r.image(rid)[p.data_offset:p.data_offset + p.region_bytes].copy()
            want = r.recv_poison[0][p.data_offset:p.data_offset + p.region_bytes].copy()
            assert (got[p.flag_offset - p.data_offset:][:4] == 0).all()     # cleared at plan time
            want[p.flag_offset - p.data_offset:][:4] = 0
            assert (got == want).all()


def test_dynamic_heap_exhaustion_and_demotion():
    dev = O.Device()
    s = dev.register_arena(np.arange(4096, dtype=np.uint8))
    r = dev.register_arena(np.zeros(4096, dtype=np.uint8))
    u8 = O.DTYPE_CODE["u8"]
    pl = O.plan(dev, [O.TensorDesc(0, u8, (-1,), r), O.TensorDesc(1, u8, (600,), r)], 256,
                max_static_bytes=512, dyn_heap_bytes=512)
    assert [p.kind for p in pl.placements] == [O.DYNAMIC, O.DYNAMIC]      # 600 B > 512 -> dynamic
    O.dyn_send(dev, pl, 0, (s, 0), u8, (300,), 1)
    O.dyn_send(dev, pl, 1, (s, 512), u8, (600,), 1)
    assert O.poll(dev, pl, 0, True, O.POLL_META)[0] and O.poll(dev, pl, 1, True, O.POLL_META)[0]
    assert O.dyn_recv(dev, pl, 0, 1) == 512                                # heap starts after two slots
    with pytest.raises(O.OracleError) as e:
        O.dyn_recv(dev, pl, 1, 1)                                          # 768 > remaining 0
    assert e.value.kind == "nomem"


@pytest.mark.parametrize("mode", [O.MODE_RPC2, O.MODE_RPC3, O.MODE_SENDERCOPY])
def test_copy_modes_deliver_what_zero_copy_delivers(mode):
    wl = W.small_mixed(21, n=10, n_recv=2, gran=1)
    total_msg = sum(128 + O.round_up(t.nbytes, 16) for t in wl.tensors)
    stage = sum(O.round_up(t.nbytes, 256) for t in wl.tensors)
    bufsz = max(total_msg, stage) + 256
    heap = stage + 512
    z = OracleRun(wl, heap=heap, extra_arenas=(bufsz, bufsz))
    c = OracleRun(wl, heap=heap, extra_arenas=(bufsz, bufsz))
    O.static_write(z.dev, z.plan, z.sources, 3)
    send = c.dev.alloc_region(c.extra_ids[0], bufsz - 256, 256)
    recv = c.dev.alloc_region(c.extra_ids[1], bufsz - 256, 256)
    O.copy_write(c.dev, c.plan, c.sources, mode, 3, send, recv)
    for p in c.plan.placements:
        zp = z.plan.get(p.tensor_id)
        want = z.image(zp.dst_arena)[zp.data_offset:zp.data_offset + zp.nbytes]
        ok, meta = O.poll(c.dev, c.plan, p.tensor_id, consume=True)
        assert ok
        if mode == O.MODE_SENDERCOPY:
            got = c.image(p.dst_arena)[p.data_offset:p.data_offset + p.nbytes]
        else:
            d = meta["dst_offset"]
            ap = c.plan.arenas[p.dst_arena]
            assert ap.heap_offset <= d and d + p.nbytes <= ap.heap_offset + ap.heap_bytes and d % 256 == 0
            got = c.image(p.dst_arena)[d:d + p.nbytes]
            # the static region itself stays untouched in the RPC modes
            k = c.recv_ids.index(p.dst_arena)
            assert (c.image(p.dst_arena)[p.data_offset:p.data_offset + p.nbytes] ==
                    c.recv_poison[k][p.data_offset:p.data_offset + p.nbytes]).all()
        assert (got == want).all()
    if mode == O.MODE_SENDERCOPY:
        # staging buffer image, byte by byte: tensor k sits at the sum of the align-rounded sizes of the
        # tensors before it, bare (no header, no padding written); everything else keeps the background
        want = [int(b) for b in c.extra_poison[0]]
        cur = send[1]
        src = c.src_images[0]
        for t in wl.tensors:
            for k in range(t.nbytes):
                want[cur + k] = int(src[t.src_offset + k])
            cur += (t.nbytes + 255) // 256 * 256
        assert c.image(c.extra_ids[0]).tolist() == want
        assert (c.image(c.extra_ids[1]) == c.extra_poison[1]).all()          # the second buffer is not used
        # and the receiver arenas equal the zero-copy run's, flags included (consumed in c, so consume in z)
        for p in z.plan.placements:
            assert O.poll(z.dev, z.plan, p.tensor_id, consume=True)[0]
        for rz, rc in zip(z.recv_ids, c.recv_ids):
            assert (z.image(rz) == c.image(rc)).all()
    # message buffer image, byte by byte, for the RPC modes
    if mode in (O.MODE_RPC2, O.MODE_RPC3):
        want = [int(b) for b in c.extra_poison[0]]
        cur = send[1]
        for i, t in enumerate(wl.tensors):
            hdr = O.encode_meta(len(t.dims), O.DTYPE_CODE[t.dtype], t.nbytes, c.send_ids[0], t.src_offset,
                                t.dims, i, 3)
            for k in range(128):
                want[cur + k] = hdr[k]
            src = c.src_images[0]
            for k in range(t.nbytes):
                want[cur + 128 + k] = int(src[t.src_offset + k])
            for k in range(t.nbytes, O.round_up(t.nbytes, 16)):
                want[cur + 128 + k] = 0
            cur += 128 + O.round_up(t.nbytes, 16)
        assert c.image(c.extra_ids[0]).tolist() == want
        if mode == O.MODE_RPC3:
            n = cur - send[1]
            assert (c.image(c.extra_ids[1])[recv[1]:recv[1] + n] ==
                    c.image(c.extra_ids[0])[send[1]:send[1] + n]).all()
            assert (c.image(c.extra_ids[1])[recv[1] + n:] == c.extra_poison[1][recv[1] + n:]).all()
        else:
            assert (c.image(c.extra_ids[1]) == c.extra_poison[1]).all()


def test_where_a_tensor_is_reported_after_rpc_then_zero_copy_delivery():
    """A copying-mode delivery lands in a fresh heap allocation and the poll says
    where; a later zero-copy delivery of the same tensor lands in its
    pre-allocated region again, so the poll must stop naming the old heap
    offset (section 3.2: the static region's address never changes; section
    2.2: an RPC receiver allocates anew for every message)."""
    wl = W.small_mixed(41, n=5, max_bytes=900, n_recv=1, gran=4)
    nmsg = sum(O.rpc_message_bytes(t.nbytes) for t in wl.tensors)
    heap = sum(O.round_up(t.nbytes, 256) for t in wl.tensors) + 256
    r = OracleRun(wl, heap=heap, extra_arenas=(nmsg + 512,))
    send = r.dev.alloc_region(r.extra_ids[0], nmsg, 256)
    sized = [i for i, t in enumerate(wl.tensors) if t.nbytes]
    O.copy_write(r.dev, r.plan, r.sources, O.MODE_RPC2, 1, send)
    ap = r.plan.arenas[r.recv_ids[0]]
    heap_ptr = ap.heap_offset
    for i, t in enumerate(wl.tensors):
        ok, meta = O.poll(r.dev, r.plan, i, consume=True)
        assert ok and meta == {"dst_offset": heap_ptr}                 # batch order, align-rounded bump
        heap_ptr += O.round_up(t.nbytes, 256)
    # zero-copy delivery of two of them: those are back in their regions, the others still in the heap
    back = sized[:2]
    O.static_write(r.dev, r.plan, r.sources, 2, tensor_ids=back)
    for i in range(len(wl.tensors)):
        ok, meta = O.poll(r.dev, r.plan, i)
        if i in back:
            assert ok and meta is None                                 # None = "in its static region"
            p = r.plan.get(i)
            t = wl.tensors[i]
            assert (r.image(p.dst_arena)[p.data_offset:p.data_offset + p.nbytes] ==
                    r.src_images[0][t.src_offset:t.src_offset + t.nbytes]).all()
        else:
            assert not ok                                              # consumed above, nothing new arrived
    assert set(r.plan.rpc_offsets) == set(range(len(wl.tensors))) - set(back)


@pytest.mark.parametrize("frag", [16, 48, 1024])
def test_fragmented_messages_byte_by_byte(frag):
    """RPC2 with fragments: the message buffer is rebuilt one byte at a time from
    the layout (128-byte header, then per fragment a 32-byte header, the piece,
    zero padding to 16), and the delivered tensors equal the unfragmented ones."""
    wl = W.small_mixed(33, n=8, max_bytes=3000, n_recv=2, gran=1)
    nmsg = sum(O.rpc_message_bytes(t.nbytes, frag) for t in wl.tensors)
    heap = sum(O.round_up(t.nbytes, 256) for t in wl.tensors) + 512
    c = OracleRun(wl, heap=heap, extra_arenas=(nmsg + 512,))
    plain = OracleRun(wl, heap=heap, extra_arenas=(nmsg + 512,))
    send = c.dev.alloc_region(c.extra_ids[0], nmsg, 256)
    O.copy_write(c.dev, c.plan, c.sources, O.MODE_RPC2, 4, send, None, frag_bytes=frag)
    O.copy_write(plain.dev, plain.plan, plain.sources, O.MODE_RPC2, 4, plain.dev.alloc_region(plain.extra_ids[0], nmsg, 256))
    for rc, rp in zip(c.recv_ids, plain.recv_ids):
        assert (c.image(rc) == plain.image(rp)).all()              # same delivery whatever the framing
    want = [int(b) for b in c.extra_poison[0]]
    cur = send[1]
    src = c.src_images[0]
    for i, t in enumerate(wl.tensors):
        hdr = O.encode_meta(len(t.dims), O.DTYPE_CODE[t.dtype], t.nbytes, c.send_ids[0], t.src_offset, t.dims, i, 4)
        want[cur:cur + 128] = list(hdr)
        cur += 128
        nfrag = -(-t.nbytes // frag)
        for k in range(nfrag):
            off = k * frag
            fb = min(frag, t.nbytes - off)
            fh = struct.pack("<IIIIQII", i, 4, k, nfrag, off, fb, 0)
            want[cur:cur + 32] = list(fh)
            for j in range(fb):
                want[cur + 32 + j] = int(src[t.src_offset + off + j])
            for j in range(fb, O.round_up(fb, 16)):
                want[cur + 32 + j] = 0
            cur += 32 + O.round_up(fb, 16)
    assert cur - send[1] == nmsg
    assert c.image(c.extra_ids[0]).tolist() == want


def test_copy_mode_buffer_too_small():
    wl = W.small_mixed(5, n=4, n_recv=1)
    c = OracleRun(wl, heap=1 << 16, extra_arenas=(512,))
    send = c.dev.alloc_region(c.extra_ids[0], 256, 256)
    before = [a.mem.copy() for a in c.dev.arenas]
    with pytest.raises(O.OracleError) as e:
        O.copy_write(c.dev, c.plan, c.sources, O.MODE_RPC2, 1, send)
    assert e.value.kind == "nomem"
    for a, b in zip(c.dev.arenas, before):
        assert (a.mem == b).all()


def test_gather_unique_rows_against_loops():
    rng = np.random.Generator(np.random.PCG64(9))
    table = rng.normal(size=(50, 6)).astype(np.float32)
    ids = rng.integers(0, 50, size=(4, 9))
    u, rows = O.gather_unique_rows(ids, table)
    seen = []
    for v in range(50):                      # ascending id, each once
        hit = False
        for a in range(4):
            for b in range(9):
                if ids[a, b] == v:
                    hit = True
        if hit:
            seen.append(v)
    assert u.tolist() == seen and u.dtype == np.int64
    for k, v in enumerate(seen):
        for j in range(6):
            assert rows[k, j] == table[v, j]


def test_lstm_sparse_workload_shape():
    ids = W.lstm_token_ids(0)
    assert ids.shape == (64, 35) and ids.dtype == np.int64 and ids.min() >= 0 and ids.max() < 40000
    counts = [len(np.unique(W.lstm_token_ids(i))) for i in range(5)]
    assert all(700 < c < 1000 for c in counts)       # about 870 distinct of 2240 Zipf(1.1) draws
    pmf = W.zipf_pmf(40000, 1.1)
    assert abs(pmf.sum() - 1) < 1e-12 and abs(pmf[0] / pmf[1] - 2 ** 1.1) < 1e-9
