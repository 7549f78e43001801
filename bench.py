#!/usr/bin/env python3
"""Benchmark of the zero-copy batched tensor transfer on one MI355X.

One step = one pass of the per-iteration hot path over one batch: the batched
one-sided write of every static tensor of the workload into its pre-planned
receiver region, publication of the per-tensor flags, and the receiver's poll +
consume of the previous iteration's flags.  Classification, placement and the
hand-off of addresses happen once before the timed region, as in the paper
(section 3.4: before the computation starts).  Sources and receiver arenas are
resident in HBM before timing starts.

Prints ONE JSON line.  `value` is payload bytes per second (GB/s); the roofline
object prices the copy kernel against the 8 TB/s HBM peak with algorithmic
traffic = 2 bytes per payload byte; cpu_baseline times the CPU checker's byte
mover on the host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per copy-kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what each
# counter reads for a plain 256 MiB device-to-device copy (profiles/copy_table_kernel_<workload>.md).
# Valid only for the kernel sources they were taken with: `hash` covers csrc/copy_kernel.h + csrc/copy_table.h.
TRAFFIC = {
    "vgg16": {"hash": "805ac29d6b5f4fc3", "fetch_bytes": 557744701, "write_bytes": 553430176},
    "alexnet": {"hash": "805ac29d6b5f4fc3", "fetch_bytes": 251482261, "write_bytes": 249513376},
    "tiny": {"hash": "805ac29d6b5f4fc3", "fetch_bytes": 3013694, "write_bytes": 2945216},
    "lstm": {"hash": "805ac29d6b5f4fc3", "fetch_bytes": 232774248, "write_bytes": 230948864},
    "inception": {"hash": "805ac29d6b5f4fc3", "fetch_bytes": 969978559, "write_bytes": 962396800},
}


def kernel_source_hash():
    """Hash of the dominant kernel's own sources: the copy kernel and the code that builds and orders its table."""
    import hashlib
    h = hashlib.sha256()
    for f in ("copy_kernel.h", "copy_table.h"):
        with open(os.path.join(ROOT, "paper_1805_08430_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    t = TRAFFIC.get(workload)
    if not t or t["hash"] != kernel_source_hash():
        return None                      # no counters for this workload, or the kernel changed since
    return t["fetch_bytes"] + t["write_bytes"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="vgg16", choices=["tiny", "alexnet", "vgg16", "lstm", "inception", "fcn5", "gru", "flat"])
    ap.add_argument("--rotate", type=int, default=0,
                    help="number of source/receiver set copies cycled through (0 = enough to exceed 1 GB)")
    ap.add_argument("--chunk-bytes", type=int, default=0)
    ap.add_argument("--small-bytes", type=int, default=0)
    ap.add_argument("--flag-groups", type=int, default=0,
                    help="launches per whole-plan transfer, each followed by its tensors' flags (default one)")
    ap.add_argument("--misalign", type=int, default=0,
                    help="vgg16 only: 16 = source k starts k mod 16 bytes off a 16-byte boundary (all alignment "
                         "classes); 1..15 = every source starts that many bytes off")
    ap.add_argument("--flat", default="", help="--workload flat: pieces,receiver arenas (default 1,1), 553430176 bytes in all")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-modes", action="store_true", help="skip the untimed comparison with the copying modes")
    ap.add_argument("--mode-steps", type=int, default=60)
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a few plain device-to-device copies of known size (for counter calibration)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--time-every", type=int, default=0,
                    help="time every n-th copy-kernel launch of a set with HIP events (the launch's own start/stop "
                         "events; one costs about 7 us of stream time); 0 = every 2nd in runs under 100 steps, else every 8th")
    ap.add_argument("--consume-stream", choices=["auto", "own", "delivery"], default="auto",
                    help="where the receiver's in-arena flag clears travel: a stream of the receiver's own, or the "
                         "delivery's; auto = own when an iteration moves 32 MiB or more (the step is bound by the "
                         "GPU and the clears are worth taking off the delivery stream), else the delivery's (the "
                         "step is bound by host launches and the extra event costs more than it saves)")
    ap.add_argument("--host-dynamic", action="store_true",
                    help="dynamic tensors: receive through the host (metadata poll, then rdev_read_batch) instead of on the device")
    return ap.parse_args()


class TransferSet:
    """One copy of the workload: a sender arena set, receiver arenas, a plan."""

    def __init__(self, R, torch, W, dev, wl, src_images, opts, copy_modes=False):
        self.R, self.dev = R, dev
        self.send = [torch.from_numpy(img).to("cuda:0") for img in src_images]
        self.arena_ids = [R.rdev_register_arena(dev, t.data_ptr(), t.numel()) for t in self.send]
        need = [0] * wl.n_receiver_arenas
        for t in wl.tensors:
            if t.is_static:
                need[t.dst_arena] += t.nbytes + 512 + 64
            else:
                need[t.dst_arena] += 512
        heap = 0
        self.dyn_variants = []
        self.produce = None
        dyn_ids = [i for i, t in enumerate(wl.tensors) if not t.is_static]
        if dyn_ids and not copy_modes:
            variants = dynamic_inputs(W, wl, 4)
            nsrc = max(sum((len(p) + 511) // 256 * 256 for _, _, p in v) for v in variants) + 1024
            self.dyn_src = torch.empty(4 * nsrc, dtype=torch.uint8, device="cuda:0")
            self.arena_ids.append(R.rdev_register_arena(dev, self.dyn_src.data_ptr(), self.dyn_src.numel()))
            heap = nsrc + 4096
            for vi, v in enumerate(variants):
                off = vi * nsrc
                xs = []
                for (dt, dims, payload), tid in zip(v, dyn_ids):
                    self.dyn_src[off:off + len(payload)].copy_(torch.from_numpy(payload))
                    xs.append(R.make_xfer(tid, self.dyn_src.data_ptr() + off, R.DTYPE[dt], dims))
                    off += (len(payload) + 255) // 256 * 256
                self.dyn_variants.append((R.XferArray(xs), sum(len(p) for _, _, p in v)))
            self.dyn_pull = R.XferArray([R.make_xfer(t) for t in dyn_ids])
            self.dyn_ids = dyn_ids
            self.produce = None
            if wl.name == "lstm":
                # the sparse gradient is produced on the GPU each iteration (distinct ids + their rows), and its
                # size travels to the metadata kernel through a device word: no host round trip on the sender
                import numpy as np
                self.table = torch.from_numpy(W.lstm_embedding_table()).to("cuda:0")
                self.ids = [torch.from_numpy(W.lstm_token_ids(it).reshape(-1)).to("cuda:0") for it in range(4)]
                self.count = torch.zeros(2, dtype=torch.int32, device="cuda:0")
                n_ids = self.ids[0].numel()
                row_bytes = W.LSTM_WIDTH * 4
                ids_off, rows_off = 0, (8 * n_ids + 255) // 256 * 256
                need_src = rows_off + n_ids * row_bytes + 256
                self.dyn_src2 = torch.empty(need_src, dtype=torch.uint8, device="cuda:0")
                self.arena_ids.append(R.rdev_register_arena(dev, self.dyn_src2.data_ptr(), self.dyn_src2.numel()))
                base = self.dyn_src2.data_ptr()
                xs_dev = R.XferArray([R.make_xfer(dyn_ids[0], base + ids_off, R.I64, (n_ids,), self.count.data_ptr()),
                                      R.make_xfer(dyn_ids[1], base + rows_off, R.F32, (n_ids, W.LSTM_WIDTH), self.count.data_ptr())])

                def produce(k, stream):
                    ids = self.ids[k % len(self.ids)]
                    R.rdev_gather_unique_rows(dev, ids.data_ptr(), ids.numel(), W.LSTM_VOCAB, self.table.data_ptr(),
                                              row_bytes, base + ids_off, base + rows_off, self.count.data_ptr(), stream)
                    return xs_dev
                self.produce = produce
                heap = max(heap, need_src + 4096)
        if copy_modes:                      # fresh allocations of an unpack: the largest arena load, align-padded
            heap = max(sum((t.nbytes + 255) // 256 * 256 for t in wl.static_tensors if t.dst_arena == a)
                       for a in range(wl.n_receiver_arenas)) + 4096
        self.recv = [torch.empty(n + heap + 1024, dtype=torch.uint8, device="cuda:0") for n in need]
        recv_ids = [R.rdev_register_arena(dev, t.data_ptr(), t.numel()) for t in self.recv]
        self.arena_ids += recv_ids
        self.regions = []
        descs = [R.make_desc(i, R.DTYPE[t.dtype], t.dims, recv_ids[t.dst_arena]) for i, t in enumerate(wl.tensors)]
        self.plan = R.rdev_plan(dev, descs, dyn_heap_bytes=heap, **opts)
        if copy_modes:
            frag = opts.get("rpc_frag_bytes", 0)
            nbuf = sum(128 + (t.nbytes + 255) // 256 * 256 + (32 * (t.nbytes // frag + 1) if frag else 0)
                       for t in wl.static_tensors) + 4096
            self.bufs = [torch.empty(nbuf, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
            ids = [R.rdev_register_arena(dev, b.data_ptr(), b.numel()) for b in self.bufs]
            self.arena_ids += ids
            regs = [R.rdev_alloc_region(dev, i, nbuf - 256, 256) for i in ids]
            self.regions = regs
            R.rdev_plan_bind_buffers(self.plan, regs[0], regs[1])
        ptrs = [self.send[t.src_arena].data_ptr() + t.src_offset if t.is_static else None for t in wl.tensors]
        R.rdev_plan_bind_sources(self.plan, ptrs)

    def close(self):
        self.R.rdev_plan_free(self.plan)
        for r in self.regions:
            self.R.rdev_free_region(self.dev, r)
        for a in self.arena_ids:
            self.R.rdev_unregister_arena(self.dev, a)


def dynamic_inputs(W, wl, n_variants):
    """Run-time shaped tensors of a few iterations: [(dtype, dims, payload bytes), ...] per iteration."""
    import numpy as np
    out = []
    if wl.name == "tiny":
        for it in range(n_variants):
            rows = W.tiny_dynamic_rows(it)
            out.append([("f32", (r, 256), W.dynamic_payload(r * 1024, 100 * it + k)) for k, r in enumerate(rows)])
    elif wl.name == "lstm":
        table = W.lstm_embedding_table()
        for it in range(n_variants):
            u = np.unique(W.lstm_token_ids(it).reshape(-1))
            rows = np.ascontiguousarray(table[u])
            out.append([("i64", (int(u.size),), u.astype(np.int64).view(np.uint8).copy()),
                        ("f32", (int(u.size), W.LSTM_WIDTH), rows.view(np.uint8).reshape(-1).copy())])
    return out


def tracing_leg(R, torch, dev, wl, s, spin, iters=20):
    """Section 3.4 end to end: per-tensor sends from buffers handed out by the
    instrumented allocator.  Mini-batch 1 is traced (every tensor staged through
    a registered buffer), later ones allocate the sent tensors in the registered
    arena and write them without a copy."""
    statics = [(i, t.nbytes) for i, t in enumerate(wl.tensors) if t.is_static and t.nbytes]
    total = sum(n + 512 for _, n in statics)
    pool = torch.empty(total + 4096, dtype=torch.uint8, device="cuda:0")
    arena = torch.empty(2 * total + 4096, dtype=torch.uint8, device="cuda:0")
    a_id = R.rdev_register_arena(dev, arena.data_ptr(), arena.numel())
    need = [4096] * wl.n_receiver_arenas
    for t in wl.tensors:
        if t.is_static:
            need[t.dst_arena] += t.nbytes + 576
    recv = [torch.empty(n, dtype=torch.uint8, device="cuda:0") for n in need]
    r_ids = [R.rdev_register_arena(dev, t.data_ptr(), t.numel()) for t in recv]
    plan = R.rdev_plan(dev, [R.make_desc(i, R.DTYPE[t.dtype], t.dims, r_ids[t.dst_arena])
                             for i, t in enumerate(wl.tensors) if t.is_static])
    tr = R.rdev_tracer_open(dev, pool.data_ptr(), pool.numel(), a_id)
    times, copied = [], []
    for it in range(1, iters + 2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        R.rdev_tracer_begin_iteration(tr)
        c = 0
        for i, n in statics:
            ptr, _, _ = R.rdev_tracer_alloc(tr, i, n)
            c += R.rdev_tracer_send(tr, plan, i, ptr, it, s)
        for i, _ in statics:
            spin(lambda: R.rdev_poll(dev, plan, i, R.POLL_CONSUME, s))
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) * 1e6)
        copied.append(c)
    R.rdev_tracer_close(tr)
    R.rdev_plan_free(plan)
    for a in [a_id] + r_ids:
        R.rdev_unregister_arena(dev, a)
    steady = sorted(times[1:])[len(times[1:]) // 2]
    return {"per_tensor_sends": len(statics), "traced_iteration_us": round(times[0], 1),
            "tensors_staged_in_traced_iteration": copied[0], "steady_iteration_us_median": round(steady, 1),
            "tensors_staged_in_steady_iterations": max(copied[1:]),
            "traced_over_steady": round(times[0] / steady, 3)}


def consumer_leg(R, torch, W, dev, wl, opts, s, spin, iters=20):
    """Sections 4 / 5.1: one send per tensor, each received tensor consumed by a
    reduce_max kernel on a second stream.  (a) one event at the end of the whole
    set, then all consumers; (b) polling-async: per-tensor flags polled on the
    host, a tensor's consumer starts while later tensors are still in flight."""
    images = W.fill_sources(wl, 0)
    ts = TransferSet(R, torch, W, dev, wl, images, opts)
    del images
    ids = [i for i, t in enumerate(wl.tensors) if t.is_static and t.nbytes % 4 == 0]
    xs = [[R.make_xfer(i)] for i in ids]
    res = torch.zeros(len(ids) * 24 + 16, dtype=torch.uint8, device="cuda:0")
    base = (res.data_ptr() + 15) // 16 * 16
    cons = torch.cuda.Stream()
    c = cons.cuda_stream
    seq = 0
    t_event, t_async = [], []
    for it in range(iters + 2):
        for variant in ("event", "async"):
            torch.cuda.synchronize()
            seq += 1
            t0 = time.perf_counter()
            for x in xs:
                R.rdev_write_batch(dev, ts.plan, x, R.ZEROCOPY, seq, s)
            if variant == "event":
                spin(lambda: all(R.rdev_poll(dev, ts.plan, i) for i in ids))
                for k, i in enumerate(ids):
                    R.rdev_poll(dev, ts.plan, i, R.POLL_CONSUME, s)
                    R.rdev_consume_reduce_max(dev, ts.plan, i, 0, base + 24 * k, c)
            else:
                ok, _ = R.rdev_recv_polling_async(dev, ts.plan, ids, base, s, c)
                assert ok
            cons.synchronize()
            torch.cuda.synchronize()
            (t_event if variant == "event" else t_async).append((time.perf_counter() - t0) * 1e6)
    ts.close()
    # the batched transfer cut into groups that publish their flags one after the other, received polling-async
    grouped = {}
    for G in (1, 4, 8):
        images = W.fill_sources(wl, 0)
        tg = TransferSet(R, torch, W, dev, wl, images, dict(opts, flag_groups=G))
        del images
        tt = []
        for it in range(iters + 2):
            torch.cuda.synchronize()
            seq += 1
            t0 = time.perf_counter()
            R.rdev_write_batch(dev, tg.plan, None, R.ZEROCOPY, seq, s)
            ok, _ = R.rdev_recv_polling_async(dev, tg.plan, ids, base, s, c)
            assert ok
            cons.synchronize()
            torch.cuda.synchronize()
            tt.append((time.perf_counter() - t0) * 1e6)
        tg.close()
        grouped[f"flag_groups_{G}"] = round(sorted(tt[2:])[len(tt[2:]) // 2], 1)
    # one batched write, then ONE consumer launch for the whole list: (a) after the host has seen the delivery,
    # (b) enqueued right behind the write, every unit waiting on the device for its tensor's in-arena flag
    one_launch = {}
    for G in (1, 4, 8):
        images = W.fill_sources(wl, 0)
        tg = TransferSet(R, torch, W, dev, wl, images, dict(opts, flag_groups=G))
        del images
        for how in ("after_host_poll", "waiting_on_device", "same_stream_behind_the_write"):
            tt = []
            for it in range(iters + 2):
                torch.cuda.synchronize()
                seq += 1
                t0 = time.perf_counter()
                R.rdev_write_batch(dev, tg.plan, None, R.ZEROCOPY, seq, s)
                if how == "after_host_poll":
                    spin(lambda: R.rdev_poll(dev, tg.plan, R.ALL_TENSORS))
                    R.rdev_consume_batch(dev, tg.plan, ids, 0, base, c)
                elif how == "same_stream_behind_the_write":      # stream order instead of flags: no wait at all
                    R.rdev_consume_batch(dev, tg.plan, ids, 0, base, s)
                else:
                    R.rdev_consume_batch(dev, tg.plan, ids, 50_000, base, c)
                cons.synchronize()
                torch.cuda.synchronize()
                tt.append((time.perf_counter() - t0) * 1e6)
                R.rdev_poll(dev, tg.plan, R.ALL_TENSORS, R.POLL_CONSUME, s)
            one_launch[f"{how}_flag_groups_{G}"] = round(sorted(tt[2:])[len(tt[2:]) // 2], 1)
        bare = []
        for it in range(iters + 2):
            torch.cuda.synchronize()
            seq += 1
            t0 = time.perf_counter()
            R.rdev_write_batch(dev, tg.plan, None, R.ZEROCOPY, seq, s)
            spin(lambda: R.rdev_poll(dev, tg.plan, R.ALL_TENSORS))
            torch.cuda.synchronize()
            bare.append((time.perf_counter() - t0) * 1e6)
            R.rdev_poll(dev, tg.plan, R.ALL_TENSORS, R.POLL_CONSUME, s)
        one_launch[f"bare_transfer_flag_groups_{G}"] = round(sorted(bare[2:])[len(bare[2:]) // 2], 1)
        tg.close()
    med = lambda v: sorted(v[2:])[len(v[2:]) // 2]
    return {"sends_per_iteration": len(ids), "end_of_set_event_us": round(med(t_event), 1),
            "polling_async_us": round(med(t_async), 1), "gain": round(med(t_event) / med(t_async), 3),
            "one_batched_write_polling_async_us": grouped, "one_batched_write_one_consumer_launch_us": one_launch}


def queues_leg(R, torch, W, dev, wl, opts, spin, iters=30):
    """Section 3.1 lets the caller pick the queue pair a transfer uses.  The HIP
    analogue is the stream: one explicit batch per destination arena, either all
    on one stream or each on a stream of its own, against the single launch that
    covers every arena."""
    images = W.fill_sources(wl, 0)
    ts = TransferSet(R, torch, W, dev, wl, images, opts)
    del images
    groups = {}
    for i, t in enumerate(wl.tensors):
        if t.is_static:
            groups.setdefault(t.dst_arena, []).append(R.make_xfer(i))
    groups = list(groups.values())
    ids = [x.tensor_id for g in groups for x in g]
    streams = [torch.cuda.Stream() for _ in groups]
    res = {}
    seq = 0
    for name in ("one_launch", "per_arena_one_stream", "per_arena_own_stream"):
        times = []
        for it in range(iters + 3):
            torch.cuda.synchronize()
            seq += 1
            t0 = time.perf_counter()
            if name == "one_launch":
                R.rdev_write_batch(dev, ts.plan, None, R.ZEROCOPY, seq, streams[0].cuda_stream)
            else:
                for k, g in enumerate(groups):
                    st = streams[k if name == "per_arena_own_stream" else 0]
                    R.rdev_write_batch(dev, ts.plan, g, R.ZEROCOPY, seq, st.cuda_stream)
            spin(lambda: all(R.rdev_poll(dev, ts.plan, i) for i in ids))
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) * 1e6)
            R.rdev_poll(dev, ts.plan, R.ALL_TENSORS, R.POLL_CONSUME, streams[0].cuda_stream)
        res[name] = round(sorted(times[3:])[len(times[3:]) // 2], 1)
    ts.close()
    return {"destination_arenas": len(groups), "us_per_iteration": res}


def graph_leg(R, torch, W, dev, wl, opts, spin, iters=30):
    """One send per tensor (the granularity of the paper's send operator) is bound by
    launches; the same sequence recorded once into a HIP graph and replayed."""
    images = W.fill_sources(wl, 0)
    ts = TransferSet(R, torch, W, dev, wl, images, opts)
    del images
    ids = [i for i, t in enumerate(wl.tensors) if t.is_static]
    xs = [[R.make_xfer(i)] for i in ids]
    st = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=st):
        for x in xs:
            R.rdev_write_batch(dev, ts.plan, x, R.ZEROCOPY, 1, st.cuda_stream)
    st.synchronize()
    res = {}
    for name in ("eager", "graph_replay"):
        tt = []
        for it in range(iters + 3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if name == "eager":
                for x in xs:
                    R.rdev_write_batch(dev, ts.plan, x, R.ZEROCOPY, 1, st.cuda_stream)
            else:
                with torch.cuda.stream(st):
                    graph.replay()
            spin(lambda: all(R.rdev_poll(dev, ts.plan, i) for i in ids))
            tt.append((time.perf_counter() - t0) * 1e6)
            for i in ids:
                R.rdev_poll(dev, ts.plan, i, R.POLL_CONSUME, st.cuda_stream)
            st.synchronize()
        res[name + "_us"] = round(sorted(tt[3:])[len(tt[3:]) // 2], 1)
    del graph
    ts.close()
    res["sends"] = len(ids)
    return res


def cpu_baseline(wl_name: str, seconds: float):
    """The CPU checker's static transfer on the same workload, as it stands."""
    import numpy as np
    from oracle import rdev_oracle as O
    from paper_1805_08430_amd import workloads as W
    wl = {**W.CONFIGS, **W.EXTRA_CONFIGS}[wl_name]()
    dev = O.Device()
    send_ids = [dev.register_arena(np.zeros(n, dtype=np.uint8)) for n in wl.sender_bytes]
    for sid in send_ids:
        dev.arenas[sid].mem[:] = 1                              # touch the pages
    need = [0] * wl.n_receiver_arenas
    for t in wl.tensors:
        need[t.dst_arena] += (t.nbytes if t.is_static else 0) + 1024
    recv_ids = [dev.register_arena(np.zeros(n + 1024, dtype=np.uint8)) for n in need]
    descs = [O.TensorDesc(i, O.DTYPE_CODE[t.dtype], tuple(t.dims), recv_ids[t.dst_arena])
             for i, t in enumerate(wl.tensors)]
    pl = O.plan(dev, descs)
    sources = {i: (send_ids[t.src_arena], t.src_offset) for i, t in enumerate(wl.tensors) if t.is_static}
    static_ids = list(sources)
    times = []
    t_end = time.perf_counter() + seconds
    it = 0
    while True:
        it += 1
        dev.log.clear()
        t0 = time.perf_counter()
        O.static_write(dev, pl, sources, it)
        for t in static_ids:
            O.poll(dev, pl, t, consume=True)
        times.append(time.perf_counter() - t0)
        if (it >= 3 and time.perf_counter() > t_end) or it >= 200:
            break
    times = times[1:] if len(times) > 3 else times               # first pass faults the pages in
    med = sorted(times)[len(times) // 2]
    out = {"value": round(wl.payload_bytes / med / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "host_cpu_count": os.cpu_count(),
           "sample": f"{len(times)} iterations of the full {wl_name} static set ({wl.payload_bytes} B each), "
                     f"median; numpy slice copies are single-threaded",
           "us_per_iteration": round(med * 1e6, 1)}
    # the same checker call spread over host threads (numpy releases the interpreter lock while copying):
    # tensors dealt to threads by size, each thread moves its share with the unchanged static_write
    import threading
    T = max(1, min(16, os.cpu_count() or 1))      # the box's share of host cores for one GPU is 16, whatever it shows
    if T > 1 and len(static_ids) > 1:
        shares = [[] for _ in range(T)]
        load = [0] * T
        for t in sorted(static_ids, key=lambda i: -wl.tensors[i].nbytes):
            k = load.index(min(load))
            shares[k].append(t)
            load[k] += wl.tensors[t].nbytes
        shares = [sh for sh in shares if sh]
        tt = []
        for it in range(8):
            dev.log.clear()
            ths = [threading.Thread(target=O.static_write, args=(dev, pl, sources, it + 1, sh)) for sh in shares]
            t0 = time.perf_counter()
            for th in ths:
                th.start()
            for th in ths:
                th.join()
            tt.append(time.perf_counter() - t0)
            for t in static_ids:
                O.poll(dev, pl, t, consume=True)
        m = sorted(tt[1:])[len(tt[1:]) // 2]
        out["threaded"] = {"value": round(wl.payload_bytes / m / 1e9, 3), "unit": "GB/s", "cores": len(shares),
                           "note": "whole tensors dealt to threads; the largest tensor bounds the speed-up"}
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: the library moves tensors inside one GPU only (sender and receiver arenas share one HBM); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1805_08430_amd import rdev as R
    from paper_1805_08430_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    R.lib()
    if a.workload == "flat":
        pieces, n_recv = (int(v) for v in (a.flat or "1,1").split(","))
        wl = W.flat(pieces=pieces, n_recv=n_recv)
    elif a.misalign and a.workload == "vgg16":
        wl = W.vgg16(misalign=True if a.misalign == 16 else a.misalign)
    else:
        wl = {**W.CONFIGS, **W.EXTRA_CONFIGS}[a.workload]()
    payload = wl.payload_bytes
    rotate = a.rotate or max(2, -(-(1 << 30) // max(2 * payload, 1)))
    rotate = min(rotate, 64)
    dev = R.rdev_open(0)
    opts = dict(chunk_bytes=a.chunk_bytes, small_bytes=a.small_bytes, flag_groups=a.flag_groups)
    images = W.fill_sources(wl, 0)
    sets = [TransferSet(R, torch, W, dev, wl, images, opts) for _ in range(rotate)]
    del images
    stream = torch.cuda.Stream()
    s = stream.cuda_stream
    stream2 = torch.cuda.Stream()           # dynamic-size traffic travels on its own queue
    s2 = stream2.cuda_stream
    stream_r = torch.cuda.Stream()          # the receiver's own queue: the in-arena clears of consumed flags
    sr = stream_r.cuda_stream
    has_dyn = bool(sets[0].dyn_variants)
    dyn_bytes = (sum(b for _, b in sets[0].dyn_variants) / len(sets[0].dyn_variants)) if has_dyn else 0
    torch.cuda.synchronize()

    consume_own = a.consume_stream == "own" or (a.consume_stream == "auto" and payload >= (32 << 20))

    def spin(fn):
        spins = 0
        while not fn():
            spins += 1
            if spins > 50_000_000:
                raise RuntimeError("flag never became visible")

    def wait_consume(ts, alone=False):
        # rotating sets: the clears travel on the receiver's own stream, off the next delivery's path; one set alone:
        # the next delivery has to wait for the clear anyway, and the delivery's own stream is the cheapest order
        own = consume_own and not alone
        spin(lambda: R.rdev_poll(dev, ts.plan, R.ALL_TENSORS, R.POLL_CONSUME, sr if own else s))
        if ts.dyn_variants:
            for t in ts.dyn_ids:
                spin(lambda: R.rdev_poll(dev, ts.plan, t, R.POLL_CONSUME, sr if own else s2))

    seq = 0

    def run(steps, group=None, mode=R.ZEROCOPY):
        nonlocal seq
        group = group or sets
        prev = None
        for k in range(steps):
            ts = group[k % len(group)]
            seq += 1
            if mode != R.ZEROCOPY:
                R.rdev_dyn_reset(ts.plan)
            R.rdev_write_batch(dev, ts.plan, None, mode, seq, s)
            if ts.dyn_variants:
                # section 3.3: metadata + flag, receiver polls, allocates, pulls, raises payload-complete
                R.rdev_dyn_reset(ts.plan)
                xs = ts.produce(k, s2) if ts.produce else ts.dyn_variants[k % len(ts.dyn_variants)][0]
                R.rdev_write_batch(dev, ts.plan, xs, R.ZEROCOPY, seq, s2)
                if a.host_dynamic:
                    for t in ts.dyn_ids:
                        spin(lambda: R.rdev_poll(dev, ts.plan, t, R.POLL_META | R.POLL_CONSUME, s2))
                    R.rdev_read_batch(dev, ts.plan, ts.dyn_pull, seq, s2)
                else:                   # the receiver's half runs on the GPU behind the metadata write
                    R.rdev_read_batch_device(dev, ts.plan, ts.dyn_pull, seq, s2)
            if len(group) == 1:
                wait_consume(ts, True)  # one set only: the next write must wait for this consumption (no ack exists)
                continue
            if prev is not None:
                wait_consume(prev)
            prev = ts
        if prev is not None:
            wait_consume(prev)

    per_set = -(-a.steps // rotate)
    time_every = a.time_every or (2 if a.steps < 100 else 8)
    for ts in sets:
        R.rdev_plan_profile(ts.plan, per_set, 1 << 30)      # create the events now; nothing is timed during warm-up
    run(a.warmup)
    torch.cuda.synchronize()                                # every stream of the device
    for ts in sets:
        R.rdev_plan_profile(ts.plan, per_set, time_every)   # re-arm only: the GPU does not sit idle before the timed region
    t0 = time.perf_counter()
    run(a.steps)
    torch.cuda.synchronize()                                # (a wait per stream first would add 10 us each to the timed region)
    t1 = time.perf_counter()

    kernel_ms = []
    for ts in sets:
        kernel_ms += R.rdev_plan_profile_read(ts.plan, per_set)
        R.rdev_plan_profile(ts.plan, 0, 1)
    ms_per_step = (t1 - t0) / a.steps * 1e3
    k_avg = sum(kernel_ms) / len(kernel_ms)
    algo_bytes = 2 * payload                                  # one read + one write per payload byte
    achieved = algo_bytes / (k_avg * 1e-3) / 1e9
    out = {
        "metric": "effective tensor-transfer GB/s (payload bytes delivered per second, zero-copy static path); "
                  "also us per iteration and fraction of HBM peak",
        "value": round((payload + dyn_bytes) / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}-shaped fp32 tensor set, {len(wl.static_tensors)} static tensors, "
                               f"{payload} payload bytes per iteration, {wl.n_sender_arenas} sender arena(s) -> "
                               f"{wl.n_receiver_arenas} receiver arena(s) in one HBM",
                   "rotating_sets": rotate, "chunk_bytes": a.chunk_bytes or 16384,
                   "dynamic_payload_bytes_per_iteration": round(dyn_bytes),
                   "step": "write_batch (copy kernel + flag kernel)" +
                           (" + dynamic tensors: " + ("distinct ids and their rows gathered on the GPU, " if sets[0].produce else "")
                            + ("metadata write, host poll of the metadata, allocate + pull" if a.host_dynamic else
                               "metadata write, then the receiver's allocate + pull on the GPU without a host poll")
                            + ", on a second stream" if has_dyn else "")
                           + " + poll/consume of the previous iteration (in-arena clears on "
                           + ("the receiver's own stream)" if consume_own else "the delivery's stream)")},
        "us_per_iteration": round(ms_per_step * 1e3, 2),
        "hbm_gbs_per_step": round(algo_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "hbm_frac_per_step": round(algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "roofline": {"bound": "hbm", "kernel": "copy_table_kernel", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(a.workload), "kernel_us_avg": round(k_avg * 1e3, 2),
                     "kernel_us_min": round(min(kernel_ms) * 1e3, 2), "kernel_us_max": round(max(kernel_ms) * 1e3, 2),
                     "launches_timed": len(kernel_ms), "timed_every": time_every, "algorithmic_bytes_per_launch": algo_bytes},
        "paper_context": {"note": "speed-ups the paper reports for its RDMA zero-copy transfer on 2 servers with "
                                  "100 Gbps InfiniBand (Xeon E5-2690v4, Tesla P100): context only",
                          "vs_grpc_tcp": "1.7x-61x", "vs_grpc_rdma": "1.3x-14x", "vs_rdma_sender_copy": "1.2x-1.8x"},
    }
    # the paper's reporting protocol (section 5): 5 runs of 100 iterations each, mean and range; outside `value`
    runs = []
    for _ in range(5):
        torch.cuda.synchronize()
        r0 = time.perf_counter()
        run(100)
        stream.synchronize()
        stream2.synchronize()
        torch.cuda.synchronize()
        runs.append((time.perf_counter() - r0) / 100 * 1e6)
    out["five_runs_of_100"] = {"us_per_iteration_mean": round(sum(runs) / 5, 2), "min": round(min(runs), 2),
                               "max": round(max(runs), 2)}
    # one set only (no rotation): every write waits for the consumption of the one before it
    torch.cuda.synchronize()
    r0 = time.perf_counter()
    run(100, [sets[0]])
    torch.cuda.synchronize()
    out["single_set_us_per_iteration"] = round((time.perf_counter() - r0) / 100 * 1e6, 2)
    if has_dyn:
        # the dynamic protocol on its own (section 3.3): metadata + flag -> receiver allocates + pulls -> payload flag
        # seen on the host; with the receiver's half driven by the host (two polls) or running on the GPU (one)
        ts = sets[0]
        rt = {}
        for how in ("host_polled", "device_side"):
            lat = []
            for k in range(203):
                xs, _ = ts.dyn_variants[k % len(ts.dyn_variants)]
                seq += 1
                torch.cuda.synchronize()
                d0 = time.perf_counter()
                R.rdev_dyn_reset(ts.plan)
                if ts.produce:
                    xs = ts.produce(k, s2)
                R.rdev_write_batch(dev, ts.plan, xs, R.ZEROCOPY, seq, s2)
                if how == "host_polled":
                    for t in ts.dyn_ids:
                        spin(lambda: R.rdev_poll(dev, ts.plan, t, R.POLL_META | R.POLL_CONSUME, s2))
                    R.rdev_read_batch(dev, ts.plan, ts.dyn_pull, seq, s2)
                else:
                    R.rdev_read_batch_device(dev, ts.plan, ts.dyn_pull, seq, s2)
                for t in ts.dyn_ids:
                    spin(lambda: R.rdev_poll(dev, ts.plan, t, R.POLL_CONSUME, s2))
                lat.append((time.perf_counter() - d0) * 1e6)
            lat = sorted(lat[3:])
            rt[how] = {"median": round(lat[len(lat) // 2], 2), "min": round(lat[0], 2),
                       "p90": round(lat[int(len(lat) * 0.9)], 2)}
        rt.update({"tensors": len(ts.dyn_ids), "payload_bytes_mean": round(dyn_bytes),
                   "includes_gather_on_gpu": bool(ts.produce)})
        out["dynamic_round_trip_us"] = rt
    props = torch.cuda.get_device_properties(0)
    dev_info = {"name": props.name, "compute_units": props.multi_processor_count,
                "hbm_bytes": props.total_memory}
    info = R.rdev_device_info(dev)
    # what the runtime reports (2 GHz x 8192 bits on this part; HBM3E moves 4 bits per pin per reported clock,
    # i.e. 8.19 TB/s); the roofline uses the published 8 TB/s
    dev_info.update(info)
    out["device"] = dev_info
    for ts in sets:
        ts.close()
    del sets
    torch.cuda.empty_cache()

    if not a.no_modes:
        # untimed-for-`value` comparison: the same batch through the copying paths the paper replaces
        images = W.fill_sources(wl, 0)
        msets = [TransferSet(R, torch, W, dev, wl, images, opts, copy_modes=True) for _ in range(2)]
        del images
        res = {}
        for name, mode in (("zerocopy", R.ZEROCOPY), ("sendercopy", R.SENDERCOPY), ("rpc2", R.RPC2), ("rpc3", R.RPC3),
                           ("runtime_memcpy_per_tensor", R.DMA)):
            run(5, msets, mode)
            torch.cuda.synchronize()
            m0 = time.perf_counter()
            run(a.mode_steps, msets, mode)
            torch.cuda.synchronize()
            res[name] = (time.perf_counter() - m0) / a.mode_steps * 1e6
        out["modes"] = {"us_per_iteration": {k: round(v, 2) for k, v in res.items()},
                        "slowdown_vs_zerocopy": {k: round(v / res["zerocopy"], 3) for k, v in res.items()},
                        "algorithmic_hbm_bytes_per_payload_byte": {"zerocopy": 2, "sendercopy": 4, "rpc2": 4, "rpc3": 6,
                                                                   "runtime_memcpy_per_tensor": 2},
                        "steps_each": a.mode_steps, "rotating_sets": 2}
        for ts in msets:
            ts.close()
        del msets
        # the same RPC3 path with every payload cut into 1 MiB fragments (section 2.2: bounded receive buffers)
        images = W.fill_sources(wl, 0)
        fsets = [TransferSet(R, torch, W, dev, wl, images, dict(opts, rpc_frag_bytes=1 << 20), copy_modes=True)
                 for _ in range(2)]
        del images
        run(5, fsets, R.RPC3)
        torch.cuda.synchronize()
        m0 = time.perf_counter()
        run(a.mode_steps, fsets, R.RPC3)
        torch.cuda.synchronize()
        res["rpc3_fragments_1MiB"] = (time.perf_counter() - m0) / a.mode_steps * 1e6
        out["modes"]["us_per_iteration"]["rpc3_fragments_1MiB"] = round(res["rpc3_fragments_1MiB"], 2)
        out["modes"]["slowdown_vs_zerocopy"]["rpc3_fragments_1MiB"] = round(res["rpc3_fragments_1MiB"] / res["zerocopy"], 3)
        for ts in fsets:
            ts.close()
        del fsets
        out["tracing"] = tracing_leg(R, torch, dev, wl, s, spin)
        out["consumer_overlap"] = consumer_leg(R, torch, W, dev, wl, opts, s, spin)
        out["queues"] = queues_leg(R, torch, W, dev, wl, opts, spin)
        out["per_tensor_sends"] = graph_leg(R, torch, W, dev, wl, opts, spin)
    if a.calibrate:
        nb = 256 << 20
        x = torch.ones(nb, dtype=torch.uint8, device="cuda:0")
        y = torch.empty_like(x)
        with torch.cuda.stream(stream):
            for _ in range(5):
                y.copy_(x)
        stream.synchronize()
        out["calibration"] = {"plain_copy_bytes": nb, "copies": 5}
    R.rdev_close(dev)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a.workload, a.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
