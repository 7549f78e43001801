"""Explicit batches recorded into a HIP graph: every replay must deliver exactly
what the eager call delivers (checked replay by replay, with the program's own
eager work and synchronisations in between)."""
import numpy as np
import pytest
import torch

from oracle import rdev_oracle as O
from paper_1805_08430_amd import rdev as R
from paper_1805_08430_amd import workloads as W
from helpers import OracleRun
from test_gpu_static import _compare_all

pytestmark = pytest.mark.gpu


def test_explicit_batch_graph_replays():
    from gpu_harness import GpuRun
    wl = W.small_mixed(91, n=20, max_bytes=400000, n_recv=2, gran=4)
    g, o = GpuRun(wl), OracleRun(wl)
    ids = list(range(20))
    xs = [R.make_xfer(t) for t in ids]
    # eager reference delivery
    R.rdev_write_batch(g.dev, g.plan, xs, R.ZEROCOPY, 3, g.s)
    O.static_write(o.dev, o.plan, o.sources, 3, tensor_ids=ids)
    for t in ids:
        g.wait(t, R.POLL_CONSUME)
        O.poll(o.dev, o.plan, t, consume=True)
    _compare_all(g, o, "eager")
    # record the same batch (one send per tensor, as the paper's runtime issues them)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=g.stream):
        for x in xs:
            R.rdev_write_batch(g.dev, g.plan, [x], R.ZEROCOPY, 7, g.stream.cuda_stream)
    g.stream.synchronize()
    _compare_all(g, o, "recording moves nothing")
    for t in ids:
        assert not R.rdev_poll(g.dev, g.plan, t)
    for rep in range(5):
        imgs = W.fill_sources(wl, variant=300 + rep)           # eager work between replays
        g.set_sources(imgs)
        for sid, img in zip(o.send_ids, imgs):
            o.image(sid)[:] = img
        with torch.cuda.stream(g.stream):
            graph.replay()
        O.static_write(o.dev, o.plan, o.sources, 7, tensor_ids=ids)
        for t in ids:
            g.wait(t)
        _compare_all(g, o, f"replay {rep}")
        for t in ids:
            assert R.rdev_poll(g.dev, g.plan, t, R.POLL_CONSUME, g.s)
            assert O.poll(o.dev, o.plan, t, consume=True)[0]
        g.stream.synchronize()
        _compare_all(g, o, f"replay {rep} consumed")
    del graph
    g.close()
