"""Glue shared by the CPU tests and the GPU parity tests: turns a workload
(inputs) into the checker's descriptions and runs the checker on it."""
from __future__ import annotations

import os

import numpy as np

from oracle import rdev_oracle as O
from paper_1805_08430_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def placement_dict(p):
    return dict(tensor_id=p.tensor_id, kind=p.kind, dst_arena=p.dst_arena, data_offset=p.data_offset,
                nbytes=p.nbytes, flag_offset=p.flag_offset, meta_offset=p.meta_offset,
                region_bytes=p.region_bytes)


def oracle_descs(wl, recv_ids):
    return [O.TensorDesc(i, O.DTYPE_CODE[t.dtype], tuple(t.dims), recv_ids[t.dst_arena])
            for i, t in enumerate(wl.tensors)]


def receiver_bytes(wl, align=256, heap=0):
    """Arena size big enough for the plan: computed from tensor sizes with slack,
    not from either planner."""
    need = [0] * wl.n_receiver_arenas
    for t in wl.tensors:
        nb = t.nbytes if t.is_static else 0
        need[t.dst_arena] += nb + 2 * align + 64
    return [n + heap + 4 * align for n in need]


class OracleRun:
    """Sender arenas first (ids 0..S-1), then receiver arenas (S..S+R-1), then
    optional extra buffers: the same registration order the GPU tests use."""

    def __init__(self, wl, variant=0, align=256, heap=0, max_static=0, extra_arenas=(), descs_fn=None):
        self.wl = wl
        self.dev = O.Device()
        self.src_images = W.fill_sources(wl, variant)
        self.send_ids = [self.dev.register_arena(img.copy()) for img in self.src_images]
        self.recv_sizes = receiver_bytes(wl, align, heap)
        self.recv_poison = [W.poison(n, wl.seed + 1000 + i) for i, n in enumerate(self.recv_sizes)]
        self.recv_ids = [self.dev.register_arena(p.copy()) for p in self.recv_poison]
        self.extra_poison = [W.poison(n, wl.seed + 5000 + i) for i, n in enumerate(extra_arenas)]
        self.extra_ids = [self.dev.register_arena(p.copy()) for p in self.extra_poison]
        self.descs = descs_fn(self.recv_ids) if descs_fn else oracle_descs(wl, self.recv_ids)
        self.plan = O.plan(self.dev, self.descs, align, max_static, heap)
        self.sources = {i: (self.send_ids[t.src_arena], t.src_offset)
                        for i, t in enumerate(wl.tensors) if t.is_static}

    def image(self, arena_id):
        return self.dev.arenas[arena_id].mem
