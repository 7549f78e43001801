"""Checks that any plan and any post-transfer arena image must pass, whoever
produced them (the CPU checker or the GPU library).  Placements are given as
plain dicts so that neither producer's types leak in here.

I1 regions inside the arena; I2 pairwise disjoint; I3 alignment; I5 bytes
outside written ranges unchanged; I10 offsets = prefix sums in input order."""
from __future__ import annotations

import numpy as np

STATIC, DYNAMIC = 0, 1


def region_span(p):
    start = p["data_offset"] if p["kind"] == STATIC else p["meta_offset"]
    return start, start + p["region_bytes"]


def check_plan(placements, arena_bytes, align, bases=None):
    """placements: list of dicts (tensor_id, kind, dst_arena, data_offset, nbytes,
    flag_offset, meta_offset, region_bytes).  arena_bytes: dict arena -> size."""
    per = {}
    for p in placements:
        lo, hi = region_span(p)
        assert lo % align == 0, ("I3 region start", p)
        assert p["region_bytes"] % align == 0 and p["region_bytes"] > 0, ("I3 region size", p)
        assert p["flag_offset"] % 4 == 0, ("I3 flag", p)
        assert 0 <= lo and hi <= arena_bytes[p["dst_arena"]], ("I1", p)
        if p["kind"] == STATIC:
            assert lo + p["nbytes"] <= p["flag_offset"], ("flag after payload", p)
            assert p["flag_offset"] - (lo + p["nbytes"]) < 16, ("flag right after padded payload", p)
            assert p["flag_offset"] % 16 == 0
        else:
            assert p["flag_offset"] == lo + 124, ("meta flag is the last word", p)
        assert p["flag_offset"] + 4 <= hi, ("flag inside region", p)
        per.setdefault(p["dst_arena"], []).append((lo, hi, p["tensor_id"]))
    for a, spans in per.items():
        # I2 by sweep
        s = sorted(spans)
        for (l0, h0, t0), (l1, h1, t1) in zip(s, s[1:]):
            assert h0 <= l1, ("I2 overlap", a, t0, t1)
        # I2 brute force for small n
        if len(spans) <= 64:
            for i in range(len(spans)):
                for j in range(i + 1, len(spans)):
                    a0, b0, _ = spans[i]
                    a1, b1, _ = spans[j]
                    assert b0 <= a1 or b1 <= a0, ("I2 brute", a, i, j)
        # I10 input order, no gaps: start of k-th region = base + sum of earlier region sizes
        base = spans[0][0] if bases is None else bases[a]
        ptr = base
        for lo, hi, t in spans:
            assert lo == ptr, ("I10 prefix sum", a, t, lo, ptr)
            ptr = hi


def written_mask(nbytes, ranges):
    m = np.zeros(nbytes, dtype=bool)
    for lo, hi in ranges:
        m[lo:hi] = True
    return m


def check_untouched(image, poison, ranges):
    """I5: every byte outside `ranges` still equals the background pattern."""
    m = written_mask(image.size, ranges)
    bad = np.nonzero((image != poison) & ~m)[0]
    assert bad.size == 0, ("I5 stray write at", bad[:8])


def check_flag_order(log):
    """I7 on an event log [(kind, tensor, arena, lo, hi)]: in each tensor's own
    sub-sequence every flag_set comes directly after a payload or metadata store
    of that tensor (never first, never after another flag_set or a clear), so no
    flag can be visible before the bytes it announces."""
    last = {}
    for kind, t, a, lo, hi in log:
        if t < 0:
            continue
        if kind == "flag_set":
            assert last.get(t) in ("payload", "meta"), ("I7 flag without preceding payload", t, last.get(t))
        if kind in ("payload", "meta", "flag_set", "flag_clear"):
            last[t] = kind
