"""CPU checker for the analyzer's static shape inference (paper section 3.4,
first step: user annotations on input tensors + a shape-inference function per
graph node tell which transferred tensors have shapes that never change).

THIS IS TEST INFRASTRUCTURE, independent of the library (no shared code).

A graph is a list of values.  Inputs carry an annotated shape (-1 = unknown dim)
and the partition they live in; a node names an op, its input values, integer
attributes and its partition, and produces one value.  `infer` walks the nodes
in insertion order and applies the op's shape rule; `transfers` lists every
(value, consumer partition) pair whose partitions differ, in (value, partition)
order: those are the tensors the planner has to place.

Pins (tests, CPU): for fully known shapes every rule is checked against what
numpy does to real arrays of that shape (broadcasting, matmul, transpose,
reshape, concatenate, reductions, fancy indexing); unknown-dim propagation and
the data-parallel parameter-server example are worked by hand in tests/golden.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

UNARY, BINARY, MATMUL, TRANSPOSE, RESHAPE, CONCAT, REDUCE, GATHER, UNIQUE, CONV2D, GRAD, CAST = range(12)


class GraphError(Exception):
    pass


@dataclass
class Val:
    dtype: int
    dims: Optional[Tuple[int, ...]]
    partition: int


@dataclass
class Nd:
    op: int
    inputs: Tuple[int, ...]
    attrs: Tuple[int, ...]
    partition: int
    out: int


class Graph:
    def __init__(self):
        self.values: List[Val] = []
        self.nodes: List[Nd] = []

    def input(self, dtype: int, dims: Sequence[int], partition: int) -> int:
        self.values.append(Val(dtype, tuple(dims), partition))
        return len(self.values) - 1

    def node(self, op: int, inputs: Sequence[int], attrs: Sequence[int], partition: int) -> int:
        for v in inputs:
            if v >= len(self.values):
                raise GraphError("input does not exist yet")
        self.values.append(Val(0, None, partition))
        self.nodes.append(Nd(op, tuple(inputs), tuple(attrs), partition, len(self.values) - 1))
        return len(self.values) - 1

    # -- shape rules ---------------------------------------------------------
    def infer(self) -> None:
        for n in self.nodes:
            ins = [self.values[v] for v in n.inputs]
            dt, dims = self._rule(n, ins)
            if len(dims) > 8:
                raise GraphError("rank too large")
            self.values[n.out].dtype, self.values[n.out].dims = dt, tuple(dims)

    @staticmethod
    def _rule(n: Nd, ins: List[Val]):
        op, at = n.op, n.attrs
        if op == UNARY:
            (a,) = ins
            return a.dtype, a.dims
        if op == CAST:
            (a,) = ins
            return at[0], a.dims
        if op == GRAD:
            return ins[-1].dtype, ins[-1].dims
        if op == UNIQUE:
            return ins[0].dtype, (-1,)
        if op == BINARY:
            a, b = ins
            if a.dtype != b.dtype:
                raise GraphError("types")
            x, y = list(a.dims)[::-1], list(b.dims)[::-1]
            out = []
            for k in range(max(len(x), len(y))):
                p = x[k] if k < len(x) else 1
                q = y[k] if k < len(y) else 1
                if p == 1:
                    out.append(q)
                elif q == 1:
                    out.append(p)
                elif p == -1:
                    out.append(q)
                elif q == -1 or p == q:
                    out.append(p)
                else:
                    raise GraphError("broadcast")
            return a.dtype, out[::-1]
        if op == MATMUL:
            a, b = ins
            if a.dtype != b.dtype or len(a.dims) < 2 or len(b.dims) != 2:
                raise GraphError("matmul operands")
            x, y = list(a.dims), list(b.dims)
            if at[0]:
                x[-1], x[-2] = x[-2], x[-1]
            if at[1]:
                y = y[::-1]
            if x[-1] >= 0 and y[0] >= 0 and x[-1] != y[0]:
                raise GraphError("inner dims")
            return a.dtype, x[:-1] + [y[1]]
        if op == TRANSPOSE:
            (a,) = ins
            if sorted(at) != list(range(len(a.dims))):
                raise GraphError("permutation")
            return a.dtype, [a.dims[p] for p in at]
        if op == RESHAPE:
            (a,) = ins
            tgt = list(at)
            if tgt.count(-1) > 1 or any(d < -1 for d in tgt):
                raise GraphError("target")
            if all(d >= 0 for d in a.dims):
                total = 1
                for d in a.dims:
                    total *= d
                rest = 1
                for d in tgt:
                    if d != -1:
                        rest *= d
                if -1 in tgt:
                    if rest == 0 or total % rest:
                        raise GraphError("count")
                    tgt[tgt.index(-1)] = total // rest
                elif rest != total:
                    raise GraphError("count")
            return a.dtype, tgt
        if op == CONCAT:
            ax = at[0]
            first = ins[0]
            if not 0 <= ax < len(first.dims):
                raise GraphError("axis")
            out = list(first.dims)
            for b in ins[1:]:
                if len(b.dims) != len(out) or b.dtype != first.dtype:
                    raise GraphError("rank/type")
                for k in range(len(out)):
                    if k == ax:
                        out[k] = out[k] + b.dims[k] if out[k] >= 0 and b.dims[k] >= 0 else -1
                    elif out[k] >= 0 and b.dims[k] >= 0:
                        if out[k] != b.dims[k]:
                            raise GraphError("dims")
                    elif out[k] < 0:
                        out[k] = b.dims[k]
            return first.dtype, out
        if op == REDUCE:
            (a,) = ins
            keep, axes = at[0], at[1:]
            if len(set(axes)) != len(axes) or any(not 0 <= x < len(a.dims) for x in axes):
                raise GraphError("axes")
            out = []
            for k, d in enumerate(a.dims):
                if k not in axes:
                    out.append(d)
                elif keep:
                    out.append(1)
            return a.dtype, out
        if op == GATHER:
            p, ids = ins
            if not p.dims:
                raise GraphError("scalar params")
            return p.dtype, list(ids.dims) + list(p.dims[1:])
        if op == CONV2D:
            x, f = ins
            if len(x.dims) != 4 or len(f.dims) != 4 or at[0] < 1 or at[1] < 1:
                raise GraphError("conv operands")
            if x.dims[3] >= 0 and f.dims[2] >= 0 and x.dims[3] != f.dims[2]:
                raise GraphError("channels")

            def od(i, k, s):
                if i < 0 or k < 0:
                    return -1
                if at[2]:
                    return -(-i // s)
                return (i - k) // s + 1 if i >= k else 0
            return x.dtype, [x.dims[0], od(x.dims[1], f.dims[0], at[0]), od(x.dims[2], f.dims[1], at[1]), f.dims[3]]
        raise GraphError("unknown op")

    def transfers(self) -> List[Tuple[int, int]]:
        """(value, consumer partition) for every edge that crosses partitions, sorted, each once."""
        out = set()
        for n in self.nodes:
            for v in n.inputs:
                if self.values[v].partition != n.partition:
                    out.add((v, n.partition))
        return sorted(out)
