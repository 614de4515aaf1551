"""Neutral, arithmetic-free description of a synthesized operator.

An operator is a primitive graph (pGraph, paper section 5.1): the bottom is the
list of output iterators, every primitive of Table 1 rewrites coordinates
bottom-up, and the top is the ordered list of coordinates that index the data
input plus the ordered list of coordinates that index the weight.

This module only *records* such a graph.  It evaluates nothing: the meaning of
each primitive lives, separately, in the CPU checker and in the GPU library,
each of which converts an `OpDesc` into its own private format.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

# Primitive kinds, in the order of Table 1 of the paper.
SPLIT, MERGE, SHIFT, EXPAND, UNFOLD, STRIDE, REDUCE, SHARE = range(8)
KIND_NAMES = ("Split", "Merge", "Shift", "Expand", "Unfold", "Stride", "Reduce", "Share")

F32, BF16 = 0, 1


@dataclass(frozen=True)
class Prim:
    """One vertex of the pGraph.

    ins  : coordinate ids consumed on the bottom side (towards the output)
    outs : coordinate ids produced on the top side (towards the input)
    param: Merge B, Stride S, Reduce N, Shift constant offset s
    shift_by / shift_coef: Shift only; the offset additionally gets
        shift_coef * value(shift_by).  shift_by is read, not consumed; -1 = none.
    """
    kind: int
    ins: Tuple[int, ...]
    outs: Tuple[int, ...]
    param: int = 0
    shift_by: int = -1
    shift_coef: int = 0


@dataclass
class OpDesc:
    out_dims: List[Tuple[str, int]]          # output iterators, in output layout order
    prims: List[Prim] = field(default_factory=list)
    input_coords: List[int] = field(default_factory=list)    # axes of X, row-major
    weight_coords: List[int] = field(default_factory=list)   # axes of W, row-major
    more_weights: List[List[int]] = field(default_factory=list)   # axes of the further weights W_1, W_2, ... (usually none)
    in_dtype: int = F32                      # dtype of X, W and the upstream gradient G
    out_dtype: int = F32                     # dtype of out and dX (dW is always fp32)
    name: str = ""


class Builder:
    """Hands out coordinate ids while a pGraph is written down bottom-up."""

    def __init__(self, out_dims: Sequence[Tuple[str, int]], name: str = ""):
        self.desc = OpDesc(out_dims=[(str(n), int(s)) for n, s in out_dims], name=name)
        self._next = len(self.desc.out_dims)

    def out(self, i: int) -> int:
        return i

    def _new(self) -> int:
        c = self._next
        self._next += 1
        return c

    def split(self, i: int, j: int) -> int:
        v = self._new()
        self.desc.prims.append(Prim(SPLIT, (i, j), (v,)))
        return v

    def merge(self, i: int, B: int) -> Tuple[int, int]:
        q, r = self._new(), self._new()
        self.desc.prims.append(Prim(MERGE, (i,), (q, r), param=int(B)))
        return q, r

    def shift(self, i: int, s: int = 1, by: int = -1, coef: int = 0) -> int:
        v = self._new()
        self.desc.prims.append(Prim(SHIFT, (i,), (v,), param=int(s), shift_by=by, shift_coef=int(coef)))
        return v

    def expand(self, i: int) -> None:
        self.desc.prims.append(Prim(EXPAND, (i,), ()))

    def unfold(self, i: int, j: int) -> int:
        v = self._new()
        self.desc.prims.append(Prim(UNFOLD, (i, j), (v,)))
        return v

    def stride(self, i: int, S: int) -> int:
        v = self._new()
        self.desc.prims.append(Prim(STRIDE, (i,), (v,), param=int(S)))
        return v

    def reduce(self, N: int) -> int:
        v = self._new()
        self.desc.prims.append(Prim(REDUCE, (), (v,), param=int(N)))
        return v

    def share(self, i: int) -> Tuple[int, int]:
        a, b = self._new(), self._new()
        self.desc.prims.append(Prim(SHARE, (i,), (a, b)))
        return a, b

    def finish(self, input_coords: Sequence[int], weight_coords: Sequence[int],
               in_dtype: int = F32, out_dtype: int = F32, more_weights: Sequence[Sequence[int]] = ()) -> OpDesc:
        self.desc.input_coords = [int(c) for c in input_coords]
        self.desc.weight_coords = [int(c) for c in weight_coords]
        self.desc.more_weights = [[int(c) for c in w] for w in more_weights]
        self.desc.in_dtype = in_dtype
        self.desc.out_dtype = out_dtype
        return self.desc
