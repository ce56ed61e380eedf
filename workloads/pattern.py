"""Neutral description of a fusion pattern: an op sequence WITHOUT shape values.

A fusion pattern in the paper's sense (Section 2: kernels are generated for shapes
that are not known yet, so the identity of a pattern does not include the shape
values) is an ordered op list whose tensor dimensions are *symbolic*.
Static rank only (same passage).  Shape constraints of the two kinds the paper
names (Section 4.2.1: dimension-size equality, tensor-size equality) may be
attached by the caller, which plays the role of the framework bridging layer.

Conventions
-----------
* A value is identified by the index of the op that produces it.
* ``dims[i] >= 0``  : symbolic dimension id (its size is given at launch time).
  ``dims[i] < 0``   : static size ``-dims[i]``.
* ``broadcast``     : HLO broadcast_in_dim; ``axis_map[k]`` is the result axis
  that operand axis ``k`` maps to (strictly increasing).  An operand axis of
  static size 1 may be expanded.
* ``reduce_*``      : reduces exactly one axis, ``axis_map[0]``; the result drops it.
* ``dim_size``      : rank-0 scalar holding the runtime size of symbolic dim
  ``axis_map[0]``.
* rank-0 values (``const``, ``dim_size``) may be used directly as operands of
  element-wise ops (scalar operand).
* ``output``        : marks value ``ins[0]`` as a result of the pattern.
* ``slice``         : dynamic slice (the paper's DHLO example, Section 4.1: the start indices
  of a slice are runtime values, not compile-time attributes).  ``dims`` are the
  sizes of the result, ``axis_map[k]`` the start along axis ``k``: ``>= 0`` the
  id of a symbolic dim whose runtime value is the start index, ``< 0`` the
  static start ``-1 - axis_map[k]`` (so ``-1`` is start 0).  Stride 1.
* ``pad``           : dynamic pad (Section 4.1 names it beside slice): ``dims`` are the sizes
  of the result, ``axis_map[k]`` the number of padding elements in front of
  axis ``k`` (encoded like a slice start), ``fconst`` the padding value; the
  padding behind an axis is whatever the result size leaves.  No interior
  padding, no negative padding.
* ``transpose``     : HLO transpose: result axis ``k`` is operand axis ``axis_map[k]``
  (``axis_map`` is a permutation).
* ``ne_prev`` / ``compact`` / ``compact_count`` / ``compact_rank`` : outputs whose size depends
  on the input values (Section 2 names Unique as that kind of op), over rank-1 values of one
  length N.  ``ne_prev(x)[i] = (i == 0) or x[i] != x[i-1]``; ``compact(value, keep)`` keeps the
  elements of ``value`` where ``keep`` is nonzero, in order (its declared dim is the upper bound
  N; ``compact_count(keep)`` of them are defined); ``compact_rank(keep)[i]`` = number of kept
  positions ``<= i``, minus one.  ``compact(x, ne_prev(x))`` with the rank is Unique of a sorted x.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

DTYPES = ("f32", "f16", "bf16", "i32", "i64", "bool")

LEAF = ("param", "const", "dim_size")
UNARY = ("neg", "abs", "exp", "log", "tanh", "sqrt", "rsqrt", "rcp", "sigmoid", "erf")
BINARY = ("add", "sub", "mul", "div", "max", "min", "pow")
COMPARE = ("lt", "le", "gt", "ge", "eq", "ne")
REDUCE = ("reduce_sum", "reduce_max", "reduce_min", "reduce_argmax")
COMPACTION = ("ne_prev", "compact", "compact_count", "compact_rank")
OPCODES = (LEAF + UNARY + BINARY + COMPARE + ("select", "cast", "broadcast") + REDUCE + ("output", "slice", "pad", "transpose")
           + COMPACTION)

DIM_EQ = 0      # dimension-size equality constraint
NUMEL_EQ = 1    # tensor-size equality constraint


@dataclass(frozen=True)
class Op:
    opcode: str
    dtype: str
    ins: Tuple[int, ...] = ()
    dims: Tuple[int, ...] = ()
    axis_map: Tuple[int, ...] = ()
    fconst: float = 0.0


@dataclass
class Pattern:
    ops: List[Op] = field(default_factory=list)
    # (kind, a_value, a_axis, b_value, b_axis); axes ignored for NUMEL_EQ
    constraints: List[Tuple[int, int, int, int, int]] = field(default_factory=list)
    n_dims: int = 0            # number of symbolic dimensions
    name: str = ""

    @property
    def params(self) -> List[int]:
        return [i for i, o in enumerate(self.ops) if o.opcode == "param"]

    @property
    def outputs(self) -> List[int]:
        """Indices of the ``output`` ops, in order."""
        return [i for i, o in enumerate(self.ops) if o.opcode == "output"]

    def shape_of(self, value: int, dims: Sequence[int]) -> Tuple[int, ...]:
        return tuple(int(dims[d]) if d >= 0 else -d for d in self.ops[value].dims)


class PatternBuilder:
    """Small convenience layer to write op lists by hand.

    It only copies dimension *names* around (an element-wise result is given
    the names of its first non-scalar operand unless ``dims`` is passed); it
    checks nothing and computes nothing.
    """

    def __init__(self, name: str = ""):
        self.p = Pattern(name=name)

    # -- symbolic dims ---------------------------------------------------
    def dim(self) -> int:
        d = self.p.n_dims
        self.p.n_dims += 1
        return d

    def dims(self, n: int) -> List[int]:
        return [self.dim() for _ in range(n)]

    @staticmethod
    def static(size: int) -> int:
        assert size > 0
        return -int(size)

    # -- ops ---------------------------------------------------------------
    def _push(self, op: Op) -> int:
        for d in op.dims:
            if d >= 0:
                self.p.n_dims = max(self.p.n_dims, d + 1)
        self.p.ops.append(op)
        return len(self.p.ops) - 1

    def param(self, dtype: str, dims: Sequence[int]) -> int:
        return self._push(Op("param", dtype, (), tuple(dims)))

    def const(self, value: float, dtype: str = "f32") -> int:
        return self._push(Op("const", dtype, (), (), (), float(value)))

    def dim_size(self, dim_id: int, dtype: str = "f32") -> int:
        return self._push(Op("dim_size", dtype, (), (), (int(dim_id),)))

    def _ew_dims(self, ins, dims):
        if dims is not None:
            return tuple(dims)
        for i in ins:
            if len(self.p.ops[i].dims) > 0:
                return self.p.ops[i].dims
        return ()

    def op(self, opcode: str, *ins: int, dtype: str | None = None, dims=None) -> int:
        assert opcode in UNARY + BINARY + COMPARE + ("select",), opcode
        if dtype is None:
            if opcode in COMPARE:
                dtype = "bool"
            elif opcode == "select":
                dtype = self.p.ops[ins[1]].dtype
            else:
                dtype = self.p.ops[ins[0]].dtype
        return self._push(Op(opcode, dtype, tuple(ins), self._ew_dims(ins, dims)))

    def cast(self, v: int, dtype: str) -> int:
        return self._push(Op("cast", dtype, (v,), self.p.ops[v].dims))

    def broadcast(self, v: int, dims: Sequence[int], axis_map: Sequence[int]) -> int:
        return self._push(Op("broadcast", self.p.ops[v].dtype, (v,), tuple(dims), tuple(axis_map)))

    def reduce(self, kind: str, v: int, axis: int, dtype: str | None = None) -> int:
        opcode = "reduce_" + kind
        assert opcode in REDUCE
        src = self.p.ops[v]
        if dtype is None:
            dtype = "i32" if kind == "argmax" else src.dtype
        dims = tuple(d for k, d in enumerate(src.dims) if k != axis)
        return self._push(Op(opcode, dtype, (v,), dims, (int(axis),)))

    @staticmethod
    def static_start(start: int) -> int:
        """Encoding of a compile-time start index of ``slice``."""
        assert start >= 0
        return -1 - int(start)

    def slice(self, v: int, starts: Sequence[int], sizes: Sequence[int]) -> int:
        """result[i0, i1, ...] = v[start0 + i0, start1 + i1, ...]; ``sizes`` are the result dims."""
        src = self.p.ops[v]
        assert len(starts) == len(sizes) == len(src.dims)
        for s_ in starts:
            if s_ >= 0:
                self.p.n_dims = max(self.p.n_dims, s_ + 1)
        return self._push(Op("slice", src.dtype, (v,), tuple(sizes), tuple(int(x) for x in starts)))

    def transpose(self, v: int, perm: Sequence[int]) -> int:
        """result axis k = operand axis perm[k]."""
        src = self.p.ops[v]
        assert sorted(perm) == list(range(len(src.dims)))
        return self._push(Op("transpose", src.dtype, (v,), tuple(src.dims[a] for a in perm), tuple(int(a) for a in perm)))

    def pad(self, v: int, low: Sequence[int], sizes: Sequence[int], value: float = 0.0) -> int:
        """result[i] = v[i - low] where that exists, ``value`` elsewhere; ``sizes`` are the result dims."""
        src = self.p.ops[v]
        assert len(low) == len(sizes) == len(src.dims)
        for s_ in low:
            if s_ >= 0:
                self.p.n_dims = max(self.p.n_dims, s_ + 1)
        return self._push(Op("pad", src.dtype, (v,), tuple(sizes), tuple(int(x) for x in low), float(value)))

    def ne_prev(self, v: int) -> int:
        src = self.p.ops[v]
        return self._push(Op("ne_prev", "bool", (v,), src.dims))

    def compact(self, value: int, keep: int) -> int:
        src = self.p.ops[value]
        return self._push(Op("compact", src.dtype, (value, keep), src.dims))

    def compact_count(self, keep: int, dtype: str = "i32") -> int:
        return self._push(Op("compact_count", dtype, (keep,), ()))

    def compact_rank(self, keep: int, dtype: str = "i32") -> int:
        return self._push(Op("compact_rank", dtype, (keep,), self.p.ops[keep].dims))

    def output(self, v: int) -> int:
        src = self.p.ops[v]
        return self._push(Op("output", src.dtype, (v,), src.dims))

    # -- constraints ---------------------------------------------------------
    def dim_eq(self, a_value: int, a_axis: int, b_value: int, b_axis: int) -> None:
        self.p.constraints.append((DIM_EQ, a_value, a_axis, b_value, b_axis))

    def numel_eq(self, a_value: int, b_value: int) -> None:
        self.p.constraints.append((NUMEL_EQ, a_value, 0, b_value, 0))

    def build(self) -> Pattern:
        return self.p
