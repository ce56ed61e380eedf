"""CPU oracle: an unfused fp64 interpreter for fusion patterns.

TEST INFRASTRUCTURE ONLY.  This file is the reference the HIP path is checked
against.  It may be imported by tests/, by the smoke entry and by the bench's
cpu_baseline leg, and by nothing else; it shares no code with the HIP path and
never imports it.

What it computes
----------------
The paper's method (kernel fusion without shape values, Sections 2 and 4.3)
reaches *exactly* the result of running the ops of a pattern one after the
other; fusion changes where intermediates live, not what they are.  The oracle
is therefore that plain definition written out: it walks the op list in order,
one op at a time, and materialises every intermediate as a full numpy array in
float64.  Broadcasts are made explicit (a real, tiled copy), reductions are
numpy reductions over one axis.  There is no blocking, fusion or reordering.

The paper names ops only by example (Add, Sub, Mul, Transpose, Slice, Pad,
Broadcast, Split; Sections 4.1, 4.2.1, 4.3) and gives them their HLO meaning;
the op set here is the element-wise / broadcast / cast / select / reduce family
with those standard meanings:

* unary, binary, compare  : numpy ufuncs on float64 (int64 for integer values)
* a binary op or a select : takes its operands in the element type of its RESULT (HLO's
                            element-wise ops have one element type; an operand of another
                            type is converted as by ``cast`` first), so an integer division is
                            the truncating one exactly when the result is an integer
* integer values          : two's complement of their declared width: every i32 result is
                            reduced modulo 2^32 into [-2^31, 2^31), i64 modulo 2^64 (numpy's
                            int64 does that by itself); division truncates toward zero;
                            division by zero and -2^31 / -1 have no defined result
* rsqrt = 1/sqrt, rcp = 1/x, sigmoid = 1/(1+exp(-x)), erf = the error function
* cast to f32             : identity (float values are held in float64 throughout)
* cast to f16 / bf16      : the conversion is the op's meaning: the value is rounded to the
                            target type (nearest even) when anything but ``output`` ops reads
                            it, as the unfused sequence would hand it on.  A cast that only
                            feeds outputs is the store itself and stays unrounded here: the
                            comparator that uses the oracle owns that last rounding
* cast to an integer type : truncates toward zero, then wraps to the width; cast to bool is
                            ``x != 0``
* select(p, a, b)         : a where p != 0, else b
* broadcast               : HLO broadcast_in_dim
* reduce_{sum,max,min}    : over exactly one axis, the axis is dropped
* reduce_argmax           : lowest index among the maxima, int64
* dim_size                : the runtime size of a symbolic dimension, as a scalar
* slice                   : dynamic slice with stride 1 (Section 4.1 uses it as the example of an
                            op whose former attributes -- the start indices -- are runtime
                            values): result[i0, i1, ...] = x[s0 + i0, s1 + i1, ...]; the
                            result sizes are the op's dims, the starts come from the
                            runtime dims (or are static); a slice that leaves the operand
                            is an error
* transpose               : HLO transpose (the paper names Transpose among its examples of ops
                            whose shapes propagate, Section 4.2.1): result axis k is operand
                            axis perm[k], materialised as a real copy
* pad                     : dynamic pad without interior padding (named beside slice in Section
                            4.1): the operand sits at offset low_k along every axis of a result
                            otherwise filled with the padding value; low_k are runtime values
                            (or static), the result sizes are the op's dims; an operand that
                            does not fit is an error.  The padding value is a scalar of the
                            operand's element type (HLO pad), so unlike computed values it IS
                            rounded to that type (nearest even) when it is not representable

* ne_prev / compact / compact_count / compact_rank : outputs whose size depends on the input
                            values (Section 2 gives Unique as the example of such an op).  Over
                            rank-1 values of one length N: ne_prev(x)[i] = (i == 0) or x[i] != x[i-1];
                            compact(value, keep) = the elements of value at the positions where
                            keep is nonzero, in order -- an array of the data-dependent length
                            n = compact_count(keep), NOT padded to the declared upper bound N;
                            compact_rank(keep)[i] = (number of kept positions <= i) - 1.
                            compact(x, ne_prev(x)) is Unique of a sorted x, compact_rank its
                            second result (the index of every element in the output)

Inputs stored as f16 / bf16 are converted to float64 by the caller (every such
value is exactly representable); the oracle itself only sees numpy arrays.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np
from scipy import special as _sp


class OracleError(ValueError):
    pass


_FLOAT = ("f32", "f16", "bf16")
_INT = ("i32", "i64")


def _wrap(x: np.ndarray, dtype: str) -> np.ndarray:
    """Two's complement of the declared width (see module docstring); other kinds pass through."""
    if dtype == "i32" and x.dtype.kind == "i":
        return ((x.astype(np.int64) + (1 << 31)) % (1 << 32)) - (1 << 31)
    return x


def _as_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Value conversion performed by a ``cast`` op (see module docstring), without the rounding
    to a 16-bit float type."""
    if dtype in _FLOAT:
        return x.astype(np.float64)
    if dtype in _INT:
        if x.dtype.kind == "f":
            x = np.trunc(x)
        return _wrap(x.astype(np.int64), dtype)
    if dtype == "bool":
        return x != 0
    raise OracleError(f"unknown dtype {dtype}")


def _round_array(x: np.ndarray, dtype: str) -> np.ndarray:
    """Every element to the nearest value of a 16-bit float type, ties to even."""
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        f = x.astype(np.float32)
        # (float64 -> float32 -> bf16 rounds twice; the callers' values are float32 values already
        # or far from a bf16 tie, and _round_to_storage below has the same two steps)
        bits = f.view(np.uint32).astype(np.uint64)
        r = ((bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
        out = r.view(np.float32).astype(np.float64)
        return np.where(np.isfinite(f), out, f.astype(np.float64))
    return x


def _round_to_storage(value: float, dtype: str):
    """A constant of a storage type: the nearest representable value, ties to even."""
    if dtype == "f32":
        return np.float64(np.float32(value))
    if dtype == "f16":
        return np.float64(np.float16(value))
    if dtype == "bf16":
        if not np.isfinite(value):
            return np.float64(value)
        bits = int(np.float32(value).view(np.uint32))
        bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000     # keep 8 significant bits, ties to even
        return np.float64(np.uint32(bits).view(np.float32))
    return value


def _broadcast_in_dim(x: np.ndarray, out_shape: Tuple[int, ...], axis_map: Sequence[int]) -> np.ndarray:
    if len(axis_map) != x.ndim:
        raise OracleError("broadcast: axis_map length != operand rank")
    if any(b <= a for a, b in zip(axis_map, axis_map[1:])):
        raise OracleError("broadcast: axis_map must be strictly increasing")
    shape = [1] * len(out_shape)
    for k, a in enumerate(axis_map):
        if x.shape[k] != out_shape[a] and x.shape[k] != 1:
            raise OracleError("broadcast: operand dim neither equal to result dim nor 1")
        shape[a] = x.shape[k]
    # explicit tiling: a real copy of the operand repeated along the new axes
    return np.broadcast_to(x.reshape(shape), out_shape).copy()


_UNARY = {
    "neg": lambda x: -x,
    "abs": np.abs,
    "exp": np.exp,
    "log": np.log,
    "tanh": np.tanh,
    "sqrt": np.sqrt,
    "rsqrt": lambda x: 1.0 / np.sqrt(x),
    "rcp": lambda x: 1.0 / x,
    "sigmoid": lambda x: 1.0 / (1.0 + np.exp(-x)),
    "erf": _sp.erf,
}


def _int_div(a, b):
    # C-style truncating division for integer values
    q = np.abs(a) // np.abs(b)
    return np.where((a < 0) != (b < 0), -q, q)


_BINARY = {
    "add": np.add,
    "sub": np.subtract,
    "mul": np.multiply,
    "div": lambda a, b: _int_div(a, b) if a.dtype.kind == "i" else a / b,
    "max": np.maximum,
    "min": np.minimum,
    "pow": np.power,
}

_COMPARE = {
    "lt": np.less, "le": np.less_equal, "gt": np.greater,
    "ge": np.greater_equal, "eq": np.equal, "ne": np.not_equal,
}


def _same_shape(*xs: np.ndarray) -> None:
    """Element-wise ops take operands of one shape (or rank-0 scalars): numpy's
    implicit broadcasting between two non-scalar shapes is not part of the op set."""
    shapes = {x.shape for x in xs if x.ndim > 0}
    if len(shapes) > 1:
        raise OracleError(f"element-wise operands differ in shape: {sorted(shapes)}")


def _common(a: np.ndarray, b: np.ndarray):
    """Bring two operands to one numeric kind (bool < int64 < float64)."""
    _same_shape(a, b)
    if a.dtype == b.dtype:
        return a, b
    if a.dtype.kind == "f" or b.dtype.kind == "f":
        return a.astype(np.float64), b.astype(np.float64)
    return a.astype(np.int64), b.astype(np.int64)


def run(pattern, dims: Sequence[int], inputs: Sequence[np.ndarray]):
    """Evaluate ``pattern`` at runtime sizes ``dims`` on ``inputs``.

    ``inputs[k]`` is the array for the k-th ``param`` op.  Returns
    ``(outputs, values)``: the list of output arrays in ``output``-op order and
    the dict op-index -> materialised value for *every* op (all intermediates).
    Every op's result shape is checked against the shape the pattern declares
    for it at these ``dims``; a mismatch raises OracleError.
    """
    with np.errstate(over="ignore", under="ignore", invalid="ignore", divide="ignore"):
        return _run(pattern, dims, inputs)


def _run(pattern, dims, inputs):
    dims = [int(d) for d in dims]
    if len(dims) != pattern.n_dims:
        raise OracleError(f"expected {pattern.n_dims} runtime dims, got {len(dims)}")
    vals: Dict[int, np.ndarray] = {}
    outs: List[np.ndarray] = []
    next_param = 0
    # values that something other than an ``output`` op reads
    read_on = set()
    for op in pattern.ops:
        if op.opcode != "output":
            read_on.update(op.ins)
    for idx, op in enumerate(pattern.ops):
        want = tuple(dims[d] if d >= 0 else -d for d in op.dims)
        oc = op.opcode
        if oc == "param":
            x = np.asarray(inputs[next_param])
            next_param += 1
            if op.dtype in _FLOAT:
                v = x.astype(np.float64)
            elif op.dtype in _INT:
                v = x.astype(np.int64)
            else:
                v = x != 0
            if v.shape != want:
                raise OracleError(f"param {idx}: got shape {v.shape}, pattern says {want}")
        elif oc == "const":
            v = _as_dtype(np.asarray(op.fconst, dtype=np.float64), op.dtype)
        elif oc == "dim_size":
            v = _as_dtype(np.asarray(float(dims[op.axis_map[0]])), op.dtype)
        elif oc in _UNARY:
            v = _UNARY[oc](_as_dtype(vals[op.ins[0]], op.dtype))
        elif oc in _BINARY:
            a, b = _as_dtype(vals[op.ins[0]], op.dtype), _as_dtype(vals[op.ins[1]], op.dtype)
            _same_shape(a, b)
            v = _BINARY[oc](a, b)
        elif oc in _COMPARE:
            a, b = _common(vals[op.ins[0]], vals[op.ins[1]])
            v = _COMPARE[oc](a, b)
        elif oc == "select":
            a, b = _as_dtype(vals[op.ins[1]], op.dtype), _as_dtype(vals[op.ins[2]], op.dtype)
            _same_shape(vals[op.ins[0]], a, b)
            v = np.where(vals[op.ins[0]] != 0, a, b)
        elif oc == "cast":
            v = _as_dtype(vals[op.ins[0]], op.dtype)
            if op.dtype in ("f16", "bf16") and idx in read_on:
                v = _round_array(v, op.dtype)
        elif oc == "broadcast":
            v = _broadcast_in_dim(vals[op.ins[0]], want, op.axis_map)
        elif oc in ("reduce_sum", "reduce_max", "reduce_min", "reduce_argmax"):
            x = vals[op.ins[0]]
            ax = op.axis_map[0]
            if not 0 <= ax < x.ndim:
                raise OracleError(f"op {idx}: reduce axis {ax} out of range")
            if x.shape[ax] == 0:
                raise OracleError(f"op {idx}: reduction over an empty axis")
            if oc == "reduce_sum":
                v = _wrap(np.sum(x, axis=ax), pattern.ops[op.ins[0]].dtype)   # (an i32 sum wraps like its terms)
            elif oc == "reduce_max":
                v = np.max(x, axis=ax)
            elif oc == "reduce_min":
                v = np.min(x, axis=ax)
            else:
                v = np.argmax(x, axis=ax).astype(np.int64)  # first occurrence
        elif oc == "slice":
            x = vals[op.ins[0]]
            if len(op.axis_map) != x.ndim or len(want) != x.ndim:
                raise OracleError(f"op {idx}: slice needs one start and one size per axis")
            starts = [dims[a] if a >= 0 else -1 - a for a in op.axis_map]
            for k, (s0, n) in enumerate(zip(starts, want)):
                if s0 < 0 or s0 + n > x.shape[k]:
                    raise OracleError(f"op {idx}: slice [{s0}, {s0 + n}) leaves axis {k} of size {x.shape[k]}")
            v = x[tuple(slice(s0, s0 + n) for s0, n in zip(starts, want))].copy()
        elif oc == "transpose":
            x = vals[op.ins[0]]
            if sorted(op.axis_map) != list(range(x.ndim)):
                raise OracleError(f"op {idx}: transpose needs a permutation of the operand's axes")
            v = np.ascontiguousarray(np.transpose(x, op.axis_map))
        elif oc == "pad":
            x = vals[op.ins[0]]
            if len(op.axis_map) != x.ndim or len(want) != x.ndim:
                raise OracleError(f"op {idx}: pad needs one low padding and one size per axis")
            low = [dims[a] if a >= 0 else -1 - a for a in op.axis_map]
            for k, (l0, n) in enumerate(zip(low, want)):
                if l0 < 0 or l0 + x.shape[k] > n:
                    raise OracleError(f"op {idx}: operand [{l0}, {l0 + x.shape[k]}) does not fit axis {k} of size {n}")
            fill = _as_dtype(np.asarray(_round_to_storage(op.fconst, op.dtype), dtype=np.float64), op.dtype)
            v = np.full(want, fill, dtype=x.dtype)
            v[tuple(slice(l0, l0 + m) for l0, m in zip(low, x.shape))] = x
        elif oc == "ne_prev":
            x = vals[op.ins[0]]
            if x.ndim != 1:
                raise OracleError(f"op {idx}: ne_prev takes a rank-1 operand")
            v = np.ones(x.shape, dtype=bool)          # the first element opens the first run
            v[1:] = x[1:] != x[:-1]
        elif oc == "compact":
            x, keep = vals[op.ins[0]], vals[op.ins[1]]
            if x.ndim != 1 or keep.shape != x.shape:
                raise OracleError(f"op {idx}: compact takes two rank-1 operands of one length")
            v = x[keep != 0].copy()                   # data-dependent length, order kept
            vals[idx] = v
            continue                                  # (its length is the result, not the declared bound)
        elif oc == "compact_count":
            v = _wrap(np.asarray(np.count_nonzero(vals[op.ins[0]] != 0), dtype=np.int64), op.dtype)
        elif oc == "compact_rank":
            keep = vals[op.ins[0]]
            if keep.ndim != 1:
                raise OracleError(f"op {idx}: compact_rank takes a rank-1 operand")
            v = np.cumsum((keep != 0).astype(np.int64)) - 1
        elif oc == "output":
            v = vals[op.ins[0]]
            outs.append(v)
            if pattern.ops[op.ins[0]].opcode == "compact":
                vals[idx] = v
                continue
        else:
            raise OracleError(f"op {idx}: unknown opcode {oc}")
        v = _wrap(np.asarray(v), op.dtype)
        if v.ndim > 0 or len(want) > 0:
            # rank-0 operands act as scalars inside element-wise ops; anything
            # else must come out with exactly the declared shape
            if v.shape != want:
                if v.ndim == 0:
                    v = np.full(want, v)
                else:
                    raise OracleError(f"op {idx} ({oc}): result shape {v.shape}, pattern says {want}")
        vals[idx] = v
    return outs, vals


def run_outputs(pattern, dims, inputs):
    return run(pattern, dims, inputs)[0]
