"""Seeded random fusion patterns against the oracle: element-wise DAGs over rank-2 / rank-3 spaces
with row vectors, per-row operands, scalars, masks, windows (dynamic slices) of larger inputs,
padded smaller inputs and mixed storage types; no reduction (loop
fusion), one or two dependent row reductions with an epilogue, or a column reduction with an
epilogue; most of the rank-2 loop and row patterns also emit a sum over the rows, and row
patterns rank-0 reductions of their per-row results, which ride along in the row kernels.  Every pattern is compiled once and launched at several shapes (ragged
and aligned).

The generator keeps the arithmetic well conditioned, so the element-wise parity bar applies:
reduced terms are non-negative (sums) or the reduction is exact (max / min), values stay O(1), and
nothing is subtracted from a sum of mixed signs.
"""
import numpy as np
import pytest
import torch

from oracle import run as oracle_run
from workloads import PatternBuilder
from workloads.configs import TORCH_DTYPE
from tests.util import assert_close, run_gpu, to_oracle_input

pytestmark = pytest.mark.gpu

FLOATS = ("f32", "f16", "bf16")
UNARY_SAFE = ("neg", "abs", "tanh", "sigmoid")       # bounded or sign-only: inputs stay O(1)
BINARY_SAFE = ("add", "mul", "max", "min", "sub")


@pytest.fixture(scope="module")
def ctx():
    from paper_2103_05288_amd import Context
    c = Context(0)
    yield c
    c.close()


class Gen:
    """Builds one random pattern; remembers how to draw its inputs."""

    def __init__(self, seed):
        self.rng = np.random.default_rng(seed)
        self.pb = PatternBuilder("random%d" % seed)
        self.rank = int(self.rng.integers(2, 4))
        self.dims = self.pb.dims(self.rank)
        self.full = list(self.dims)
        self.inputs = []          # (kind, dtype, dims)
        self.extra = []           # windows / pads: the symbolic dims that need runtime values of their own
        self.kind = ["loop", "row", "row2", "col"][int(self.rng.integers(0, 4))]
        # a sum over the rows beside the loop fusion / the row reductions (drawn from a generator of
        # its own, so that the rest of the pattern does not depend on it)
        self.side_sum = self.rank == 2 and self.kind != "col" and np.random.default_rng(5000 + seed).random() < 0.7
        # rank-0 outputs: per-row reduction results reduced once more over the rows
        self.scalar_out = self.rank == 2 and self.kind in ("row", "row2") and np.random.default_rng(7000 + seed).random() < 0.7

    def pick(self, seq):
        return seq[int(self.rng.integers(0, len(seq)))]

    def f32(self, v):
        return v if self.pb.p.ops[v].dtype == "f32" else self.pb.cast(v, "f32")

    def leaf(self):
        """A full-shaped fp32 value from a fresh or broadcast operand."""
        pb, full, rank = self.pb, self.full, self.rank
        what = self.pick(["full", "full", "rowvec", "perrow", "const", "window", "padded"])
        if what == "full":
            dt = self.pick(FLOATS)
            v = pb.param(dt, full)
            self.inputs.append(("normal", dt, full))
            return self.f32(v)
        if what == "rowvec":                      # varies along the innermost axis only
            dt = self.pick(FLOATS)
            v = pb.param(dt, [full[-1]])
            self.inputs.append(("normal", dt, [full[-1]]))
            return pb.broadcast(self.f32(v), full, [rank - 1])
        if what == "perrow":                      # constant along the innermost axis
            v = pb.param("f32", full[:-1])
            self.inputs.append(("normal", "f32", full[:-1]))
            return pb.broadcast(v, full, list(range(rank - 1)))
        if what in ("window", "padded"):
            # an input with extents of its own along the last two axes; the full shape is a window
            # of it at a runtime offset (slice) or it sits inside the full shape at a runtime
            # offset, the rest being a constant (pad)
            dt = self.pick(FLOATS)
            own = list(full)
            starts = [pb.static_start(0)] * rank
            spec = {"kind": what, "axes": []}
            for ax in (rank - 2, rank - 1):
                if self.rng.random() < 0.7:
                    own[ax] = pb.dim()
                    starts[ax] = pb.dim()
                    spec["axes"].append((ax, own[ax], starts[ax]))
            if not spec["axes"]:
                own[rank - 1] = pb.dim()
                starts[rank - 1] = pb.dim()
                spec["axes"].append((rank - 1, own[rank - 1], starts[rank - 1]))
            v = pb.param(dt, own)
            self.inputs.append(("normal", dt, own))
            self.extra.append(spec)
            if what == "window":
                return self.f32(pb.slice(v, starts, full))
            return self.f32(pb.pad(v, starts, full, float(self.rng.uniform(-1.0, 1.0))))
        c = pb.const(float(self.rng.uniform(-1.5, 1.5)))
        return pb.op("add", self.leaf_full(), c)

    def leaf_full(self):
        v = self.pb.param("f32", self.full)
        self.inputs.append(("normal", "f32", self.full))
        return v

    def chain(self, v, n):
        pb = self.pb
        for _ in range(n):
            if self.rng.random() < 0.45:
                v = pb.op(self.pick(UNARY_SAFE), v)
            else:
                w = self.leaf()
                op = self.pick(BINARY_SAFE)
                v = pb.op(op, v, w) if self.rng.random() < 0.5 else pb.op(op, w, v)
            if self.rng.random() < 0.2:           # a masked select
                m = pb.param("bool", self.full)
                self.inputs.append(("mask", "bool", self.full))
                v = pb.op("select", m, self.leaf(), v, dims=self.full)
        return v

    def build(self):
        pb, full, rank = self.pb, self.full, self.rank
        v = self.chain(self.leaf_full(), int(self.rng.integers(1, 5)))
        if self.kind == "loop":
            pb.output(pb.cast(v, self.pick(FLOATS)))
            if self.rng.random() < 0.4:
                pb.output(pb.op("gt", v, pb.const(0.25), dims=full))
            if self.side_sum:
                pb.output(pb.reduce("sum", pb.op("sigmoid", v), 0))
        elif self.kind in ("row", "row2"):
            axis = rank - 1
            back = list(range(rank - 1))
            m = pb.reduce("max", v, axis)
            e = pb.op("exp", pb.op("sub", v, pb.broadcast(m, full, back)))            # in (0, 1]
            s = pb.reduce("sum", e, axis)
            y = pb.op("div", e, pb.broadcast(s, full, back))
            if self.kind == "row2":
                t = pb.reduce("max", pb.op("mul", y, pb.op("sigmoid", self.leaf())), axis)   # third phase
                y = pb.op("add", y, pb.broadcast(t, full, back))
                pb.output(t)
            y = self.chain(y, int(self.rng.integers(0, 3)))
            pb.output(pb.cast(y, self.pick(FLOATS)))
            if self.rng.random() < 0.5:
                pb.output(s)
            if self.side_sum:
                pb.output(pb.reduce("sum", pb.op("sigmoid", y), 0))      # non-negative terms
            if self.scalar_out:
                pb.output(pb.reduce("sum", s, 0))                        # positive terms
                pb.output(pb.reduce("min", m, 0))
        else:
            axis = rank - 2
            keep = [k for k in range(rank) if k != axis]
            kind = self.pick(["sum", "max", "min"])
            src = pb.op("sigmoid", v) if kind == "sum" else v
            r = pb.reduce(kind, src, axis)
            pb.output(r)
            if self.rng.random() < 0.7:
                y = pb.op("mul", v, pb.op("tanh", pb.broadcast(r, full, keep)))
                pb.output(pb.cast(y, self.pick(FLOATS)))
        return pb.build()

    def draw(self, dims, seed):
        g = torch.Generator().manual_seed(seed)
        out = []
        for kind, dt, sym in self.inputs:
            shape = [int(dims[d]) for d in sym]
            if kind == "mask":
                out.append((torch.rand(shape, generator=g) < 0.3).to(torch.uint8))
            else:
                out.append(torch.randn(shape, generator=g).to(TORCH_DTYPE[dt]))
        return out


def complete_dims(gen, pat, base, rng):
    """Runtime values for the extents and offsets of windowed / padded inputs, given the base shape."""
    dims = list(base) + [0] * (pat.n_dims - len(base))
    for spec in gen.extra:
        for ax, own, start in spec["axes"]:
            n = int(dims[gen.full[ax]])
            if spec["kind"] == "window":          # the input is larger: own = start + n + slack
                st = int(rng.integers(0, 9))
                dims[start] = st
                dims[own] = st + n + int(rng.integers(0, 9))
            else:                                  # the input is smaller: start + own <= n
                o = int(rng.integers(0, n + 1))
                dims[own] = o
                dims[start] = int(rng.integers(0, n - o + 1))
    return dims


def shapes_for(gen, rng):
    inner = [1, 7, 8, 33, 127, 200, 513, 1000, 1025, 2047, 3001, 4099]
    res = []
    for _ in range(3):
        h = int(inner[int(rng.integers(0, len(inner)))])
        t = int(rng.integers(1, 70))
        res.append([t, h] if gen.rank == 2 else [int(rng.integers(1, 5)), t, h])
    if gen.kind == "col":                      # one tall shape: chunks of the reduced axis, three launches
        res.append([3000, 520] if gen.rank == 2 else [2, 2500, 130])
    if gen.side_sum or gen.scalar_out:         # many rows per block, several blocks
        res.append([2500, 130])
    return res


@pytest.mark.parametrize("seed", list(range(40)))
def test_random_pattern(ctx, seed):
    gen = Gen(seed)
    pat = gen.build()
    h = ctx.register(pat)
    want_tmpl = {"loop": "loop", "row": "row_reduce", "row2": "row_reduce", "col": "col_reduce"}[gen.kind]
    if gen.side_sum:
        want_tmpl = "row_reduce"               # also for a loop fusion: the row template without reduction phases
    assert h.info["template"] == want_tmpl, (seed, gen.kind, h.info["template"])
    rng = np.random.default_rng(1000 + seed)
    for base in shapes_for(gen, rng):
        dims = complete_dims(gen, pat, base, rng)
        ins = gen.draw(dims, seed=seed * 7 + len(dims))
        got = run_gpu(h, pat, dims, ins)
        want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
        for k, (g, w) in enumerate(zip(got, want)):
            if not g.dtype.is_floating_point:      # comparison outputs: only where the value is clear of the threshold
                continue
            assert_close(g, w, f"seed {seed} ({gen.kind}, rank {gen.rank}) dims={dims} out{k} variant={h.plan(dims)['variant_name']}")
    assert h.info["compile_events"] == 1
