"""Seeded random op graphs against the oracle: element-wise chains over a [T, H] space interleaved
with row reductions (results broadcast back along rows), column reductions (broadcast back along
columns) and fresh inputs, several outputs.  Most of them are not one fusion pattern: the graph
path has to cut them, plan buffers for what crosses the cuts and still produce what the uncut op
list defines.  Values stay O(1) (bounded functions, means instead of sums), so the element-wise
parity bar applies."""
import numpy as np
import pytest
import torch

from oracle import run as oracle_run
from workloads import PatternBuilder
from workloads.configs import TORCH_DTYPE
from tests.util import assert_close, to_oracle_input

pytestmark = pytest.mark.gpu

BOUNDED = ("tanh", "sigmoid")
BINARY = ("add", "mul", "max", "min", "sub")


class GraphGen:
    def __init__(self, seed):
        self.rng = np.random.default_rng(seed)
        self.pb = PatternBuilder("random_graph%d" % seed)
        self.T, self.H = self.pb.dims(2)
        self.full = [self.T, self.H]
        self.inputs = []            # (dtype, dims)
        self.windows = []           # (extent dim, start dim) of windowed inputs

    def pick(self, seq):
        return seq[int(self.rng.integers(0, len(seq)))]

    def fresh(self):
        pb = self.pb
        kind = self.pick(["full", "full", "row", "col", "transposed", "window"])
        dt = self.pick(["f32", "bf16", "f16"])
        if kind == "full":
            v = pb.param(dt, self.full)
            self.inputs.append((dt, self.full))
            return pb.cast(v, "f32") if dt != "f32" else v
        if kind == "transposed":    # stored as [H, T]: the transpose moves the innermost axis, a kernel of its own
            v = pb.param(dt, [self.H, self.T])
            self.inputs.append((dt, [self.H, self.T]))
            v = pb.transpose(v, (1, 0))
            return pb.cast(v, "f32") if dt != "f32" else v
        if kind == "window":        # a window of a wider input at a runtime offset
            W, s0 = pb.dim(), pb.dim()
            self.windows.append((W, s0))
            v = pb.param(dt, [self.T, W])
            self.inputs.append((dt, [self.T, W]))
            v = pb.slice(v, [pb.static_start(0), s0], self.full)
            return pb.cast(v, "f32") if dt != "f32" else v
        if kind == "col":           # a row vector: one value per column
            v = pb.param("f32", [self.H])
            self.inputs.append(("f32", [self.H]))
            return pb.broadcast(v, self.full, [1])
        v = pb.param("f32", [self.T])
        self.inputs.append(("f32", [self.T]))
        return pb.broadcast(v, self.full, [0])

    def build(self):
        pb, rng = self.pb, self.rng
        live = [self.fresh()]        # full-shaped fp32 values that later ops may use
        n_out = 0
        for _ in range(int(rng.integers(6, 16))):
            what = self.pick(["unary", "binary", "binary", "rowred", "rowred", "colred", "colred", "fresh"])
            a = self.pick(live)
            if what == "unary":
                v = pb.op(self.pick(BOUNDED), a)
            elif what == "binary":
                b = self.pick(live) if rng.random() < 0.5 else self.fresh()
                v = pb.op(self.pick(BINARY), a, b)
                if rng.random() < 0.5:
                    v = pb.op("tanh", v)                  # keep magnitudes bounded along long chains
            elif what == "fresh":
                v = self.fresh()
            else:
                axis = 1 if what == "rowred" else 0
                kind = self.pick(["mean", "max"])
                src = pb.op("sigmoid", a)
                r = pb.reduce("sum" if kind == "mean" else "max", src, axis)
                if kind == "mean":
                    r = pb.op("div", r, pb.dim_size(self.H if axis == 1 else self.T))
                if rng.random() < 0.3 and n_out < 3:
                    pb.output(r)
                    n_out += 1
                v = pb.op("sub", a, pb.broadcast(r, self.full, [0] if axis == 1 else [1]))
            live.append(v)
            if rng.random() < 0.2 and n_out < 3:
                pb.output(pb.cast(v, self.pick(["f32", "bf16"])))
                n_out += 1
        pb.output(pb.cast(live[-1], self.pick(["f32", "bf16", "f16"])))
        return pb.build()

    def draw(self, dims, seed):
        g = torch.Generator().manual_seed(seed)
        return [torch.randn([int(dims[d]) for d in sym], generator=g).to(TORCH_DTYPE[dt]) for dt, sym in self.inputs]


@pytest.fixture(scope="module")
def ctx():
    from paper_2103_05288_amd import Context
    c = Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_graph(ctx, seed):
    gen = GraphGen(seed)
    pat = gen.build()
    pat = dedupe_outputs(pat)        # an output named twice is not allowed by the graph ABI
    g = ctx.register_graph(pat)
    info = g.info
    assert 1 <= info["n_patterns"] <= 64 and info["n_buffers"] <= info["n_intermediates"]
    rng = np.random.default_rng(500 + seed)
    for base in ([int(rng.integers(1, 40)), int(rng.integers(1, 200))], [int(rng.integers(100, 700)), 513], [37, 4099]):
        dims = list(base) + [0] * (pat.n_dims - 2)
        for W, s0 in gen.windows:
            dims[s0] = int(rng.integers(0, 9))
            dims[W] = dims[s0] + base[1] + int(rng.integers(0, 9))
        ins = gen.draw(dims, seed=seed * 11 + dims[1])
        outs = [torch.full(pat.shape_of(o, dims), float("nan"), dtype=TORCH_DTYPE[pat.ops[o].dtype], device="cuda") for o in pat.outputs]
        ws = torch.empty(max(16, g.workspace_bytes(dims)), dtype=torch.uint8, device="cuda")
        g.launch(dims, [t.cuda() for t in ins], outs, workspace=ws)
        torch.cuda.synchronize()
        want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
        for k, (o, w) in enumerate(zip(outs, want)):
            assert_close(o.cpu(), w, f"graph seed {seed} dims={dims} out{k} patterns={info['n_patterns']} buffers={info['n_buffers']}")


def dedupe_outputs(pat):
    """The same op list without `output` ops that name a value already output (the generator may
    draw one twice); later ops are renumbered."""
    from workloads.pattern import Op, Pattern
    seen, remap, new_ops = set(), {}, []
    for i, o in enumerate(pat.ops):
        if o.opcode == "output":
            if o.ins[0] in seen:
                continue
            seen.add(o.ins[0])
        remap[i] = len(new_ops)
        new_ops.append(Op(o.opcode, o.dtype, tuple(remap[x] for x in o.ins), o.dims, o.axis_map, o.fconst))
    return Pattern(ops=new_ops, constraints=list(pat.constraints), n_dims=pat.n_dims, name=pat.name)
