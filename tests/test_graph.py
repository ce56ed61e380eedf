"""Op graphs larger than one fusion pattern: the cut into patterns and the buffer plan on the host
(no GPU), and parity of the whole graph with the oracle on the GPU."""
import numpy as np
import pytest
import torch

from workloads import PatternBuilder
from workloads.extras import layernorm_backward_graph
from workloads.configs import TORCH_DTYPE


def block_graph(p_is_output=True):
    """bias + tanh -> residual -> LayerNorm * gamma -> row softmax -> column mean -> centred."""
    pb = PatternBuilder("block")
    T, H = pb.dims(2)
    x = pb.param("bf16", [T, H]); b = pb.param("f32", [H]); r = pb.param("bf16", [T, H]); gam = pb.param("f32", [H])
    row = lambda v: pb.broadcast(v, [T, H], [0])
    col = lambda v: pb.broadcast(v, [T, H], [1])
    h = pb.op("tanh", pb.op("add", pb.cast(x, "f32"), col(b)))
    v = pb.op("add", h, pb.cast(r, "f32"))
    mean = pb.op("div", pb.reduce("sum", v, 1), pb.dim_size(H))
    d = pb.op("sub", v, row(mean))
    var = pb.op("div", pb.reduce("sum", pb.op("mul", d, d), 1), pb.dim_size(H))
    y = pb.op("mul", pb.op("mul", d, row(pb.op("rsqrt", pb.op("add", var, pb.const(1e-5))))), col(gam))
    pb.output(pb.cast(y, "bf16"))
    m = pb.reduce("max", y, 1)
    e = pb.op("exp", pb.op("sub", y, row(m)))
    p = pb.op("div", e, row(pb.reduce("sum", e, 1)))
    if p_is_output:
        pb.output(p)
    cm = pb.op("div", pb.reduce("sum", p, 0), pb.dim_size(T))
    pb.output(cm)
    pb.output(pb.cast(pb.op("sub", p, col(cm)), "f16"))
    return pb.build()


def chain_graph(n_stages=4):
    """Column-centre, row-normalise, column-centre, ...: every stage is a pattern of its own and
    hands a [T, H] fp32 value to the next, so the buffers between them can be shared."""
    pb = PatternBuilder("chain")
    T, H = pb.dims(2)
    v = pb.param("f32", [T, H])
    for s in range(n_stages):
        if s % 2 == 0:
            cm = pb.op("div", pb.reduce("sum", v, 0), pb.dim_size(T))
            v = pb.op("sub", v, pb.broadcast(cm, [T, H], [1]))
        else:
            m = pb.reduce("max", pb.op("abs", v), 1)
            v = pb.op("div", v, pb.broadcast(pb.op("add", m, pb.const(1.0)), [T, H], [0]))
    pb.output(v)
    return pb.build()


@pytest.fixture(scope="module")
def hctx():
    from paper_2103_05288_amd import Context
    c = Context(device=-1)
    yield c
    c.close()


def test_cut_into_patterns(hctx):
    pat = block_graph()
    g = hctx.register_graph(pat)
    info = g.info
    assert (info["n_inputs"], info["n_outputs"], info["n_dims"]) == (4, 4, 2)
    # everything up to the row softmax is one row-reduce pattern with four dependent reductions, which
    # also carries the column sum of p along (a sum over the rows next to row reductions); the
    # division by T and the centring are two loop fusions of different iteration spaces
    assert info["n_patterns"] == 3
    t = [hctx.pattern_info(p) for p in info["pattern_id"][:3]]
    assert [x["template"] for x in t] == ["row_reduce", "loop", "loop"] and t[0]["n_phases"] == 4 and t[0]["n_outputs"] == 3
    assert sum(info["pattern_ops"]) == sum(1 for o in pat.ops if o.opcode not in ("param", "const", "dim_size", "output"))
    groups = [x for x in info["group_of_op"] if x >= 0]
    assert groups == sorted(groups)                       # consecutive cuts in list order
    for i, o in enumerate(pat.ops):
        assert (info["group_of_op"][i] == -1) == (o.opcode in ("param", "const", "dim_size", "output"))
    # the only planned value is the column sum, H floats; the rest of the workspace is the first
    # pattern's partial sums
    assert info["n_intermediates"] == 1 and info["n_buffers"] == 1
    assert g.workspace_bytes([100, 768]) < 64 * 1024
    # the same graph with p no longer an output: p now lives in a planned buffer of T * H * 4 bytes
    g2 = hctx.register_graph(block_graph(p_is_output=False))
    i2 = g2.info
    assert i2["n_patterns"] == 3 and i2["n_intermediates"] == 2 and i2["n_buffers"] == 2
    assert g2.workspace_bytes([100, 768]) >= 100 * 768 * 4
    # one compile per distinct pattern: registering the graph again compiles nothing
    before = hctx.stats()["compile_events"]
    hctx.register_graph(block_graph())
    assert hctx.stats()["compile_events"] == before


def test_buffers_are_shared_by_lifetime(hctx):
    # five stages: a row stage carries the column sum of the following column stage along, so four
    # patterns; every stage output is recomputed by the later stages from the graph input and the
    # (small) reduction results of the stages before, so only small vectors cross the cuts
    g = hctx.register_graph(chain_graph(5))
    info = g.info
    assert info["n_patterns"] == 4 and info["n_intermediates"] == 5 and info["n_buffers"] == 5
    assert g.workspace_bytes([1000, 300]) < 1000 * 300 * 4 // 4
    # twelve stages: beyond four reduction results per value the stage outputs are stored in full,
    # and those buffers ping-pong (a value dies when the next stage has read it)
    g = hctx.register_graph(chain_graph(12))
    info = g.info
    assert info["n_patterns"] == 7 and info["n_intermediates"] == 11 and info["n_buffers"] == 8
    ws = g.workspace_bytes([1000, 300])
    assert 2 * 1000 * 300 * 4 <= ws < 3 * 1000 * 300 * 4
    one = hctx.register_graph(chain_graph(1)).info
    assert one["n_patterns"] == 1 and one["n_buffers"] == 0


def test_row_and_column_reductions_in_one_graph(hctx):
    g = hctx.register_graph(layernorm_backward_graph())
    info = g.info
    t = [hctx.pattern_info(p)["template"] for p in info["pattern_id"][:info["n_patterns"]]]
    # one row-reduce pattern: dgamma and dbeta are sums over the rows that the row kernels carry
    # along, so nothing crosses a cut and x and dy are read once
    assert t == ["row_reduce"], t
    assert hctx.pattern_info(info["pattern_id"][0])["n_phases"] == 3
    assert info["n_intermediates"] == 0 and info["n_buffers"] == 0
    assert g.workspace_bytes([65536, 1000]) < 65536 * 1000 * 4 // 8      # partial sums only
    # with a column MAXIMUM instead the column part stays a pattern of its own, and the normalised
    # activations do not cross the cut in full: the column pattern recomputes them from x and
    # the two per-row sums
    pb = PatternBuilder("row_then_col_max")
    T, H = pb.dims(2)
    x = pb.param("f32", [T, H])
    row = lambda v: pb.broadcast(v, [T, H], [0])
    mean = pb.op("div", pb.reduce("sum", x, 1), pb.dim_size(H))
    xc = pb.op("sub", x, row(mean))
    var = pb.op("div", pb.reduce("sum", pb.op("mul", xc, xc), 1), pb.dim_size(H))
    xhat = pb.op("mul", xc, row(pb.op("rsqrt", pb.op("add", var, pb.const(1e-5)))))
    pb.output(xhat)
    pb.output(pb.reduce("max", pb.op("abs", xhat), 0))
    g = hctx.register_graph(pb.build())
    info = g.info
    t = [hctx.pattern_info(p)["template"] for p in info["pattern_id"][:info["n_patterns"]]]
    assert t == ["row_reduce", "col_reduce"], t


def test_dead_code_belongs_to_no_pattern(hctx):
    """Ops that no output depends on are left out: they neither form patterns nor turn the values
    they read into buffers."""
    pb = PatternBuilder("dead")
    T, H = pb.dims(2)
    x = pb.param("f32", [T, H])
    y = pb.op("tanh", x)
    dead_col = pb.reduce("sum", pb.op("mul", y, y), 0)            # a column reduction nothing reads
    pb.op("neg", dead_col)
    m = pb.reduce("max", y, 1)
    pb.output(pb.op("sub", y, pb.broadcast(m, [T, H], [0])))
    pb.op("exp", y)                                               # trailing dead element-wise op
    g = hctx.register_graph(pb.build())
    info = g.info
    assert info["n_patterns"] == 1 and info["n_intermediates"] == 0 and g.workspace_bytes([10, 20]) == 0
    assert hctx.pattern_info(info["pattern_id"][0])["template"] == "row_reduce"
    assert sum(1 for x in info["group_of_op"][:10] if x == 0) == 4          # tanh, max, broadcast, sub


def test_graph_counts_runtime_starts_among_its_dims(hctx):
    """The start of a slice is a runtime value of its own: the graph expects it in dims[] even
    though no tensor has it as an extent."""
    pb = PatternBuilder("sliced_graph")
    T, H, W, s0 = pb.dims(4)
    x = pb.slice(pb.param("f32", [T, W]), [pb.static_start(0), s0], [T, H])
    m = pb.reduce("max", x, 1)
    c = pb.reduce("sum", pb.op("sub", x, pb.broadcast(m, [T, H], [0])), 0)
    pb.output(c)
    g = hctx.register_graph(pb.build())
    assert g.info["n_dims"] == 4 and g.info["n_patterns"] == 1     # (the column sum rides along with the row maximum)
    assert g.info["n_intermediates"] == 0 and g.workspace_bytes([10, 20, 30, 5]) >= 20 * 4    # a row of partial sums


def test_graph_errors(hctx):
    from paper_2103_05288_amd import DiscError
    pb = PatternBuilder()
    T, H = pb.dims(2)
    x = pb.param("f32", [T, H])
    pb.output(x)                                          # nothing computed
    with pytest.raises(DiscError) as e:
        hctx.register_graph(pb.build())
    assert e.value.status == "BAD_PATTERN"
    pb = PatternBuilder()
    T, H = pb.dims(2)
    x = pb.param("f32", [T, H])
    y = pb.op("neg", x)
    pb.output(y)
    pb.output(y)
    with pytest.raises(DiscError) as e:
        hctx.register_graph(pb.build())
    assert e.value.status == "BAD_PATTERN"
    g = hctx.register_graph(chain_graph(2))
    with pytest.raises(DiscError) as e:
        g.workspace_bytes([1, 2, 3])
    assert e.value.status == "INVALID_ARG"


@pytest.mark.gpu
@pytest.mark.parametrize("which", ["block", "block_inter", "chain", "chain12", "ln_bwd"])
def test_graph_matches_oracle(which):
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from tests.util import assert_close, to_oracle_input
    pat = {"block": block_graph(), "block_inter": block_graph(False), "chain": chain_graph(5), "chain12": chain_graph(12),
           "ln_bwd": layernorm_backward_graph()}[which]
    ctx = Context(0)
    try:
        g = ctx.register_graph(pat)
        gen = torch.Generator().manual_seed(11)
        for dims in ([7, 33], [300, 768], [1500, 1021], [64, 4099]):
            ins = []
            for pi in pat.params:
                shp = pat.shape_of(pi, dims)
                ins.append(torch.randn(shp, generator=gen).to(TORCH_DTYPE[pat.ops[pi].dtype]))
            dev_in = [t.cuda() for t in ins]
            outs = [torch.full(pat.shape_of(o, dims), float("nan"), dtype=TORCH_DTYPE[pat.ops[o].dtype], device="cuda")
                    for o in pat.outputs]
            ws = torch.empty(max(16, g.workspace_bytes(dims)), dtype=torch.uint8, device="cuda")
            g.launch(dims, dev_in, outs, workspace=ws)
            torch.cuda.synchronize()
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
            for k, (o, w) in enumerate(zip(outs, want)):
                if which == "ln_bwd" and k > 0:
                    # Column sums of T terms of mixed sign: the element-wise bar relative to the
                    # (cancelled) result does not apply.  Each term reaches the sum through at most 8
                    # fp32 roundings (centring, rstd, two products, the stored intermediate), the sum
                    # itself runs in fp64: |err| <= 8 * 2^-24 * sum_t |term_t| + 1e-6.
                    x64, dy64 = ins[0].double().numpy(), ins[1].double().numpy()
                    xc = x64 - x64.mean(1, keepdims=True)
                    xhat = xc / np.sqrt((xc * xc).mean(1, keepdims=True) + 1e-5)
                    terms = np.abs(dy64 * xhat) if k == 1 else np.abs(dy64)
                    lim = 8 * 2.0 ** -24 * terms.sum(0) + 1e-6
                    err = np.abs(o.cpu().double().numpy() - np.asarray(w, dtype=np.float64))
                    assert (err <= lim).all(), (which, dims, k, float((err / lim).max()))
                    continue
                assert_close(o.cpu(), w, f"graph {which} dims={dims} out{k}")
    finally:
        ctx.close()
