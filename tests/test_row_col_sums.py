"""Sums over the rows fused into a row-reduce pattern (the weight gradients of a normalisation next
to its input gradient, Section 4.3's input fusion with both reduction kinds in one kernel): the
checker's acceptance rule, the launch plan, and parity with the oracle through the C ABI."""
import numpy as np
import pytest
import torch

from workloads.configs import TORCH_DTYPE
from workloads.extras import gelu_backward_bias_gradient, layernorm_backward_graph, logsumexp_with_total_and_amax
from workloads.pattern import PatternBuilder


@pytest.fixture(scope="module")
def hctx():
    from paper_2103_05288_amd import Context
    c = Context(device=-1)
    yield c
    c.close()


def softmax_backward_with_bias_gradient():
    """dx of a row softmax (one row reduction) and the column sum of dx's upstream gradient."""
    pb = PatternBuilder("softmax_bwd_bias")
    t, h = pb.dims(2)
    y = pb.cast(pb.param("bf16", [t, h]), "f32")
    dy = pb.cast(pb.param("bf16", [t, h]), "f32")
    dot = pb.reduce("sum", pb.op("mul", dy, y), 1)
    dx = pb.op("mul", y, pb.op("sub", dy, pb.broadcast(dot, [t, h], [0])))
    pb.output(pb.cast(dx, "bf16"))
    pb.output(pb.reduce("sum", dx, 0))
    return pb.build()


def test_one_pattern_two_launches(hctx):
    pat = layernorm_backward_graph()
    h = hctx.register(pat)
    assert h.info["template"] == "row_reduce" and h.info["n_phases"] == 3 and h.info["n_outputs"] == 3
    pl = h.plan([4096, 1024])
    assert pl["n_launches"] == 2 and pl["kernels"][0].split("k_row_")[1].startswith("vec_nv2") and pl["kernels"][1].endswith("k_colsum_finish")
    # one row of fp32 partial sums per block and summed output
    assert pl["workspace_bytes"] == pl["grid"][0][0] * 1024 * 4 * 2
    assert pl["grid"][1][0] == 1024 // 16 and pl["block"][1][0] == 256
    # rows too long for registers: the streaming version keeps the partial sums in the workspace
    pl = h.plan([100, 30000])
    assert pl["kernels"][0].endswith("k_row_stream_vec") and pl["workspace_bytes"] == 100 * 30000 * 4 * 2
    # wide blocks (one lane group per block): still one row of partial sums per block
    pl = h.plan([3000, 8192])
    assert pl["block"][0][0] == 512 and pl["workspace_bytes"] == pl["grid"][0][0] * 8192 * 4 * 2
    # the graph front end now keeps the whole backward pass in this one pattern
    g = hctx.register_graph(pat)
    assert g.info["n_patterns"] == 1 and g.info["n_intermediates"] == 0
    # a sum over zero rows has no value
    from paper_2103_05288_amd import DiscError
    with pytest.raises(DiscError) as e:
        h.plan([0, 64])
    assert "size 0" in str(e.value)


def test_acceptance_rule(hctx):
    from paper_2103_05288_amd import DiscError

    def build(kind="sum", consume=False, rank3=False, integer=False):
        pb = PatternBuilder("rule")
        if rank3:
            b, t, h = pb.dims(3)
            shape, rows_axes = [b, t, h], [0, 1]
        else:
            t, h = pb.dims(2)
            shape, rows_axes = [t, h], [0]
        x = pb.param("i32" if integer else "f32", shape)
        m = pb.reduce("max", x, len(shape) - 1)
        d = pb.op("sub", x, pb.broadcast(m, shape, rows_axes))
        pb.output(d)
        s = pb.reduce(kind, d, 0)
        if consume:
            s = pb.op("neg", s)
        pb.output(s)
        return pb.build()

    assert hctx.register(build()).info["template"] == "row_reduce"
    for kw, word in ((dict(kind="max"), "floating-point sum"), (dict(consume=True), "outputs alone"),
                     (dict(rank3=True), "two-dimensional"), (dict(integer=True), "floating-point sum")):
        with pytest.raises(DiscError) as e:
            hctx.register(build(**kw))
        assert e.value.status == "UNFUSIBLE" and word in str(e.value), (kw, str(e.value))


def test_sum_over_rows_beside_a_loop_fusion(hctx):
    """No row reduction at all: an element-wise backward with its bias gradient runs in the row
    template without reduction phases (operands read once); a pattern whose element-wise output
    needs the column sum keeps the column-reduce template."""
    h = hctx.register(gelu_backward_bias_gradient())
    assert h.info["template"] == "row_reduce" and h.info["n_phases"] == 0 and h.info["n_outputs"] == 2
    pl = h.plan([4096, 1024])
    assert pl["n_launches"] == 2 and pl["kernels"][1].endswith("k_colsum_finish")
    assert pl["workspace_bytes"] == pl["grid"][0][0] * 1024 * 4
    assert h.plan([5, 0])["n_launches"] == 0           # nothing to compute, and no reduction over an empty axis
    pb = PatternBuilder("centre")
    t, hh = pb.dims(2)
    x = pb.param("f32", [t, hh])
    m = pb.op("div", pb.reduce("sum", x, 0), pb.dim_size(t))
    pb.output(pb.op("sub", x, pb.broadcast(m, [t, hh], [1])))
    assert hctx.register(pb.build()).info["template"] == "col_reduce"
    # a column sum alone (no full-shape output) also stays a column reduce: more parallel over the rows
    pb = PatternBuilder("bias_grad_alone")
    t, hh = pb.dims(2)
    pb.output(pb.reduce("sum", pb.op("tanh", pb.param("f32", [t, hh])), 0))
    assert hctx.register(pb.build()).info["template"] == "col_reduce"


def test_per_row_values_reduced_over_the_rows(hctx):
    """Rank-0 outputs: a sum / maximum / minimum of per-row values over the rows rides along in the
    row kernels (one partial result per block, a last one-block launch)."""
    from paper_2103_05288_amd import DiscError
    pat = logsumexp_with_total_and_amax()
    h = hctx.register(pat)
    assert h.info["template"] == "row_reduce" and h.info["n_phases"] == 2 and h.info["n_outputs"] == 3
    pl = h.plan([4096, 1024])
    assert pl["n_launches"] == 2 and pl["kernels"][1].endswith("k_rowred_finish") and pl["grid"][1] == [1, 1, 1]
    assert pl["workspace_bytes"] == 2 * pl["grid"][0][0] * 4
    assert h.plan([100, 30000])["kernels"][0].endswith("k_row_stream_vec")
    with pytest.raises(DiscError) as e:
        h.plan([0, 64])
    assert e.value.status == "EMPTY_REDUCE"
    assert pat.shape_of(pat.outputs[1], [7, 5]) == ()
    # with sums over the rows of full-size values in the same pattern: three launches
    pb = PatternBuilder("both")
    t, hh = pb.dims(2)
    x = pb.param("f32", [t, hh])
    m = pb.reduce("max", x, 1)
    d = pb.op("sub", x, pb.broadcast(m, [t, hh], [0]))
    pb.output(d)
    pb.output(pb.reduce("sum", d, 0))
    pb.output(pb.reduce("min", m, 0))
    hb = hctx.register(pb.build())
    pl = hb.plan([4096, 1024])
    assert [k.split("_k_")[1] for k in pl["kernels"]][1:] == ["colsum_finish", "rowred_finish"]
    assert pl["workspace_bytes"] == (pl["grid"][0][0] * 1024 * 4 + 255) // 256 * 256 + pl["grid"][0][0] * 4
    # what is not fused: a rank-0 result of anything else
    for build in ("prod_like_argmax", "consumed", "column_vector", "no_row_reduce"):
        pb = PatternBuilder(build)
        t, hh = pb.dims(2)
        x = pb.param("f32", [t, hh])
        m = pb.reduce("max", x, 1)
        pb.output(pb.op("sub", x, pb.broadcast(m, [t, hh], [0])))
        if build == "prod_like_argmax":
            pb.output(pb.reduce("argmax", m, 0))
        elif build == "consumed":
            s = pb.reduce("sum", m, 0)
            pb.output(pb.op("sub", m, pb.broadcast(s, [t], [])))
        elif build == "column_vector":
            pb.output(pb.reduce("sum", pb.reduce("sum", x, 0), 0))
        else:
            pb = PatternBuilder(build)
            t = pb.dim()
            pb.output(pb.reduce("sum", pb.param("f32", [t]), 0))
        with pytest.raises(DiscError) as e:
            hctx.register(pb.build())
        assert e.value.status in ("UNFUSIBLE", "BAD_PATTERN"), (build, str(e.value))


def _inputs(pat, dims, gen):
    ins = []
    for pi in pat.params:
        shp = pat.shape_of(pi, dims)
        ins.append(torch.randn(shp, generator=gen).to(TORCH_DTYPE[pat.ops[pi].dtype]))
    return ins


def _check_sum(got, want, terms_abs, rows_per_block, what):
    """A sum of T terms of mixed sign cannot meet a bar relative to the (cancelled) result.  Each
    term carries at most 8 fp32 roundings from the element-wise arithmetic; a lane then adds the
    terms of its block's rows in fp32 (rows_per_block additions), the lane groups of a block meet in
    at most 8 more fp32 additions, and the partial rows are added in fp64:
    |err| <= (16 + rows_per_block) * 2^-24 * sum_t |term_t| + 1e-6."""
    lim = (16 + rows_per_block) * 2.0 ** -24 * terms_abs.sum(0) + 1e-6
    err = np.abs(got.double().numpy() - np.asarray(want, dtype=np.float64))
    assert (err <= lim).all(), (what, float((err / lim).max()))


LN_SHAPES = [[7, 5], [300, 1], [1000, 77], [20000, 16], [4096, 1024], [513, 2050], [1500, 1021], [300, 4100],
             [65, 8200], [40, 30000], [3, 40000]]


@pytest.mark.gpu
@pytest.mark.parametrize("dims", LN_SHAPES, ids=lambda d: f"{d[0]}x{d[1]}")
def test_layernorm_backward_single_pattern_matches_oracle(dims):
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from tests.util import assert_close, run_gpu, to_oracle_input
    pat = layernorm_backward_graph()
    ctx = Context(0)
    try:
        h = ctx.register(pat)
        gen = torch.Generator().manual_seed(dims[0] * 7919 + dims[1])
        ins = _inputs(pat, dims, gen)
        pl = h.plan(dims)
        assert pl["n_launches"] == 2
        got = run_gpu(h, pat, dims, ins)
        want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
        assert_close(got[0], want[0], f"dx dims={dims}")
        x64, dy64 = ins[0].double().numpy(), ins[1].double().numpy()
        xc = x64 - x64.mean(1, keepdims=True)
        xhat = xc / np.sqrt((xc * xc).mean(1, keepdims=True) + 1e-5)
        rpb = -(-dims[0] // pl["grid"][0][0])
        _check_sum(got[1], want[1], np.abs(dy64 * xhat), rpb, f"dgamma dims={dims} {pl['kernels'][0]}")
        _check_sum(got[2], want[2], np.abs(dy64), rpb, f"dbeta dims={dims} {pl['kernels'][0]}")
        # the same call again on the same workspace gives the same bits (fixed summation order)
        again = run_gpu(h, pat, dims, ins)
        for a, b in zip(got, again):
            assert torch.equal(a, b)
    finally:
        ctx.close()


@pytest.mark.gpu
def test_forced_versions_and_one_phase_pattern():
    """Every row-kernel version carries the sums (scalar and streaming versions forced on shapes the
    host would give to the vector version), and a one-phase pattern (softmax backward) with a single
    summed output."""
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from paper_2103_05288_amd.binding import VARIANTS
    from tests.util import assert_close, run_gpu, to_oracle_input
    ctx = Context(0)
    try:
        pat = layernorm_backward_graph()
        h = ctx.register(pat)
        gen = torch.Generator().manual_seed(5)
        for force in ("row_reg_vec", "row_reg_scalar", "row_stream_vec", "row_stream_scalar"):
            for dims in ([33, 768], [600, 100]):
                ins = _inputs(pat, dims, gen)
                ctx.force_variant(VARIANTS.index(force))
                try:
                    pl = h.plan(dims, force_variant=VARIANTS.index(force))
                    got = run_gpu(h, pat, dims, ins)
                finally:
                    ctx.force_variant(-1)
                want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
                assert_close(got[0], want[0], f"dx {force} {dims}")
                x64, dy64 = ins[0].double().numpy(), ins[1].double().numpy()
                xc = x64 - x64.mean(1, keepdims=True)
                xhat = xc / np.sqrt((xc * xc).mean(1, keepdims=True) + 1e-5)
                rpb = -(-dims[0] // pl["grid"][0][0])
                _check_sum(got[1], want[1], np.abs(dy64 * xhat), rpb, f"dgamma {force} {dims}")
                _check_sum(got[2], want[2], np.abs(dy64), rpb, f"dbeta {force} {dims}")
        pat = softmax_backward_with_bias_gradient()
        h = ctx.register(pat)
        assert h.info["template"] == "row_reduce" and h.info["n_phases"] == 1
        for dims in ([3, 7], [2000, 1000], [9, 5739], [5000, 48]):
            probs = torch.softmax(torch.randn(*dims, generator=gen), dim=1).bfloat16()
            ins = [probs, torch.randn(*dims, generator=gen).bfloat16()]
            pl = h.plan(dims)
            got = run_gpu(h, pat, dims, ins)
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
            assert_close(got[0], want[0], f"softmax backward dx {dims}")
            y64, dy64 = ins[0].double().numpy(), ins[1].double().numpy()
            dx = y64 * (dy64 - (dy64 * y64).sum(1, keepdims=True))
            _check_sum(got[1], want[1], np.abs(dx) + np.abs(y64 * dy64), -(-dims[0] // pl["grid"][0][0]), f"sum of dx {dims}")
    finally:
        ctx.close()


@pytest.mark.gpu
def test_gelu_backward_with_bias_gradient_matches_oracle():
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from tests.util import assert_close, run_gpu, to_oracle_input
    pat = gelu_backward_bias_gradient()
    ctx = Context(0)
    try:
        h = ctx.register(pat)
        gen = torch.Generator().manual_seed(17)
        for dims in ([1, 1], [7, 5], [1000, 77], [20000, 16], [4096, 1024], [513, 2050], [300, 4100], [65, 8200], [40, 30000]):
            ins = _inputs(pat, dims, gen)
            pl = h.plan(dims)
            got = run_gpu(h, pat, dims, ins)
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
            assert_close(got[0], want[0], f"gelu backward dx dims={dims}")
            dy, x, b = (t.double().numpy() for t in ins)
            a = 1.702 * (x + b)
            s = 1.0 / (1.0 + np.exp(-a))
            dx = dy * s * (1.0 + a * (1.0 - s))
            _check_sum(got[1], want[1], np.abs(dx), -(-dims[0] // pl["grid"][0][0]), f"bias gradient dims={dims} {pl['kernels'][0]}")
    finally:
        ctx.close()


@pytest.mark.gpu
def test_single_shape_build_of_a_pattern_with_sums_over_rows():
    """The shape-specialised build (every extent and plan member a constant, Section 5.3's static
    counterpart) of LayerNorm backward: the number of partial-sum rows follows the grid of the
    launch, not the one planned at registration."""
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from tests.util import assert_close, run_gpu, to_oracle_input
    pat = layernorm_backward_graph()
    ctx = Context(0)
    try:
        gen = torch.Generator().manual_seed(23)
        for dims in ([20000, 768], [3000, 2050]):
            ins = _inputs(pat, dims, gen)
            hs = ctx.register_static(pat, dims)
            pl = hs.plan(dims)
            got = run_gpu(hs, pat, dims, ins)
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
            assert_close(got[0], want[0], f"static dx dims={dims}")
            x64, dy64 = ins[0].double().numpy(), ins[1].double().numpy()
            xc = x64 - x64.mean(1, keepdims=True)
            xhat = xc / np.sqrt((xc * xc).mean(1, keepdims=True) + 1e-5)
            rpb = -(-dims[0] // pl["grid"][0][0])
            _check_sum(got[1], want[1], np.abs(dy64 * xhat), rpb, f"static dgamma dims={dims}")
            _check_sum(got[2], want[2], np.abs(dy64), rpb, f"static dbeta dims={dims}")
    finally:
        ctx.close()


@pytest.mark.gpu
def test_logsumexp_total_and_amax_match_oracle():
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from paper_2103_05288_amd.binding import VARIANTS
    from tests.util import assert_close, run_gpu, to_oracle_input
    pat = logsumexp_with_total_and_amax()
    ctx = Context(0)
    try:
        h = ctx.register(pat)
        gen = torch.Generator().manual_seed(29)
        cases = [([1, 1], None), ([7, 5], None), ([1000, 77], None), ([20000, 16], None), ([4096, 1024], None), ([513, 2050], None),
                 ([300, 4100], None), ([65, 8200], None), ([40, 30000], None),
                 ([33, 768], "row_reg_scalar"), ([600, 100], "row_stream_vec"), ([600, 100], "row_stream_scalar")]
        for dims, force in cases:
            ins = [(3 * torch.randn(*dims, generator=gen)).bfloat16()]
            fv = VARIANTS.index(force) if force else -1
            ctx.force_variant(fv)
            try:
                pl = h.plan(dims, force_variant=fv)
                got = run_gpu(h, pat, dims, ins)
            finally:
                ctx.force_variant(-1)
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
            assert_close(got[0], want[0], f"lse dims={dims} {force}")
            # the total: terms of either sign, each with fp32 roundings of its own; a lane adds the
            # rows of its block in fp32, the blocks are added in fp64
            lse = np.asarray(want[0], dtype=np.float64)
            rpb = -(-dims[0] // pl["grid"][0][0])
            lim = (16 + rpb) * 2.0 ** -24 * np.abs(lse).sum() + 1e-6
            assert abs(float(got[1]) - float(want[1])) <= lim, (dims, force, float(got[1]), float(want[1]), lim)
            # the amax of bf16 inputs is exact
            assert float(got[2]) == float(want[2]) == float(ins[0].float().abs().max()), (dims, force)
    finally:
        ctx.close()


@pytest.mark.gpu
def test_column_sums_and_scalar_reductions_together():
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from tests.util import assert_close, run_gpu, to_oracle_input
    pb = PatternBuilder("both")
    t, hh = pb.dims(2)
    x = pb.param("f32", [t, hh])
    m = pb.reduce("max", x, 1)
    e = pb.op("exp", pb.op("sub", x, pb.broadcast(m, [t, hh], [0])))        # in (0, 1]
    pb.output(pb.cast(e, "bf16"))
    pb.output(pb.reduce("sum", e, 0))                                      # non-negative terms: the element-wise bar applies
    pb.output(pb.reduce("min", m, 0))
    pb.output(pb.reduce("sum", pb.reduce("sum", e, 1), 0))
    pat = pb.build()
    ctx = Context(0)
    try:
        h = ctx.register(pat)
        assert h.info["n_phases"] == 2
        gen = torch.Generator().manual_seed(37)
        for dims in ([5, 3], [3000, 130], [700, 1024], [129, 5000], [50, 26000]):
            ins = [torch.randn(*dims, generator=gen)]
            assert h.plan(dims)["n_launches"] == 3
            got = run_gpu(h, pat, dims, ins)
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
            for k, (g, w) in enumerate(zip(got, want)):
                assert_close(g, w, f"dims={dims} out{k}")
    finally:
        ctx.close()
