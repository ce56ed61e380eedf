"""Transposes of inputs: those that keep the innermost axis are fused as indexing functions; one
that moves it is a pattern of its own (a batched 2-D tile transpose), which an op graph cuts out.
Host analysis without a GPU, parity with the oracle on the GPU."""
import pytest
import torch

from workloads import PatternBuilder
from workloads.extras import heads_softmax, pure_transpose
from workloads.configs import TORCH_DTYPE


def add_transposed():
    """[S, B, H] + transpose([B, S, H]) + a row vector."""
    pb = PatternBuilder("add_transposed")
    B, S, H = pb.dims(3)
    a = pb.param("f32", [S, B, H])
    b = pb.transpose(pb.param("f16", [B, S, H]), (1, 0, 2))
    v = pb.param("f32", [H])
    pb.output(pb.op("add", pb.op("add", a, pb.cast(b, "f32")), pb.broadcast(v, [S, B, H], [2])))
    return pb.build()


def column_sum_of_transposed():
    """Sum over B of a [B, S, H] input read as [S, B, H]: a column reduction over the middle axis of
    the iteration space, which is the outermost axis of the input."""
    pb = PatternBuilder("colsum_transposed")
    B, S, H = pb.dims(3)
    t = pb.transpose(pb.param("f32", [B, S, H]), (1, 0, 2))
    pb.output(pb.reduce("sum", pb.op("sigmoid", t), 1))
    return pb.build()


def transpose_then_softmax():
    """softmax over the rows of x^T: the transpose cannot be fused, the softmax reads its result."""
    pb = PatternBuilder("transpose_softmax")
    H, T = pb.dims(2)
    xt = pb.cast(pb.transpose(pb.param("bf16", [H, T]), (1, 0)), "f32")          # [T, H]
    e = pb.op("exp", pb.op("sub", xt, pb.broadcast(pb.reduce("max", xt, 1), [T, H], [0])))
    pb.output(pb.cast(pb.op("div", e, pb.broadcast(pb.reduce("sum", e, 1), [T, H], [0])), "bf16"))
    return pb.build()


@pytest.fixture(scope="module")
def hctx():
    from paper_2103_05288_amd import Context
    c = Context(device=-1)
    yield c
    c.close()


def test_transpose_analysis(hctx):
    from paper_2103_05288_amd import DiscError
    h = hctx.register(heads_softmax())
    assert h.info["template"] == "row_reduce" and h.info["n_collapsed"] == 4      # nothing merges across the swap
    assert "rc.b0 = ig[0] * A.st0 + ig[1] * A.st1 + ig[2] * A.st2;" in h.source
    assert hctx.register(add_transposed()).info["template"] == "loop"
    assert hctx.register(column_sum_of_transposed()).info["template"] == "col_reduce"
    # an identity permutation changes nothing: the axes merge as for the input itself
    pb = PatternBuilder()
    B, S, H = pb.dims(3)
    pb.output(pb.op("neg", pb.transpose(pb.param("f32", [B, S, H]), (0, 1, 2))))
    assert hctx.register(pb.build()).info["n_collapsed"] == 1
    # moving the innermost axis would make every access strided: not fused with anything, with a reason
    pb = PatternBuilder()
    T, H = pb.dims(2)
    pb.output(pb.op("neg", pb.transpose(pb.param("f32", [H, T]), (1, 0))))
    with pytest.raises(DiscError) as e:
        hctx.register(pb.build())
    assert e.value.status == "UNFUSIBLE" and "tile transpose" in str(e.value)
    # ... but alone it is a pattern: a batched 2-D transpose after collapsing
    for perm, collapsed in (((1, 0), 2), ((0, 2, 1), 3), ((2, 0, 1), 2), ((1, 2, 0), 2), ((0, 1, 3, 2), 3)):
        h = hctx.register(pure_transpose("bf16", perm))
        assert h.info["template"] == "transpose" and h.info["n_collapsed"] == collapsed, perm
    dims = [3, 100, 200]
    pl = hctx.register(pure_transpose("f32", (0, 2, 1))).plan(dims)
    assert pl["variant_name"] == "transpose_tile" and pl["grid"][0][0] == 3 * 2 * 4 and pl["algorithmic_bytes"] == 2 * 4 * 60000
    with pytest.raises(DiscError) as e:
        hctx.register(pure_transpose("f32", (2, 1, 0)))       # a full reversal is no batched 2-D transpose
    assert e.value.status == "UNFUSIBLE"
    # in an op graph such a transpose becomes a pattern of its own with a planned buffer behind it
    g = hctx.register_graph(transpose_then_softmax())
    info = g.info
    t = [hctx.pattern_info(p)["template"] for p in info["pattern_id"][:info["n_patterns"]]]
    assert t == ["transpose", "row_reduce"] and info["n_intermediates"] == 1 and info["n_buffers"] == 1
    pb = PatternBuilder()
    T, H = pb.dims(2)
    pb.output(pb.transpose(pb.op("neg", pb.param("f32", [H, T])), (1, 0)))
    with pytest.raises(DiscError) as e:
        hctx.register(pb.build())
    assert e.value.status == "BAD_PATTERN"


CASES = {
    "heads_softmax": (heads_softmax, [[2, 100, 12, 64], [1, 7, 3, 33], [3, 257, 5, 128], [2, 33, 16, 1000]]),
    "add_transposed": (add_transposed, [[4, 50, 64], [3, 7, 33], [17, 300, 1021], [1, 9, 4099], [64, 1, 100]]),
    "colsum_transposed": (column_sum_of_transposed, [[4, 50, 64], [3, 700, 33], [2, 3000, 520], [9, 1, 1000]]),
}


@pytest.mark.gpu
@pytest.mark.parametrize("which", sorted(CASES))
def test_transpose_matches_oracle(which):
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from tests.util import assert_close, run_gpu, to_oracle_input
    make, shapes = CASES[which]
    pat = make()
    ctx = Context(0)
    try:
        h = ctx.register(pat)
        gen = torch.Generator().manual_seed(8)
        for dims in shapes:
            ins = [torch.randn(pat.shape_of(pi, dims), generator=gen).to(TORCH_DTYPE[pat.ops[pi].dtype]) for pi in pat.params]
            got = run_gpu(h, pat, dims, ins)
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
            for k, (g, w) in enumerate(zip(got, want)):
                assert_close(g, w, f"{which} dims={dims} out{k} kernel={h.plan(dims)['kernels']}")
        assert h.info["compile_events"] == 1
    finally:
        ctx.close()


@pytest.mark.gpu
def test_tile_transpose_matches_oracle():
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from tests.util import run_gpu, to_oracle_input
    ctx = Context(0)
    try:
        gen = torch.Generator().manual_seed(9)
        cases = [("f32", (1, 0), [[100, 200], [1, 7], [64, 64], [65, 129], [1000, 3], [0, 5]]),
                 ("bf16", (0, 2, 1), [[3, 100, 200], [2, 1, 77], [5, 130, 63]]),
                 ("bool", (2, 0, 1), [[3, 4, 50], [7, 9, 200]]),
                 ("f16", (1, 2, 0), [[33, 4, 50]]),
                 ("i32", (0, 1, 3, 2), [[2, 3, 40, 50]])]
        for dtype, perm, shapes in cases:
            pat = pure_transpose(dtype, perm)
            h = ctx.register(pat)
            for dims in shapes:
                n = 1
                for d in dims:
                    n *= d
                if dtype == "bool":
                    x = (torch.rand(dims, generator=gen) < 0.5).to(torch.uint8)
                elif dtype == "i32":
                    x = torch.randint(-1000, 1000, dims, generator=gen, dtype=torch.int32)
                else:
                    x = torch.randn(dims, generator=gen).to(TORCH_DTYPE[dtype])
                got = run_gpu(h, pat, dims, [x])[0]
                want = oracle_run(pat, dims, [to_oracle_input(x)])[0][0]
                assert got.shape == want.shape
                assert (got.double().numpy() == want.astype("float64")).all(), (dtype, perm, dims)   # a copy: bit-exact
            assert h.info["compile_events"] == 1
        # the graph: transpose kernel, then the fused softmax on its result
        from tests.util import assert_close
        pat = transpose_then_softmax()
        g = ctx.register_graph(pat)
        for dims in ([100, 37], [1021, 300], [64, 4099]):
            x = torch.randn(dims, generator=gen).bfloat16()
            out = torch.full((dims[1], dims[0]), float("nan"), dtype=torch.bfloat16, device="cuda")
            ws = torch.empty(max(16, g.workspace_bytes(dims)), dtype=torch.uint8, device="cuda")
            g.launch(dims, [x.cuda()], [out], workspace=ws)
            torch.cuda.synchronize()
            want = oracle_run(pat, dims, [to_oracle_input(x)])[0][0]
            assert_close(out.cpu(), want, f"transpose + softmax graph dims={dims}")
    finally:
        ctx.close()
