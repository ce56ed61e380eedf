"""Transposes of inputs that keep the innermost axis: host analysis without a GPU, parity with the
oracle on the GPU."""
import pytest
import torch

from workloads import PatternBuilder
from workloads.configs import TORCH_DTYPE


def heads_softmax():
    """[B, S, NH, D] read as [B, NH, S, D] (the attention-head transpose), softmax over D."""
    pb = PatternBuilder("heads_softmax")
    B, S, NH, D = pb.dims(4)
    full = [B, NH, S, D]
    t = pb.cast(pb.transpose(pb.param("bf16", [B, S, NH, D]), (0, 2, 1, 3)), "f32")
    e = pb.op("exp", pb.op("sub", t, pb.broadcast(pb.reduce("max", t, 3), full, [0, 1, 2])))
    pb.output(pb.cast(pb.op("div", e, pb.broadcast(pb.reduce("sum", e, 3), full, [0, 1, 2])), "bf16"))
    return pb.build()


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
    # moving the innermost axis would make every access strided: refused, with a reason
    pb = PatternBuilder()
    T, H = pb.dims(2)
    pb.output(pb.op("neg", pb.transpose(pb.param("f32", [H, T]), (1, 0))))
    with pytest.raises(DiscError) as e:
        hctx.register(pb.build())
    assert e.value.status == "UNFUSIBLE" and "tile transpose" in str(e.value)
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
