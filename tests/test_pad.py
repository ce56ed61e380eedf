"""Dynamic pads of inputs (the padding in front of every axis and the result sizes are runtime
values): host analysis without a GPU, parity with the oracle on the GPU."""
import numpy as np
import pytest
import torch

from workloads import PatternBuilder
from workloads.extras import padded_softmax
from workloads.configs import TORCH_DTYPE


def pad_scale():
    """Both axes of a 2-D input padded with 1.5, then scaled."""
    pb = PatternBuilder("pad_scale")
    T, H, l0, l1, P0, P1 = pb.dims(6)
    xp = pb.pad(pb.param("f32", [T, H]), [l0, l1], [P0, P1], 1.5)
    pb.output(pb.op("mul", xp, pb.const(2.0)))
    return pb.build()


def padded_middle_axis():
    """[B, S, H] padded along S only: S and H still collapse into one group and the operand is a
    window of that group's index; added to a full-size second input."""
    pb = PatternBuilder("pad_middle")
    B, S, H, l1, P = pb.dims(5)
    z = pb.static_start(0)
    xp = pb.pad(pb.param("f16", [B, S, H]), [z, l1, z], [B, P, H], 0.0)
    y = pb.param("f16", [B, P, H])
    pb.output(pb.cast(pb.op("add", pb.cast(xp, "f32"), pb.cast(y, "f32")), "f16"))
    return pb.build()


def padded_rows_column_sum():
    pb = PatternBuilder("pad_colsum")
    T, C, l0, P = pb.dims(4)
    xp = pb.pad(pb.param("f32", [T, C]), [l0, pb.static_start(0)], [P, C], 0.25)
    s = pb.reduce("sum", pb.op("sigmoid", xp), 0)
    pb.output(s)
    pb.output(pb.op("sub", xp, pb.broadcast(s, [P, C], [1])))
    return pb.build()


def concat_then_layernorm_free():
    """concat(a, b) along the last axis, written as the sum of two zero-padded inputs (x + 0 = x), then
    a mean-centring over the joined row: no concatenated tensor ever exists in memory."""
    pb = PatternBuilder("concat_centre")
    T, Ha, Hb, P = pb.dims(4)                       # P = Ha + Hb, checked at launch by the pads
    z = pb.static_start(0)
    a = pb.cast(pb.pad(pb.param("bf16", [T, Ha]), [z, z], [T, P], 0.0), "f32")
    b = pb.cast(pb.pad(pb.param("bf16", [T, Hb]), [z, Ha], [T, P], 0.0), "f32")
    c = pb.op("add", a, b)
    mean = pb.op("div", pb.reduce("sum", c, 1), pb.dim_size(P))
    pb.output(pb.cast(pb.op("sub", c, pb.broadcast(mean, [T, P], [0])), "bf16"))
    return pb.build()


@pytest.fixture(scope="module")
def hctx():
    from paper_2103_05288_amd import Context
    c = Context(device=-1)
    yield c
    c.close()


def test_pad_analysis(hctx):
    from paper_2103_05288_amd import DiscError
    h = hctx.register(pad_scale())
    assert h.info["template"] == "loop" and h.info["n_dims"] == 6 and h.info["n_collapsed"] == 2
    assert "disc::ld_win(" in h.source and "rc.v0 = ig[0] >= A.st" in h.source
    pl = h.plan([10, 20, 2, 3, 15, 30])
    assert pl["algorithmic_bytes"] == 10 * 20 * 4 + 15 * 30 * 4      # the operand read once, the padded result written once
    for bad in ([10, 20, 6, 3, 15, 30], [10, 20, 2, 11, 15, 30], [10, 20, 0, 0, 9, 30]):
        with pytest.raises(DiscError) as e:
            h.plan(bad)
        assert e.value.status == "SHAPE"
    assert h.plan([10, 20, 5, 10, 15, 30])["kernels"]                 # flush against the far edges
    assert hctx.register(padded_middle_axis()).info["n_collapsed"] == 2
    for make, tmpl in ((padded_softmax, "row_reduce"), (padded_rows_column_sum, "col_reduce")):
        assert hctx.register(make()).info["template"] == tmpl
    pb = PatternBuilder()
    T, H, l1, P = pb.dims(4)
    y = pb.op("neg", pb.param("f32", [T, H]))
    pb.output(pb.pad(y, [pb.static_start(0), l1], [T, P], 0.0))
    with pytest.raises(DiscError) as e:
        hctx.register(pb.build())
    assert e.value.status == "BAD_PATTERN"


CASES = {
    "pad_scale": (pad_scale, [[10, 20, 2, 3, 15, 30], [7, 33, 0, 0, 7, 33], [300, 1021, 5, 3, 400, 1030], [64, 4099, 1, 8, 65, 4200],
                              [5, 9, 3, 11, 8, 20], [0, 9, 0, 2, 4, 16]]),
    "padded_softmax": (padded_softmax, [[40, 100, 0, 128], [9, 1000, 24, 1024], [700, 2047, 1, 2049], [30, 8190, 0, 8192], [3, 5, 4, 9]]),
    "pad_middle": (padded_middle_axis, [[4, 50, 64, 10, 70], [2, 9, 1000, 0, 9], [3, 700, 33, 5, 800], [1, 1, 9000, 7, 30]]),
    "concat_centre": (concat_then_layernorm_free, [[40, 100, 28, 128], [9, 1000, 1000, 2000], [700, 2047, 3, 2050], [30, 1, 8191, 8192]]),
    "pad_colsum": (padded_rows_column_sum, [[100, 64, 10, 150], [3000, 520, 100, 3200], [17, 1000, 1, 18], [500, 33, 0, 500]]),
}


@pytest.mark.gpu
@pytest.mark.parametrize("which", sorted(CASES))
def test_pad_matches_oracle(which):
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from tests.util import assert_close, run_gpu, to_oracle_input
    make, shapes = CASES[which]
    pat = make()
    ctx = Context(0)
    try:
        h = ctx.register(pat)
        gen = torch.Generator().manual_seed(6)
        for dims in shapes:
            ins = [torch.randn(pat.shape_of(pi, dims), generator=gen).to(TORCH_DTYPE[pat.ops[pi].dtype]) for pi in pat.params]
            got = run_gpu(h, pat, dims, ins)
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
            for k, (g, w) in enumerate(zip(got, want)):
                assert_close(g, w, f"{which} dims={dims} out{k} kernel={h.plan(dims)['kernels']}")
        assert h.info["compile_events"] == 1
    finally:
        ctx.close()
