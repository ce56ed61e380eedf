"""Dynamic slices of inputs (start indices and sizes are runtime values): host analysis without a
GPU, parity with the oracle on the GPU."""
import numpy as np
import pytest
import torch

from workloads import PatternBuilder
from workloads.extras import qkv_split, softmax_of_window
from workloads.configs import TORCH_DTYPE


def loop_slice():
    pb = PatternBuilder("slice_scale")
    T, H, s0, n = pb.dims(4)
    xs = pb.slice(pb.param("f32", [T, H]), [pb.static_start(0), s0], [T, n])
    pb.output(pb.op("mul", xs, pb.const(2.0)))
    return pb.build(), lambda t, h, s, m: [t, h, s, m], lambda d: [(d[0], d[1])]


def column_sum_of_rows_window():
    pb = PatternBuilder("window_colsum")
    T, C, r0, m = pb.dims(4)
    x = pb.param("f32", [T, C])
    xs = pb.slice(x, [r0, pb.static_start(0)], [m, C])
    s = pb.reduce("sum", pb.op("sigmoid", xs), 0)
    pb.output(s)
    pb.output(pb.op("mul", xs, pb.broadcast(pb.op("rcp", s), [m, C], [1])))
    return pb.build()


@pytest.fixture(scope="module")
def hctx():
    from paper_2103_05288_amd import Context
    c = Context(device=-1)
    yield c
    c.close()


def test_slice_analysis(hctx):
    from paper_2103_05288_amd import DiscError
    pat, _, _ = loop_slice()
    h = hctx.register(pat)
    assert h.info["template"] == "loop" and h.info["n_dims"] == 4
    assert "A.st1 + ig[0] * A.st0" in h.source          # base offset + row * (row pitch of the input)
    pl = h.plan([100, 64, 8, 40])
    assert pl["algorithmic_bytes"] == 2 * 100 * 40 * 4   # the window read once, the result written once
    # a window that leaves the input is refused at launch, before anything runs
    for bad in ([100, 64, 30, 40], [100, 64, 0, 65]):
        with pytest.raises(DiscError) as e:
            h.plan(bad)
        assert e.value.status == "SHAPE"
    assert h.plan([100, 64, 24, 40])["kernels"]          # up to the last element is fine
    # whole axes keep collapsing: [B, S, H] sliced along S only is walked as [B] x [S * H]
    pb = PatternBuilder()
    B, S, H, r0, m = pb.dims(5)
    z = pb.static_start(0)
    pb.output(pb.op("neg", pb.slice(pb.param("f32", [B, S, H]), [z, r0, z], [B, m, H])))
    assert hctx.register(pb.build()).info["n_collapsed"] == 2
    # ... and sliced along H they do not
    pb = PatternBuilder()
    B, S, H, s0, n = pb.dims(5)
    pb.output(pb.op("neg", pb.slice(pb.param("f32", [B, S, H]), [z, z, s0], [B, S, n])))
    assert hctx.register(pb.build()).info["n_collapsed"] == 2      # [B * S] x [n]: B and S still merge
    for make, tmpl in ((qkv_split, "loop"), (softmax_of_window, "row_reduce"), (column_sum_of_rows_window, "col_reduce")):
        assert hctx.register(make()).info["template"] == tmpl
    # a slice of a computed value is not a producer-side indexing function: refused
    pb = PatternBuilder()
    T, H, s0, n = pb.dims(4)
    y = pb.op("neg", pb.param("f32", [T, H]))
    pb.output(pb.slice(y, [z, s0], [T, n]))
    with pytest.raises(DiscError) as e:
        hctx.register(pb.build())
    assert e.value.status == "BAD_PATTERN"


CASES = {
    "loop": (lambda: loop_slice()[0], [[100, 64, 8, 40], [7, 33, 5, 28], [1500, 1021, 3, 1013], [64, 4099, 1, 4097], [5, 9, 0, 9]]),
    "qkv": (qkv_split, [[100, 64, 192, 64, 128], [33, 100, 300, 100, 200], [2000, 768, 2304, 768, 1536], [9, 7, 21, 7, 14]]),
    "window_softmax": (softmax_of_window, [[4, 50, 64, 10, 20, 3, 40], [2, 9, 1000, 0, 9, 17, 777], [3, 700, 2100, 5, 600, 1, 2049],
                                            [1, 40, 9000, 7, 30, 100, 8192]]),
    "window_colsum": (column_sum_of_rows_window, [[100, 64, 10, 50], [3000, 520, 100, 2700], [17, 1000, 16, 1], [500, 33, 0, 500]]),
}


@pytest.mark.gpu
@pytest.mark.parametrize("which", sorted(CASES))
def test_slice_matches_oracle(which):
    from oracle import run as oracle_run
    from paper_2103_05288_amd import Context
    from tests.util import assert_close, run_gpu, to_oracle_input
    make, shapes = CASES[which]
    pat = make()
    ctx = Context(0)
    try:
        h = ctx.register(pat)
        gen = torch.Generator().manual_seed(5)
        for dims in shapes:
            ins = [torch.randn(pat.shape_of(pi, dims), generator=gen).to(TORCH_DTYPE[pat.ops[pi].dtype]) for pi in pat.params]
            got = run_gpu(h, pat, dims, ins)
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
            for k, (g, w) in enumerate(zip(got, want)):
                assert_close(g, w, f"{which} dims={dims} out{k} kernel={h.plan(dims)['kernels']}")
        assert h.info["compile_events"] == 1
    finally:
        ctx.close()
