"""Integer arithmetic and rounding casts on the GPU, bit-exact against the oracle: i32 / i64
add, sub, mul, div, max, min, neg, abs in the loop, row-reduce and column-reduce templates (values
beyond 2^24 and beyond 2^31, so a detour through fp32 or a missing wrap would show), and casts to
f16 / bf16 in the middle of a chain."""
import numpy as np
import pytest
import torch

from oracle import run as oracle_run
from workloads import PatternBuilder
from tests.util import assert_close, run_gpu, to_oracle_input

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2103_05288_amd import Context
    c = Context(0)
    yield c
    c.close()


def V(name):
    from paper_2103_05288_amd import VARIANTS
    return VARIANTS.index(name)


def check(ctx, pat, dims, ins, what, force=None):
    h = ctx.register(pat)
    if force is not None:
        ctx.force_variant(V(force))
    try:
        got = run_gpu(h, pat, dims, ins)
    finally:
        ctx.force_variant(-1)
    want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
    for k, (g, w) in enumerate(zip(got, want)):
        if not g.dtype.is_floating_point:
            assert np.array_equal(g.numpy().astype(np.int64), np.asarray(w).astype(np.int64)), \
                f"{what} dims={dims} out{k} force={force}: integer output differs"
        else:
            assert_close(g, w, f"{what} dims={dims} out{k} force={force}")
    return h


def _ints(shape, dtype, seed, lo_bits):
    """Seeded integers spread over [-2^lo_bits, 2^lo_bits), with small values mixed in."""
    g = torch.Generator().manual_seed(seed)
    big = torch.randint(-(1 << lo_bits), 1 << lo_bits, shape, generator=g, dtype=torch.int64)
    small = torch.randint(-9, 10, shape, generator=g, dtype=torch.int64)
    pick = torch.rand(shape, generator=g) < 0.3
    return torch.where(pick, small, big).to(dtype)


def _nonzero(t):
    return torch.where(t == 0, torch.full_like(t, 3), t)


@pytest.mark.parametrize("dtype,bits", [("i32", 31), ("i64", 62)])
def test_integer_loop_fusion_is_bit_exact(ctx, dtype, bits):
    tdt = torch.int32 if dtype == "i32" else torch.int64
    pb = PatternBuilder()
    t, h = pb.dims(2)
    a = pb.param(dtype, [t, h])
    b = pb.param(dtype, [t, h])
    r = pb.param(dtype, [h])
    rb = pb.broadcast(r, [t, h], [1])
    for oc in ("add", "sub", "mul", "div", "max", "min"):
        pb.output(pb.op(oc, a, b))
    pb.output(pb.op("neg", a))
    pb.output(pb.op("abs", a))
    pb.output(pb.op("add", pb.op("mul", a, rb), pb.const(-3.0, dtype), dims=[t, h]))
    pb.output(pb.op("sub", a, pb.op("neg", rb)))
    pb.output(pb.op("lt", a, b))
    pb.output(pb.op("select", pb.op("ge", a, rb), a, b))
    pb.output(pb.cast(a, "f32"))
    pat = pb.build()
    for dims, force in (([37, 129], None), ([5, 8], None), ([300, 77], "loop_scalar"), ([64, 256], "loop_vec_i64")):
        n = dims[0] * dims[1]
        av = _ints((dims[0], dims[1]), tdt, 3 + n, bits)
        bv = _nonzero(_ints((dims[0], dims[1]), tdt, 4 + n, bits // 2))
        rv = _ints((dims[1],), tdt, 5 + n, bits // 2)
        # (INT_MIN / -1 has no defined result; the draw cannot produce INT_MIN)
        print(f"[int loop] {dtype} dims={dims} force={force}", flush=True)
        check(ctx, pat, dims, [av, bv, rv], f"int loop {dtype}", force=force)


@pytest.mark.parametrize("dtype,bits", [("i32", 31), ("i64", 40)])
def test_integer_row_and_column_reductions_are_bit_exact(ctx, dtype, bits):
    tdt = torch.int32 if dtype == "i32" else torch.int64
    # row template: sum (wraps for i32), max, min of a*b + r, then an epilogue that uses them
    pb = PatternBuilder()
    t, h = pb.dims(2)
    a = pb.param(dtype, [t, h])
    r = pb.param(dtype, [h])
    v = pb.op("add", pb.op("mul", a, pb.const(3.0, dtype), dims=[t, h]), pb.broadcast(r, [t, h], [1]))
    s = pb.reduce("sum", v, 1)
    m = pb.reduce("max", v, 1)
    lo = pb.reduce("min", v, 1)
    pb.output(s)
    pb.output(m)
    pb.output(lo)
    pb.output(pb.op("sub", v, pb.broadcast(m, [t, h], [0])))
    pb.output(pb.op("div", pb.broadcast(s, [t, h], [0]), pb.op("max", pb.op("abs", v), pb.const(1.0, dtype), dims=[t, h])))
    row_pat = pb.build()
    for dims, force in (([33, 100], None), ([7, 1031], None), ([3, 5000], None), ([9, 300], "row_reg_scalar"), ([4, 700], "row_stream_vec")):
        av = _ints((dims[0], dims[1]), tdt, 11 + dims[1], bits)
        rv = _ints((dims[1],), tdt, 12 + dims[1], bits // 2)
        print(f"[int row] {dtype} dims={dims} force={force}", flush=True)
        check(ctx, row_pat, dims, [av, rv], f"int row {dtype}", force=force)
    # column template
    pb = PatternBuilder()
    t, h = pb.dims(2)
    a = pb.param(dtype, [t, h])
    s = pb.reduce("sum", a, 0)
    m = pb.reduce("max", a, 0)
    pb.output(s)
    pb.output(m)
    pb.output(pb.op("sub", a, pb.broadcast(m, [t, h], [1])))
    col_pat = pb.build()
    for dims, force in (([300, 64], None), ([5000, 257], None), ([2100, 600], "col_3stage_vec"), ([77, 33], "col_strip_scalar"),
                        ([3000, 130], "col_2stage_scalar")):
        av = _ints((dims[0], dims[1]), tdt, 21 + dims[1], bits)
        print(f"[int col] {dtype} dims={dims} force={force}", flush=True)
        check(ctx, col_pat, dims, [av], f"int col {dtype}", force=force)


def test_negative_constants_under_neg_and_abs(ctx):
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("f32", [n])
    xi = pb.param("i32", [n])
    pb.output(pb.op("add", x, pb.op("neg", pb.const(-1.5)), dims=[n]))
    pb.output(pb.op("mul", x, pb.op("abs", pb.const(-2.0)), dims=[n]))
    pb.output(pb.op("add", xi, pb.op("abs", pb.const(-3.0, "i32")), dims=[n]))
    pb.output(pb.op("sub", xi, pb.op("neg", pb.const(-7.0, "i32")), dims=[n]))
    pat = pb.build()
    g = torch.Generator().manual_seed(5)
    check(ctx, pat, [1000], [torch.randn(1000, generator=g), _ints((1000,), torch.int32, 6, 30)], "negative constants")


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_mid_chain_cast_rounds_like_the_unfused_sequence(ctx, kind):
    """x (fp32) -> cast to a 16-bit type -> arithmetic in fp32: the cast's rounding must be there.
    The cast's operand is an input, so both sides round the same fp32 value."""
    pb = PatternBuilder()
    t, h = pb.dims(2)
    x = pb.param("f32", [t, h])
    c = pb.cast(pb.cast(x, kind), "f32")
    pb.output(pb.op("mul", c, pb.const(3.0), dims=[t, h]))
    s = pb.reduce("sum", c, 1)
    pb.output(pb.op("sub", c, pb.broadcast(pb.op("div", s, pb.dim_size(h)), [t, h], [0])))
    pb.output(pb.cast(x, kind))
    pat = pb.build()
    g = torch.Generator().manual_seed(9)
    for dims in ([17, 100], [3, 2049]):
        xv = torch.randn(dims, generator=g) * 4.0
        xv[0, :4] = torch.tensor([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11])   # ties of both types
        check(ctx, pat, dims, [xv], f"mid-chain cast {kind}")
        # and the rounding is really there: the unrounded product differs from the output
        h_ = ctx.register(pat)
        got = run_gpu(h_, pat, dims, [xv])[0]
        assert not torch.equal(got, xv * 3.0)
