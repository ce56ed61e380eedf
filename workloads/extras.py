"""Op lists beyond the five benchmark configurations: an op graph that is not one pattern and
patterns whose inputs enter through slices, pads and transposes.  Declarative only (what the
tests check against the oracle and bench.py times as its secondary figures)."""
from .pattern import PatternBuilder


def layernorm_backward_graph():
    """dx, dgamma, dbeta of LayerNorm from x, dy, gamma: three dependent row reductions for dx and two
    column reductions that need the normalised activations again -- row and column reductions in
    one op list, which is never one pattern."""
    pb = PatternBuilder("ln_bwd")
    T, H = pb.dims(2)
    x = pb.cast(pb.param("bf16", [T, H]), "f32")
    dy = pb.cast(pb.param("bf16", [T, H]), "f32")
    gam = pb.param("f32", [H])
    row = lambda v: pb.broadcast(v, [T, H], [0])
    col = lambda v: pb.broadcast(v, [T, H], [1])
    mean = pb.op("div", pb.reduce("sum", x, 1), pb.dim_size(H))
    xc = pb.op("sub", x, row(mean))
    var = pb.op("div", pb.reduce("sum", pb.op("mul", xc, xc), 1), pb.dim_size(H))
    rstd = pb.op("rsqrt", pb.op("add", var, pb.const(1e-5)))
    xhat = pb.op("mul", xc, row(rstd))
    g = pb.op("mul", dy, col(gam))
    c1 = pb.op("div", pb.reduce("sum", g, 1), pb.dim_size(H))
    c2 = pb.op("div", pb.reduce("sum", pb.op("mul", g, xhat), 1), pb.dim_size(H))
    dx = pb.op("mul", pb.op("sub", pb.op("sub", g, row(c1)), pb.op("mul", xhat, row(c2))), row(rstd))
    pb.output(pb.cast(dx, "bf16"))
    pb.output(pb.reduce("sum", pb.op("mul", dy, xhat), 0))     # dgamma
    pb.output(pb.reduce("sum", dy, 0))                          # dbeta
    return pb.build()


def qkv_split():
    """q, k, v are three slices of one [T, 3H] input; bias is a slice of a [3H] row vector."""
    pb = PatternBuilder("qkv")
    T, H, H3, s1, s2 = pb.dims(5)
    qkv = pb.param("bf16", [T, H3])
    bias = pb.param("f32", [H3])
    z = pb.static_start(0)
    f = lambda t: pb.cast(t, "f32")
    q = f(pb.slice(qkv, [z, z], [T, H]))
    k = f(pb.slice(qkv, [z, s1], [T, H]))
    v = f(pb.slice(qkv, [z, s2], [T, H]))
    bk = pb.broadcast(pb.slice(bias, [s1], [H]), [T, H], [1])
    pb.output(pb.cast(pb.op("add", pb.op("mul", q, pb.op("add", k, bk)), v), "bf16"))
    return pb.build()


def softmax_of_window():
    """Row softmax over a window [s0, s0 + n) of every row of a 3-D input, rows taken from a window
    of the middle axis as well."""
    pb = PatternBuilder("window_softmax")
    B, S, H, r0, m, s0, n = pb.dims(7)
    xs = pb.slice(pb.param("f16", [B, S, H]), [pb.static_start(0), r0, s0], [B, m, n])
    x = pb.cast(xs, "f32")
    e = pb.op("exp", pb.op("sub", x, pb.broadcast(pb.reduce("max", x, 2), [B, m, n], [0, 1])))
    pb.output(pb.cast(pb.op("div", e, pb.broadcast(pb.reduce("sum", e, 2), [B, m, n], [0, 1])), "f16"))
    return pb.build()


def padded_softmax():
    """Rows padded with -inf behind (and in front of) the data, then a softmax: the padding gets
    probability 0 and the data the softmax of the unpadded row."""
    pb = PatternBuilder("padded_softmax")
    T, H, l1, P = pb.dims(4)
    xp = pb.cast(pb.pad(pb.param("bf16", [T, H]), [pb.static_start(0), l1], [T, P], float("-inf")), "f32")
    e = pb.op("exp", pb.op("sub", xp, pb.broadcast(pb.reduce("max", xp, 1), [T, P], [0])))
    pb.output(pb.cast(pb.op("div", e, pb.broadcast(pb.reduce("sum", e, 1), [T, P], [0])), "bf16"))
    return pb.build()


def heads_softmax():
    """[B, S, NH, D] read as [B, NH, S, D] (the attention-head transpose), softmax over D."""
    pb = PatternBuilder("heads_softmax")
    B, S, NH, D = pb.dims(4)
    full = [B, NH, S, D]
    t = pb.cast(pb.transpose(pb.param("bf16", [B, S, NH, D]), (0, 2, 1, 3)), "f32")
    e = pb.op("exp", pb.op("sub", t, pb.broadcast(pb.reduce("max", t, 3), full, [0, 1, 2])))
    pb.output(pb.cast(pb.op("div", e, pb.broadcast(pb.reduce("sum", e, 3), full, [0, 1, 2])), "bf16"))
    return pb.build()


def pure_transpose(dtype, perm):
    pb = PatternBuilder("transpose" + "".join(str(a) for a in perm))
    pb.output(pb.transpose(pb.param(dtype, pb.dims(len(perm))), perm))
    return pb.build()


def gelu_backward_bias_gradient():
    """Backward of bias + GELU (the sigmoid form used by the C0 pattern family): dx = dy * gelu'(x + b)
    as bf16, and the bias gradient db = sum over the rows of dx -- an element-wise chain with a sum
    over the rows riding along."""
    pb = PatternBuilder("gelu_bwd_bias")
    T, H = pb.dims(2)
    dy = pb.cast(pb.param("bf16", [T, H]), "f32")
    x = pb.cast(pb.param("bf16", [T, H]), "f32")
    b = pb.param("f32", [H])
    u = pb.op("add", x, pb.broadcast(b, [T, H], [1]))
    a = pb.op("mul", u, pb.const(1.702))
    s = pb.op("sigmoid", a)
    g = pb.op("mul", s, pb.op("add", pb.const(1.0), pb.op("mul", a, pb.op("sub", pb.const(1.0), s))))
    dx = pb.op("mul", dy, g)
    pb.output(pb.cast(dx, "bf16"))
    pb.output(pb.reduce("sum", dx, 0))
    return pb.build()


def logsumexp_with_total_and_amax():
    """Per-row log-sum-exp of bf16 logits (two dependent row reductions), its sum over all rows (the
    normaliser part of a summed cross-entropy loss) and the largest |logit| of the whole tensor (the
    amax a scaling recipe tracks): two rank-0 outputs that reduce per-row values over the rows."""
    pb = PatternBuilder("lse_total_amax")
    T, H = pb.dims(2)
    x = pb.cast(pb.param("bf16", [T, H]), "f32")
    m = pb.reduce("max", x, 1)
    e = pb.op("exp", pb.op("sub", x, pb.broadcast(m, [T, H], [0])))
    lse = pb.op("add", pb.op("log", pb.reduce("sum", e, 1)), m)
    pb.output(lse)
    pb.output(pb.reduce("sum", lse, 0))
    pb.output(pb.reduce("max", pb.reduce("max", pb.op("abs", x), 1), 0))
    return pb.build()


def unique_of_sorted(dtype="i32"):
    """Unique of a sorted rank-1 tensor (Section 2 names Unique as the op whose output size depends on
    the input values): the distinct values in order, the index of every element in them, the count."""
    pb = PatternBuilder("unique_sorted")
    n = pb.dim()
    x = pb.param(dtype, [n])
    keep = pb.ne_prev(x)
    pb.output(pb.compact(x, keep))
    pb.output(pb.compact_rank(keep, "i32"))
    pb.output(pb.compact_count(keep, "i64"))
    return pb.build()
