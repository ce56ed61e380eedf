"""Pins for the CPU oracle: what the mathematics fixes, independent of the oracle.

Every check compares the oracle with something that is not the oracle:
Python-scalar loops over ``math`` functions, ``math.fsum`` brute force, explicit
np.tile / np.repeat constructions, closed forms and invariants, and library
special cases (torch / scipy in float64).  The paper prints no worked numeric
example for its kernels, so there are no printed values to match.
"""
import itertools
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import OracleError, run
from workloads import PatternBuilder
from workloads.configs import (c0_pattern, c1_pattern, c2_pattern, c3_pattern, c4_pattern,
                               c1_inputs, c4_inputs)

rng = np.random.default_rng(7)


def _single(opcode, *arrays, dtype="f32"):
    """Pattern applying one element-wise op to same-shape rank-1 params."""
    pb = PatternBuilder()
    n = pb.dim()
    ps = [pb.param(dtype, [n]) for _ in arrays]
    pb.output(pb.op(opcode, *ps))
    return run(pb.build(), [len(arrays[0])], list(arrays))[0][0]


# ---------------------------------------------------------------- per-op pins
UNARY_REF = {
    "neg": lambda v: -v, "abs": abs, "exp": math.exp, "log": math.log, "tanh": math.tanh,
    "sqrt": math.sqrt, "rsqrt": lambda v: 1.0 / math.sqrt(v), "rcp": lambda v: 1.0 / v,
    "sigmoid": lambda v: 1.0 / (1.0 + math.exp(-v)), "erf": math.erf,
}


@pytest.mark.parametrize("opcode", sorted(UNARY_REF))
def test_unary_matches_python_math(opcode):
    x = rng.uniform(0.1, 3.0, 17) if opcode in ("log", "sqrt", "rsqrt", "rcp") else rng.normal(0, 2, 17)
    got = _single(opcode, x)
    ref = np.array([UNARY_REF[opcode](float(v)) for v in x])
    np.testing.assert_allclose(got, ref, rtol=1e-14, atol=0)


BINARY_REF = {
    "add": lambda a, b: a + b, "sub": lambda a, b: a - b, "mul": lambda a, b: a * b,
    "div": lambda a, b: a / b, "max": max, "min": min, "pow": lambda a, b: a ** b,
}


@pytest.mark.parametrize("opcode", sorted(BINARY_REF))
def test_binary_matches_python_scalars_and_operand_order(opcode):
    a = rng.uniform(0.5, 3.0, 13)
    b = rng.uniform(0.5, 3.0, 13)
    got = _single(opcode, a, b)
    ref = np.array([BINARY_REF[opcode](float(u), float(v)) for u, v in zip(a, b)])
    np.testing.assert_allclose(got, ref, rtol=1e-15, atol=0)
    if opcode in ("sub", "div", "pow"):          # a swapped operand must show
        assert not np.allclose(got, np.array([BINARY_REF[opcode](float(v), float(u)) for u, v in zip(a, b)]))


@pytest.mark.parametrize("opcode,fn", [("lt", lambda a, b: a < b), ("le", lambda a, b: a <= b),
                                       ("gt", lambda a, b: a > b), ("ge", lambda a, b: a >= b),
                                       ("eq", lambda a, b: a == b), ("ne", lambda a, b: a != b)])
def test_compare(opcode, fn):
    a = np.array([1.0, 2.0, 3.0, -1.0, 0.0])
    b = np.array([2.0, 2.0, 1.0, -1.0, -0.0])
    got = _single(opcode, a, b)
    assert got.dtype == np.bool_
    assert got.tolist() == [fn(float(u), float(v)) for u, v in zip(a, b)]


def test_select_orientation_and_nonzero_predicate():
    pb = PatternBuilder()
    n = pb.dim()
    p = pb.param("bool", [n])
    a = pb.param("f32", [n])
    b = pb.param("f32", [n])
    pb.output(pb.op("select", p, a, b))
    out = run(pb.build(), [4], [np.array([1, 0, 7, 0], dtype=np.uint8),
                                np.array([10., 11., 12., 13.]), np.array([20., 21., 22., 23.])])[0][0]
    assert out.tolist() == [10., 21., 12., 23.]      # true (any nonzero) picks the first value


def test_cast_rules():
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("f32", [n])
    pb.output(pb.cast(x, "i32"))
    pb.output(pb.cast(x, "bf16"))
    pb.output(pb.cast(x, "bool"))
    xs = np.array([-1.7, -0.2, 0.0, 0.9, 2.5, 1.0 + 2.0 ** -20])
    i, f, b = run(pb.build(), [6], [xs])[0]
    assert i.tolist() == [-1, 0, 0, 0, 2, 1] and i.dtype == np.int64   # truncation toward zero
    assert np.array_equal(f, xs)                                         # float casts do not round
    assert b.tolist() == [True, True, False, True, True, True]


def test_const_and_dim_size_scalars():
    pb = PatternBuilder()
    t, h = pb.dims(2)
    x = pb.param("f32", [t, h])
    y = pb.op("add", pb.op("mul", x, pb.const(3.0)), pb.dim_size(h))
    z = pb.op("sub", pb.dim_size(t), y, dims=[t, h])
    pb.output(z)
    xs = rng.normal(size=(3, 5))
    out = run(pb.build(), [3, 5], [xs])[0][0]
    np.testing.assert_allclose(out, 3.0 - (xs * 3.0 + 5.0), rtol=1e-15)


# ---------------------------------------------------------------- broadcast
def test_broadcast_equals_explicit_tiling():
    pb = PatternBuilder()
    a, b, c = pb.dims(3)
    v_b = pb.param("f32", [b])
    v_ac = pb.param("f32", [a, c])
    v_a1c = pb.param("f32", [a, pb.static(1), c])
    pb.output(pb.broadcast(v_b, [a, b, c], [1]))
    pb.output(pb.broadcast(v_ac, [a, b, c], [0, 2]))
    pb.output(pb.broadcast(v_a1c, [a, b, c], [0, 1, 2]))
    A, B, C = 2, 3, 4
    xb = rng.normal(size=B)
    xac = rng.normal(size=(A, C))
    xa1c = rng.normal(size=(A, 1, C))
    o1, o2, o3 = run(pb.build(), [A, B, C], [xb, xac, xa1c])[0]
    assert np.array_equal(o1, np.tile(xb.reshape(1, B, 1), (A, 1, C)))
    assert np.array_equal(o2, np.repeat(xac[:, None, :], B, axis=1))
    assert np.array_equal(o3, np.repeat(xa1c, B, axis=1))
    # element-by-element definition
    for i, j, k in itertools.product(range(A), range(B), range(C)):
        assert o1[i, j, k] == xb[j] and o2[i, j, k] == xac[i, k] and o3[i, j, k] == xa1c[i, 0, k]


def test_broadcast_rejects_mismatch_and_implicit_numpy_broadcast():
    pb = PatternBuilder()
    a, b = pb.dims(2)
    x = pb.param("f32", [a])
    pb.output(pb.broadcast(x, [a, b], [1]))       # maps axis of size a onto axis of size b
    with pytest.raises(OracleError):
        run(pb.build(), [2, 3], [np.zeros(2)])
    pb = PatternBuilder()
    a, b = pb.dims(2)
    x = pb.param("f32", [a, b])
    y = pb.param("f32", [b])
    pb.output(pb.op("add", x, y))                 # no explicit broadcast: not allowed
    with pytest.raises(OracleError):
        run(pb.build(), [2, 3], [np.zeros((2, 3)), np.zeros(3)])


# ---------------------------------------------------------------- reductions
@pytest.mark.parametrize("axis", [0, 1, 2])
def test_reductions_equal_brute_force(axis):
    shape = (3, 4, 5)
    x = rng.normal(size=shape)
    pb = PatternBuilder()
    d = pb.dims(3)
    p = pb.param("f32", d)
    for kind in ("sum", "max", "min", "argmax"):
        pb.output(pb.reduce(kind, p, axis))
    s, mx, mn, am = run(pb.build(), shape, [x])[0]
    rest = [r for k, r in enumerate(shape) if k != axis]
    assert s.shape == tuple(rest)
    for idx in itertools.product(*[range(r) for r in rest]):
        sl = list(idx)
        sl.insert(axis, slice(None))
        line = [float(v) for v in x[tuple(sl)]]
        assert abs(s[idx] - math.fsum(line)) <= 1e-15 * sum(abs(v) for v in line)
        assert mx[idx] == max(line) and mn[idx] == min(line)
        assert am[idx] == line.index(max(line))


def test_reduce_size_one_and_empty_axis():
    pb = PatternBuilder()
    d = pb.dims(2)
    p = pb.param("f32", d)
    pb.output(pb.reduce("sum", p, 1))
    x = rng.normal(size=(4, 1))
    assert np.array_equal(run(pb.build(), [4, 1], [x])[0][0], x[:, 0])
    with pytest.raises(OracleError):
        run(pb.build(), [4, 0], [np.zeros((4, 0))])
    assert run(pb.build(), [0, 3], [np.zeros((0, 3))])[0][0].shape == (0,)


def test_argmax_planted_maxima_and_ties():
    pb = PatternBuilder()
    d = pb.dims(2)
    p = pb.param("f32", d)
    pb.output(pb.reduce("argmax", p, 1))
    x = rng.normal(size=(6, 9))
    want = [3, 0, 8, 5, 5, 1]
    for r, c in enumerate(want):
        x[r, c] = 10.0
    x[3, 7] = 10.0      # tie after the planted one: lowest index wins
    x[4, 2] = 10.0      # tie before the planted one
    want[4] = 2
    got = run(pb.build(), [6, 9], [x])[0][0]
    assert got.dtype == np.int64 and got.tolist() == want
    assert got.tolist() == np.argmax(x, axis=1).tolist()


# ---------------------------------------------------------------- C0 GELU
def _c0(x, b, r):
    return run(c0_pattern(), list(x.shape), [x, b, r])[0][0]


def test_c0_gelu_closed_forms():
    H = 5
    zero = np.zeros(H)
    u = rng.normal(0, 2, size=(4, H))
    g = _c0(u, zero, np.zeros_like(u))
    gm = _c0(-u, zero, np.zeros_like(u))
    np.testing.assert_allclose(g - gm, u, rtol=0, atol=1e-15)      # tanh is odd => g(u) - g(-u) = u
    assert _c0(np.zeros((1, H)), zero, np.zeros((1, H))).tolist() == [[0.0] * H]
    big = np.full((1, H), 12.0)
    np.testing.assert_allclose(_c0(big, zero, np.zeros((1, H))), big, rtol=1e-15)
    assert np.all(np.abs(_c0(-big, zero, np.zeros((1, H)))) < 1e-15)


def test_c0_matches_scalar_loop_and_torch():
    T, H = 3, 7
    x = rng.normal(size=(T, H))
    b = rng.normal(0, 0.02, size=H)
    r = rng.normal(size=(T, H))
    got = _c0(x, b, r)
    for t in range(T):
        for h in range(H):
            u = x[t, h] + b[h]
            ref = 0.5 * u * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (u + 0.044715 * u ** 3))) + r[t, h]
            assert abs(got[t, h] - ref) < 1e-14
    ref = torch.nn.functional.gelu(torch.from_numpy(x + b), approximate="tanh").numpy() + r
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- C1 softmax
def _c1(x, mask):
    B, NH, S, _ = x.shape
    return run(c1_pattern(), [B, NH, S], [x, mask])[0][0]


def test_c1_rows_sum_to_one_and_shift_invariance():
    x, mask = [t.double().numpy() for t in c1_inputs([2, 3, 11], seed=5)]
    y = _c1(x, mask)
    np.testing.assert_allclose(y.sum(-1), 1.0, rtol=0, atol=1e-12)
    shift = rng.normal(size=(2, 3, 11, 1)) * 8.0          # x*0.125 shifts by a per-row constant
    np.testing.assert_allclose(_c1(x + shift, mask), y, rtol=1e-12, atol=1e-15)


def test_c1_constant_row_and_masked_equals_textbook_softmax_of_valid_slice():
    B, NH, S = 2, 2, 9
    lens = [4, 9]
    mask = np.zeros((B, 1, 1, S))
    for b, L in enumerate(lens):
        mask[b, 0, 0, L:] = -1.0e4
    y = _c1(np.full((B, NH, S, S), 0.37), mask)
    for b, L in enumerate(lens):
        np.testing.assert_allclose(y[b, :, :, :L], 1.0 / L, rtol=1e-15)
        assert np.all(y[b, :, :, L:] == 0.0)               # exp(-1e4) underflows to exactly 0
    x = rng.normal(size=(B, NH, S, S))
    y = _c1(x, mask)
    for b, L in enumerate(lens):
        ref = scipy.special.softmax(x[b, :, :, :L] * 0.125, axis=-1)
        np.testing.assert_allclose(y[b, :, :, :L], ref, rtol=1e-14, atol=0)
        ref_t = torch.softmax(torch.from_numpy(x[b, :, :, :L] * 0.125), dim=-1).numpy()
        np.testing.assert_allclose(y[b, :, :, :L], ref_t, rtol=1e-14, atol=0)


# ---------------------------------------------------------------- C2 LayerNorm
def test_c2_pre_affine_moments_and_torch_special_case():
    T, H = 5, 33
    pat = c2_pattern()
    x = rng.normal(size=(T, H))
    r = rng.normal(size=(T, H))
    b = rng.normal(size=H)
    gamma = rng.normal(1, 0.1, size=H)
    beta = rng.normal(0, 0.1, size=H)
    outs, vals = run(pat, [T, H], [x, r, b, gamma, beta])
    # the normalised value n is the operand of the first multiply by broadcast(gamma)
    n = None
    for i, op in enumerate(pat.ops):
        if op.opcode == "mul" and pat.ops[op.ins[1]].opcode == "broadcast" and pat.ops[op.ins[0]].opcode == "mul":
            n = vals[op.ins[0]]
    assert n is not None
    v = x + r + b
    var = v.var(axis=1)                                  # population variance
    np.testing.assert_allclose(n.mean(axis=1), 0.0, atol=1e-14)
    np.testing.assert_allclose(n.var(axis=1), var / (var + 1e-5), rtol=1e-12)
    np.testing.assert_allclose(n.var(axis=1), 1.0, atol=1e-4)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(v), (H,), torch.from_numpy(gamma),
                                         torch.from_numpy(beta), eps=1e-5).numpy()
    np.testing.assert_allclose(outs[0], ref, rtol=1e-12, atol=1e-13)
    # gamma = 1, beta = 0, r = b = 0 reduces to the library's plain layer_norm
    o = run(pat, [T, H], [x, np.zeros((T, H)), np.zeros(H), np.ones(H), np.zeros(H)])[0][0]
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (H,), eps=1e-5).numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-12, atol=1e-13)


def test_c2_constant_row_gives_beta():
    T, H = 2, 8
    beta = rng.normal(size=H)
    o = run(c2_pattern(), [T, H], [np.full((T, H), 0.75), np.zeros((T, H)), np.zeros(H),
                                   rng.normal(1, 0.1, size=H), beta])[0][0]
    np.testing.assert_allclose(o, np.tile(beta, (T, 1)), rtol=0, atol=1e-15)


# ---------------------------------------------------------------- C3 column reduction
def test_c3_invariants():
    pat = c3_pattern()
    T, C = 37, 6
    x = rng.uniform(-1, 1, size=(T, C))
    s, mean, y = run(pat, [T, C], [x])[0]
    for c in range(C):
        assert abs(s[c] - math.fsum(float(v) for v in x[:, c])) < 1e-14
        assert abs(mean[c] - math.fsum(float(v) for v in x[:, c]) / T) < 1e-15
    np.testing.assert_allclose(y.sum(axis=0), 0.0, atol=1e-9 * T)
    np.testing.assert_allclose(y, x - x.mean(axis=0, keepdims=True), atol=1e-15)
    s, mean, y = run(pat, [T, C], [np.ones((T, C))])[0]
    assert np.all(s == T) and np.all(mean == 1.0) and np.all(y == 0.0)
    x1 = rng.uniform(-1, 1, size=(1, C))
    s, mean, y = run(pat, [1, C], [x1])[0]
    assert np.array_equal(s, x1[0]) and np.array_equal(mean, x1[0]) and np.all(y == 0.0)


# ---------------------------------------------------------------- C4 mixed chain
def _c4(x, mask, bH, cT):
    T, H = x.shape
    return run(c4_pattern(), [T, H], [x, mask, bH, cT])


def _c4_named(pat, vals):
    """Pick p (the div), q (the select), s (the row sum), w (rsqrt) out of the intermediates."""
    named = {}
    for i, op in enumerate(pat.ops):
        if op.opcode == "div":
            named["p"] = vals[i]
        elif op.opcode == "select":
            named["q"] = vals[i]
        elif op.opcode == "reduce_sum":
            named["s"] = vals[i]
        elif op.opcode == "rsqrt":
            named["w"] = vals[i]
        elif op.opcode == "cast" and op.dtype == "f32":
            named["x32"] = vals[i]
    return named


def test_c4_invariants():
    pat = c4_pattern()
    T, H = 6, 19
    x, mask, bH, cT = [t.double().numpy() for t in c4_inputs([T, H], seed=3)]
    mask[0, :] = 0
    outs, vals = _c4(x, mask, bH, cT)
    nm = _c4_named(pat, vals)
    p, q, s, w, x32 = nm["p"], nm["q"], nm["s"], nm["w"], nm["x32"]
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-12)
    np.testing.assert_allclose(q.sum(axis=1), 1.0 - (p * (mask != 0)).sum(axis=1), atol=1e-12)
    assert np.all(s >= 1.0) and np.all(s <= H)            # the max term contributes exp(0) = 1
    np.testing.assert_allclose(w, s ** -0.5, rtol=1e-15)
    y32 = outs[0]
    np.testing.assert_allclose(y32 - x32 * w[:, None], q, atol=1e-14)
    assert np.all(q[mask != 0] == 0.0)                    # true => zeroed
    np.testing.assert_allclose(y32[mask != 0], (x32 * w[:, None])[mask != 0], rtol=1e-15)
    # p, q do not depend on the per-row shift cT
    outs2, vals2 = _c4(x, mask, bH, cT + rng.normal(size=(T, 1)))
    np.testing.assert_allclose(_c4_named(pat, vals2)["p"], p, rtol=1e-11, atol=1e-16)
    # mask all false, bH = 0: p is the textbook softmax of x
    outs3, vals3 = _c4(x, np.zeros_like(mask), np.zeros(H), cT)
    np.testing.assert_allclose(_c4_named(pat, vals3)["p"], scipy.special.softmax(x, axis=1), rtol=1e-12)
    # and the whole chain against a direct transcription with scalar loops on one row
    t = 2
    b = [x[t, h] + bH[h] + cT[t, 0] for h in range(H)]
    m = max(b)
    e = [math.exp(v - m) for v in b]
    ssum = math.fsum(e)
    for h in range(H):
        qh = 0.0 if mask[t, h] else e[h] / ssum
        assert abs(y32[t, h] - (qh + x[t, h] / math.sqrt(ssum))) < 1e-14


# ---------------------------------------------------------------- dynamic slice (Section 4.1)
def _slice_pattern(rank, static_axes=()):
    """out = slice(x): start and size of every axis are runtime values, except the axes in
    ``static_axes``, which start at the static index 1 and have the static size 2."""
    pb = PatternBuilder()
    src = pb.dims(rank)
    starts, sizes = [], []
    for k in range(rank):
        if k in static_axes:
            starts.append(pb.static_start(1))
            sizes.append(pb.static(2))
        else:
            starts.append(pb.dim())
            sizes.append(pb.dim())
    x = pb.param("f32", src)
    pb.output(pb.slice(x, starts, sizes))
    return pb.build(), starts, sizes


def test_slice_matches_index_loops():
    """Brute force: every element of the result by explicit index arithmetic."""
    for rank, static_axes in ((1, ()), (2, ()), (3, (1,)), (2, (0, 1))):
        pat, starts, sizes = _slice_pattern(rank, static_axes)
        shape = (5, 4, 6)[:rank]
        x = rng.normal(size=shape)
        dims = [0] * pat.n_dims
        for k in range(rank):
            dims[k] = shape[k]
        st = [1, 0, 2][:rank]
        sz = [3, 4, 3][:rank]
        for k in range(rank):
            if k in static_axes:
                st[k], sz[k] = 1, 2
            else:
                dims[starts[k]], dims[sizes[k]] = st[k], sz[k]
        out = run(pat, dims, [x])[0][0]
        assert out.shape == tuple(sz)
        for idx in itertools.product(*[range(n) for n in sz]):
            assert out[idx] == x[tuple(s + i for s, i in zip(st, idx))]


def test_slice_identity_tiling_and_bounds():
    pat, starts, sizes = _slice_pattern(2)
    x = rng.normal(size=(7, 9))

    def sl(s0, n0, s1, n1):
        d = [0] * pat.n_dims
        d[0], d[1] = 7, 9
        d[starts[0]], d[sizes[0]], d[starts[1]], d[sizes[1]] = s0, n0, s1, n1
        return run(pat, d, [x])[0][0]

    assert np.array_equal(sl(0, 7, 0, 9), x)                                   # the whole operand
    # adjacent slices tile the operand: gluing them back gives the operand (the Split case)
    assert np.array_equal(np.concatenate([sl(0, 7, 0, 4), sl(0, 7, 4, 5)], axis=1), x)
    assert np.array_equal(np.concatenate([sl(0, 2, 0, 9), sl(2, 5, 0, 9)], axis=0), x)
    assert sl(3, 0, 0, 9).shape == (0, 9)                                      # an empty slice is legal
    for bad in ((0, 8, 0, 9), (1, 7, 0, 9), (0, 7, 5, 5)):
        with pytest.raises(OracleError):
            sl(*bad)
    # a slice is a producer like any other value: softmax over the second half of each row
    pb = PatternBuilder()
    T, H, s0, n = pb.dims(4)
    xs = pb.slice(pb.param("f32", [T, H]), [pb.static_start(0), s0], [T, n])
    e = pb.op("exp", pb.op("sub", xs, pb.broadcast(pb.reduce("max", xs, 1), [T, n], [0])))
    pb.output(pb.op("div", e, pb.broadcast(pb.reduce("sum", e, 1), [T, n], [0])))
    got = run(pb.build(), [7, 9, 4, 5], [x])[0][0]
    np.testing.assert_allclose(got, scipy.special.softmax(x[:, 4:], axis=1), rtol=1e-13)


# ---------------------------------------------------------------- dynamic pad (Section 4.1)
def _pad_pattern(rank, value):
    pb = PatternBuilder()
    src = pb.dims(rank)
    low = pb.dims(rank)
    sizes = pb.dims(rank)
    x = pb.param("f32", src)
    pb.output(pb.pad(x, low, sizes, value))
    return pb.build()


def test_pad_matches_index_loops_and_inverts_slice():
    for rank in (1, 2, 3):
        pat = _pad_pattern(rank, -2.5)
        shape = (3, 4, 2)[:rank]
        low = (2, 0, 1)[:rank]
        size = (7, 4, 5)[:rank]
        x = rng.normal(size=shape)
        out = run(pat, list(shape) + list(low) + list(size), [x])[0][0]
        assert out.shape == tuple(size)
        for idx in itertools.product(*[range(n) for n in size]):
            src = tuple(i - l for i, l in zip(idx, low))
            inside = all(0 <= s < d for s, d in zip(src, shape))
            assert out[idx] == (x[src] if inside else -2.5)
        # slicing the padded result at the same offsets gives the operand back
        assert np.array_equal(out[tuple(slice(l, l + d) for l, d in zip(low, shape))], x)
        # numpy's own pad agrees
        ref = np.pad(x, [(l, n - l - d) for l, n, d in zip(low, size, shape)], constant_values=-2.5)
        assert np.array_equal(out, ref)
    pat = _pad_pattern(1, 0.0)
    x = rng.normal(size=5)
    assert np.array_equal(run(pat, [5, 0, 5], [x])[0][0], x)          # no padding at all
    assert run(pat, [0, 0, 4], [np.zeros(0)])[0][0].tolist() == [0.0] * 4   # an empty operand: padding only
    for bad in ([5, 1, 5], [5, 0, 4]):
        with pytest.raises(OracleError):
            run(pat, bad, [x])
    # softmax with -inf padding behind each row equals softmax of the row, zeros in the padding
    pb = PatternBuilder()
    T, H, P = pb.dims(3)
    xp = pb.pad(pb.param("f32", [T, H]), [pb.static_start(0), pb.static_start(0)], [T, P], float("-inf"))
    e = pb.op("exp", pb.op("sub", xp, pb.broadcast(pb.reduce("max", xp, 1), [T, P], [0])))
    pb.output(pb.op("div", e, pb.broadcast(pb.reduce("sum", e, 1), [T, P], [0])))
    x2 = rng.normal(size=(4, 6))
    got = run(pb.build(), [4, 6, 9], [x2])[0][0]
    np.testing.assert_allclose(got[:, :6], scipy.special.softmax(x2, axis=1), rtol=1e-13)
    assert np.all(got[:, 6:] == 0.0)


def test_pad_value_has_the_operands_type():
    """The padding value is a scalar of the operand's element type: 0.654... is not a bf16 / f16 /
    f32 number and arrives as the nearest one (torch's conversion as the independent reference)."""
    for dtype, tdt in (("bf16", torch.bfloat16), ("f16", torch.float16), ("f32", torch.float32)):
        for value in (0.6540060516381072, -1.0e-3, 3.0, float("-inf"), 1.00390625, 1.01171875):   # the last two: bf16 ties
            pb = PatternBuilder()
            H, P = pb.dims(2)
            pb.output(pb.pad(pb.param(dtype, [H]), [pb.static_start(0)], [P], value))
            out = run(pb.build(), [2, 5], [np.zeros(2)])[0][0]
            assert out[2] == out[3] == out[4] == float(torch.tensor(value, dtype=torch.float64).to(tdt).double())


def test_transpose_matches_index_loops():
    for perm in ((1, 0), (0, 2, 1), (2, 0, 1), (1, 0, 2, 3), (3, 2, 1, 0)):
        rank = len(perm)
        shape = (3, 4, 2, 5)[:rank]
        pb = PatternBuilder()
        x = pb.param("f32", pb.dims(rank))
        t = pb.transpose(x, perm)
        pb.output(t)
        xa = rng.normal(size=shape)
        out = run(pb.build(), list(shape), [xa])[0][0]
        assert out.shape == tuple(shape[a] for a in perm)
        for idx in itertools.product(*[range(n) for n in out.shape]):
            src = [0] * rank
            for k, a in enumerate(perm):
                src[a] = idx[k]
            assert out[idx] == xa[tuple(src)]
        assert np.array_equal(out, torch.from_numpy(xa).permute(*perm).numpy())
    # the inverse permutation undoes it
    pb = PatternBuilder()
    B, S, H = pb.dims(3)
    x = pb.param("f32", [B, S, H])
    t = pb.transpose(x, (2, 0, 1))               # [H, B, S]
    pb.output(pb.op("neg", t))
    xa = rng.normal(size=(2, 3, 4))
    out = run(pb.build(), [2, 3, 4], [xa])[0][0]
    assert np.array_equal(np.transpose(-out, (1, 2, 0)), xa)


def test_backward_workloads_equal_autograd():
    """The two backward workloads of workloads/extras.py, run by the oracle over their op lists,
    against reverse-mode differentiation of the forward functions in fp64 (torch.autograd): pins
    the op lists themselves (a dropped term or a swapped operand in the hand-written gradient
    formulas fails here) and the oracle's handling of row and column reductions in one list."""
    from workloads.extras import gelu_backward_bias_gradient, layernorm_backward_graph
    g = torch.Generator().manual_seed(31)
    T, H = 9, 13
    # inputs that are exact in their storage types, so the oracle and autograd see the same values
    x = torch.randn(T, H, generator=g).bfloat16().double()
    dy = torch.randn(T, H, generator=g).bfloat16().double()
    gam = torch.randn(H, generator=g).float().double()

    xr = x.clone().requires_grad_(True)
    gr = gam.clone().requires_grad_(True)
    beta = torch.zeros(H, dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.layer_norm(xr, (H,), gr, beta, eps=1e-5)
    y.backward(dy)
    out = run(layernorm_backward_graph(), [T, H], [x.numpy(), dy.numpy(), gam.numpy()])[0]
    # dx is stored as bf16 (8 significant bits); dgamma and dbeta are fp32 sums
    np.testing.assert_allclose(np.asarray(out[0], dtype=np.float64), xr.grad.numpy(), rtol=2.0 ** -8, atol=1e-6)
    np.testing.assert_allclose(np.asarray(out[1], dtype=np.float64), gr.grad.numpy(), rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(np.asarray(out[2], dtype=np.float64), beta.grad.numpy(), rtol=1e-6, atol=1e-6)

    b = torch.randn(H, generator=g).float().double()
    xr = x.clone().requires_grad_(True)
    br = b.clone().requires_grad_(True)
    u = xr + br
    (u * torch.sigmoid(1.702 * u)).backward(dy)
    out = run(gelu_backward_bias_gradient(), [T, H], [dy.numpy(), x.numpy(), b.numpy()])[0]
    np.testing.assert_allclose(np.asarray(out[0], dtype=np.float64), xr.grad.numpy(), rtol=2.0 ** -8, atol=1e-6)
    np.testing.assert_allclose(np.asarray(out[1], dtype=np.float64), br.grad.numpy(), rtol=1e-6, atol=1e-6)


def test_reduction_of_per_row_values_to_one_number():
    """A rank-1 value reduced over its only axis gives a rank-0 result: against Python's own sum /
    max / min over a list, for a chain of two reductions of a matrix."""
    rng = np.random.default_rng(3)
    x = rng.standard_normal((6, 5))
    for inner, outer, py_in, py_out in (("sum", "sum", sum, sum), ("max", "min", max, min), ("min", "max", min, max), ("max", "sum", max, sum)):
        pb = PatternBuilder()
        t, h = pb.dims(2)
        v = pb.param("f32", [t, h])
        r = pb.reduce(inner, v, 1)
        pb.output(r)
        pb.output(pb.reduce(outer, r, 0))
        out = run(pb.build(), [6, 5], [x])[0]
        rows = [py_in(float(a) for a in x[i]) for i in range(6)]
        assert np.asarray(out[1]).shape == ()
        assert float(out[1]) == pytest.approx(py_out(rows), rel=1e-6, abs=1e-6)


# ---------------------------------------------------------------- integer arithmetic
def _wrap_py(v: int, bits: int) -> int:
    """Two's complement of a Python int, written with Python's own arithmetic."""
    v &= (1 << bits) - 1
    return v - (1 << bits) if v >> (bits - 1) else v


def _trunc_div(a: int, b: int) -> int:
    """C-style division from exact rationals: toward zero (Python's // floors)."""
    from fractions import Fraction
    return math.trunc(Fraction(a, b))


INT_REF = {
    "add": lambda a, b: a + b, "sub": lambda a, b: a - b, "mul": lambda a, b: a * b,
    "div": _trunc_div, "max": max, "min": min,
}
# values beyond 2^24 (a detour through fp32 would show), beyond 2^31 for i64, all sign combinations,
# exact multiples and non-multiples
INT_A = [7, -7, 7, -7, 0, 123456789, -123456789, 2147483647, -2147483647, 40000, -65536, 99, 1 << 30, 16777217, -16777219, 6]
INT_B = [2, 2, -2, -2, 5, 1000, 1000, 3, -3, 50000, 65536, -99, 4, -16777213, 3, -3]


@pytest.mark.parametrize("dtype,bits", [("i32", 32), ("i64", 64)])
@pytest.mark.parametrize("opcode", sorted(INT_REF))
def test_integer_binary_ops_match_python_ints(opcode, dtype, bits):
    a = np.array(INT_A, dtype=np.int64)
    b = np.array(INT_B, dtype=np.int64)
    if dtype == "i64":
        a = a * 3000000007 + 1
        b = np.where(np.abs(b) > 1000, b * 1000003, b)
    got = _single(opcode, a, b, dtype=dtype)
    assert got.dtype == np.int64
    ref = [_wrap_py(INT_REF[opcode](int(u), int(v)), bits) for u, v in zip(a, b)]
    assert got.tolist() == ref
    if opcode in ("sub", "div"):
        assert got.tolist() != [_wrap_py(INT_REF[opcode](int(v), int(u)), bits) if u != 0 else 0 for u, v in zip(a, b)]


def test_integer_division_truncates_toward_zero_for_all_signs():
    cases = [(7, 2, 3), (-7, 2, -3), (7, -2, -3), (-7, -2, 3), (6, 3, 2), (-6, 3, -2), (6, -3, -2), (-6, -3, 2),
             (1, 5, 0), (-1, 5, 0), (0, -5, 0), (2147483647, -1, -2147483647)]
    a = np.array([c[0] for c in cases]); b = np.array([c[1] for c in cases])
    for dt in ("i32", "i64"):
        assert _single("div", a, b, dtype=dt).tolist() == [c[2] for c in cases]


def test_i32_results_wrap_and_i64_results_do_not():
    a = np.array([2147483647, -2147483648, 65536, 2147483647])
    b = np.array([1, -1, 65536, 2147483647])
    assert _single("add", a, b, dtype="i32").tolist() == [-2147483648, 2147483647, 131072, -2]
    assert _single("mul", a, b, dtype="i32").tolist() == [2147483647, -2147483648, 0, 1]
    assert _single("add", a, b, dtype="i64").tolist() == [2147483648, -2147483649, 131072, 4294967294]
    assert _single("mul", a, b, dtype="i64").tolist() == [2147483647, 2147483648, 1 << 32, 2147483647 ** 2]
    # neg / abs of integers stay integers
    x = np.array([5, -5, 0, -2147483647])
    assert _single("neg", x, dtype="i32").tolist() == [-5, 5, 0, 2147483647]
    assert _single("abs", x, dtype="i64").tolist() == [5, 5, 0, 2147483647]


def test_binary_operands_take_the_result_type():
    """An op's operands are converted to the element type of its result first: integer operands
    of a float division divide as floats, an i64 operand of an i32 op is wrapped before the op."""
    pb = PatternBuilder()
    n = pb.dim()
    a = pb.param("i32", [n])
    b = pb.param("i64", [n])
    pb.output(pb.op("div", a, b, dtype="f32"))
    pb.output(pb.op("div", a, b, dtype="i64"))
    pb.output(pb.op("max", a, b, dtype="i32"))
    pb.output(pb.op("lt", a, b))
    m = pb.param("bool", [n])
    pb.output(pb.op("select", m, a, b, dtype="i32"))
    pb.output(pb.op("add", pb.cast(m, "i32"), a))
    av = np.array([7, -7, 9, 5]); bv = np.array([2, 2, (1 << 32) + 3, -4]); mv = np.array([1, 0, 0, 1], dtype=np.uint8)
    o = run(pb.build(), [4], [av, bv, mv])[0]
    assert o[0].dtype == np.float64 and o[0].tolist() == [3.5, -3.5, 9 / ((1 << 32) + 3), -1.25]
    assert o[1].tolist() == [3, -3, 0, -1]
    assert o[2].tolist() == [7, 2, 9, 5]              # max(9, wrap32(2^32 + 3) = 3) = 9
    assert o[3].tolist() == [False, True, True, False]   # compared as 64-bit integers
    assert o[4].tolist() == [7, 2, 3, 5]
    assert o[5].tolist() == [8, -7, 9, 6]


def test_integer_reductions_and_casts():
    pb = PatternBuilder()
    t, h = pb.dims(2)
    x = pb.param("i32", [t, h])
    pb.output(pb.reduce("sum", x, 1))
    pb.output(pb.reduce("max", x, 1))
    pb.output(pb.reduce("min", x, 0))
    pb.output(pb.reduce("sum", pb.cast(x, "i64"), 1))
    f = pb.param("f32", [t, h])
    pb.output(pb.cast(f, "i32"))
    pb.output(pb.cast(pb.cast(x, "i64"), "i32"))
    xv = np.array([[2147483647, 1, 5], [-3, -4, 16777217]])
    fv = np.array([[2.9, -2.9, 0.5], [-0.5, 1e9, -16777216.0]])
    o = run(pb.build(), [2, 3], [xv, fv])[0]
    assert o[0].tolist() == [_wrap_py(2147483647 + 1 + 5, 32), 16777210]
    assert o[1].tolist() == [2147483647, 16777217]
    assert o[2].tolist() == [-3, -4, 5]
    assert o[3].tolist() == [2147483653, 16777210]
    assert o[4].tolist() == [[2, -2, 0], [0, 1000000000, -16777216]]
    assert o[5].tolist() == xv.tolist()


# ---------------------------------------------------------------- a cast to a 16-bit float type mid-chain rounds
def _bf16_rne_py(v: float) -> float:
    """Nearest bf16 value, ties to even, from exact rational arithmetic (normal range)."""
    from fractions import Fraction
    if v == 0 or not math.isfinite(v):
        return v
    fr = Fraction(v)
    e = math.floor(math.log2(abs(v)))
    if Fraction(2) ** e > abs(fr):
        e -= 1
    q = Fraction(2) ** (e - 7)                  # spacing of values with 8 significant bits
    n = fr / q
    lo = math.floor(n)
    r = n - lo
    k = lo + 1 if r > Fraction(1, 2) or (r == Fraction(1, 2) and lo % 2 == 1) else lo
    return float(k * q)


def test_mid_chain_cast_to_16_bit_rounds_and_output_cast_does_not():
    xs = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 3.14159, -2.71828, 1e-3, 65504.0, 1.0 + 2.0 ** -9, 1.0 + 2.0 ** -11 + 2.0 ** -12])
    xs = xs.astype(np.float32).astype(np.float64)
    for kind, ref in (("bf16", _bf16_rne_py), ("f16", lambda v: float(np.float16(v)))):
        pb = PatternBuilder()
        n = pb.dim()
        x = pb.param("f32", [n])
        c = pb.cast(x, kind)
        pb.output(pb.op("mul", pb.cast(c, "f32"), pb.const(3.0)))    # the cast is read by an op: it rounds
        pb.output(pb.cast(x, kind))                                  # a cast that only feeds an output: the store
        o = run(pb.build(), [len(xs)], [xs])[0]
        want = np.array([ref(float(v)) for v in xs])
        assert (want != xs).any()
        np.testing.assert_array_equal(o[0], want * 3.0)
        np.testing.assert_array_equal(o[1], xs)
    # ties go to the even neighbour (1 + 2^-8 lies halfway between 1 and 1 + 2^-7)
    assert _bf16_rne_py(1.0 + 2.0 ** -8) == 1.0 and _bf16_rne_py(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    # and the rounding agrees with torch's conversion
    t = torch.tensor(xs, dtype=torch.float32)
    assert torch.equal(t.to(torch.bfloat16).to(torch.float64), torch.tensor([_bf16_rne_py(float(v)) for v in xs], dtype=torch.float64))


# ---------------------------------------------------------------- data-dependent output sizes (Unique-style)
def _unique_sorted_pattern(dtype="i32"):
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param(dtype, [n])
    keep = pb.ne_prev(x)
    pb.output(pb.compact(x, keep))
    pb.output(pb.compact_rank(keep))
    pb.output(pb.compact_count(keep))
    return pb.build()


def test_unique_of_sorted_input_matches_python_sets():
    pat = _unique_sorted_pattern()
    r = np.random.default_rng(3)
    for n, hi in ((1, 3), (2, 1), (17, 4), (300, 7), (300, 100000), (1000, 2)):
        x = np.sort(r.integers(-hi, hi + 1, size=n))
        y, idx, cnt = run(pat, [n], [x])[0]
        want = sorted(set(int(v) for v in x))                 # distinct values, ascending = order of first occurrence
        assert y.tolist() == want and int(cnt) == len(want)
        assert y.shape == (len(want),)                        # the output HAS the data-dependent length
        assert [want[i] for i in idx.tolist()] == x.tolist()  # idx maps every element to its slot in y
        assert idx.tolist() == [want.index(int(v)) for v in x]
    # all equal: one value; all distinct: everything kept
    y, idx, cnt = run(pat, [5], [np.array([4, 4, 4, 4, 4])])[0]
    assert y.tolist() == [4] and idx.tolist() == [0] * 5 and int(cnt) == 1
    y, idx, cnt = run(pat, [4], [np.array([-2, 0, 1, 9])])[0]
    assert y.tolist() == [-2, 0, 1, 9] and idx.tolist() == [0, 1, 2, 3] and int(cnt) == 4


def test_ne_prev_marks_run_starts_also_in_unsorted_input():
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("f32", [n])
    pb.output(pb.cast(pb.ne_prev(x), "i32"))
    x = np.array([1.5, 1.5, -2.0, -2.0, -2.0, 1.5, 0.0, -0.0, 7.0])
    got = run(pb.build(), [len(x)], [x])[0][0].tolist()
    assert got == [1] + [int(x[i] != x[i - 1]) for i in range(1, len(x))] == [1, 0, 1, 0, 0, 1, 1, 0, 1]


def test_compaction_by_a_computed_predicate_matches_list_comprehension():
    """keep = (x * w > c): the kept values of another expression, in order; none kept and all kept."""
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("f32", [n])
    w = pb.param("f32", [n])
    thr = pb.param("f32", [])            # a rank-0 input decides how much survives
    keep = pb.op("gt", pb.op("mul", x, w), thr, dims=[n])
    pb.output(pb.compact(pb.op("add", x, pb.const(1.0), dims=[n]), keep))
    pb.output(pb.compact(pb.cast(w, "i32"), keep))
    pb.output(pb.compact_count(keep, "i64"))
    pb.output(pb.compact_rank(keep, "i64"))
    pat = pb.build()
    r = np.random.default_rng(8)
    xv = r.normal(size=200)
    wv = np.round(r.normal(size=200) * 4)
    for c in (0.0, -1e9, 1e9, 2.5):
        y, wi, cnt, rank = run(pat, [200], [xv, wv, np.asarray(c)])[0]
        kept = [i for i in range(200) if float(xv[i]) * float(wv[i]) > c]
        assert y.tolist() == [float(xv[i]) + 1.0 for i in kept]
        assert wi.tolist() == [int(wv[i]) for i in kept]
        assert int(cnt) == len(kept) == y.shape[0]
        seen, want_rank = 0, []
        for i in range(200):
            seen += i in kept
            want_rank.append(seen - 1)
        assert rank.tolist() == want_rank
    assert run(pat, [200], [xv, wv, np.asarray(1e9)])[0][0].shape == (0,)      # nothing kept: an empty result
