"""More GPU parity: every kernel version forced on the same input, bench-size shapes checked on
sampled rows, index outputs, generic patterns outside the five configurations, error paths that
need a device, determinism."""
import numpy as np
import pytest
import torch

from oracle import run as oracle_run
from workloads import PatternBuilder
from workloads.configs import CONFIGS, TORCH_DTYPE
from tests.util import alloc_outputs, assert_close, run_gpu, to_oracle_input

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


def compare(ctx, pat, dims, ins, what, force=None, handle=None):
    h = handle or ctx.register(pat)
    if force is not None:
        ctx.force_variant(V(force))
    try:
        got = run_gpu(h, pat, dims, ins)
    finally:
        ctx.force_variant(-1)
    want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
    for k, (g, w) in enumerate(zip(got, want)):
        assert_close(g, w, f"{what} dims={dims} out{k} force={force}")
    return h, got


# ---------------------------------------------------------------- every version agrees with the oracle
FORCED = {
    "C0": (["loop_vec", "loop_vec_i64", "loop_scalar", "loop_scalar_i64"], [[37, 768], [5, 13]]),
    "C1": (["row_reg_vec", "row_reg_scalar", "row_stream_vec", "row_stream_scalar"], [[2, 3, 77], [1, 2, 256]]),
    "C2": (["row_reg_vec", "row_reg_scalar", "row_stream_vec", "row_stream_scalar"], [[33, 768], [9, 1021]]),
    "C3": (["col_3stage_vec", "col_3stage_scalar", "col_strip_vec", "col_strip_scalar", "col_2stage_vec", "col_2stage_scalar"],
           [[700, 1024], [129, 37], [3, 1024], [4099, 519]]),
    "C4": (["row_reg_vec", "row_reg_scalar", "row_stream_vec", "row_stream_scalar"], [[41, 1000], [7, 2040]]),
}


@pytest.mark.parametrize("cfg_name", sorted(FORCED))
def test_every_version_matches_oracle(ctx, cfg_name):
    cfg = CONFIGS[cfg_name]
    pat = cfg.pattern()
    h = ctx.register(pat)
    versions, shapes = FORCED[cfg_name]
    for dims in shapes:
        ins = cfg.inputs(dims, seed=31)
        for v in versions:
            print(f"[forced] {cfg_name} dims={dims} version={v}", flush=True)
            compare(ctx, pat, dims, ins, cfg_name, force=v, handle=h)
    assert ctx.pattern_info(h.id)["compile_events"] == 1


# ---------------------------------------------------------------- bench-size shapes, sampled rows
def _rows_oracle(pat, dims, dev_ins, rows):
    """Oracle on a subset of rows of a row-independent pattern (operands whose leading axis is the
    row dim are sliced on the device, the rest are taken whole)."""
    sub = []
    for t, pi in zip(dev_ins, pat.params):
        op = pat.ops[pi]
        if len(op.dims) >= 1 and op.dims[0] == 0:
            sub.append(t[rows])
        else:
            sub.append(t)
    return oracle_run(pat, [len(rows)] + list(dims[1:]), [to_oracle_input(t) for t in sub])[0]


@pytest.mark.parametrize("cfg_name,dims", [
    ("C4", [667763, 5966]),       # largest call of the sweep: 3.98e9 elements, offsets beyond 2^32
    ("C4", [1048576, 64]),        # most rows, shortest rows
    ("C4", [300, 8192]),          # longest rows
    ("C2", [19273, 4096]),
    ("C0", [512, 768]),
])
def test_bench_size_shapes_on_sampled_rows(ctx, cfg_name, dims):
    cfg = CONFIGS[cfg_name]
    pat = cfg.pattern()
    h = ctx.register(pat)
    print(f"[full-size] {cfg_name} dims={dims} generating", flush=True)
    ins = cfg.inputs(dims, seed=77, device="cuda")
    outs = alloc_outputs(pat, dims, "cuda")
    for o in outs:
        o.view(-1)[:: max(1, o.numel() // 4096)].fill_(float("nan"))
    h.launch(dims, ins, outs)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    T = dims[0]
    rows = np.unique(np.concatenate([[0, 1, T - 2, T - 1], rng.integers(0, T, size=60)]).clip(0, T - 1))
    rows_t = torch.from_numpy(rows).to("cuda")
    want = _rows_oracle(pat, dims, ins, rows_t)
    for k, (o, w) in enumerate(zip(outs, want)):
        assert_close(o[rows_t].cpu(), w, f"{cfg_name} dims={dims} out{k} (sampled rows)")
    # property that holds at any size: no element left unwritten / non-finite
    for o in outs:
        assert bool(torch.isfinite(o.view(-1)[:: max(1, o.numel() // (1 << 22))].float()).all())


def test_c1_largest_call_full_compare(ctx):
    cfg = CONFIGS["C1"]
    dims = [8, 12, 505]
    compare(ctx, cfg.pattern(), dims, cfg.inputs(dims, seed=3), "C1")


def test_c3_largest_call(ctx):
    cfg = CONFIGS["C3"]
    pat = cfg.pattern()
    dims = [54784, 1024]
    ins = cfg.inputs(dims, seed=9)
    h, got = compare(ctx, pat, dims, ins, "C3")
    # determinism: no atomics anywhere, so a second run is bit-identical
    again = run_gpu(h, pat, dims, ins)
    for a, b in zip(got, again):
        assert torch.equal(a, b)
    # cancellation: columns whose sum is near zero still meet the absolute part of the fp32 bar
    x = ins[0].clone()
    x[1::2] = -x[0::2]                       # exact cancellation: every column sums to 0
    got = run_gpu(h, pat, dims, [x])
    assert float(got[0].abs().max()) <= 1e-6 and float(got[1].abs().max()) <= 1e-6


# ---------------------------------------------------------------- index outputs: bit-exact
def test_row_argmax_with_planted_ties(ctx):
    pb = PatternBuilder()
    t, h = pb.dims(2)
    x = pb.param("f32", [t, h])
    pb.output(pb.reduce("argmax", x, 1))
    pb.output(pb.reduce("max", x, 1))
    pat = pb.build()
    hd = ctx.register(pat)
    rng = np.random.default_rng(2)
    for T, H in ((64, 7), (33, 100), (9, 1000), (5, 5000), (3, 70000)):
        x = rng.normal(size=(T, H)).astype(np.float32)
        for r in range(T):
            c = rng.integers(0, H, size=3)
            x[r, c] = 9.0                     # ties: the lowest index must win
        compare(ctx, pat, [T, H], [torch.from_numpy(x)], "argmax", handle=hd)
    x = rng.normal(size=(9, 1000)).astype(np.float32)
    x[:, [17, 400, 999]] = 9.0
    for v in ("row_reg_scalar", "row_stream_vec", "row_stream_scalar"):
        compare(ctx, pat, [9, 1000], [torch.from_numpy(x)], "argmax", force=v, handle=hd)


def test_column_argmax_and_minmax(ctx):
    pb = PatternBuilder()
    t, c = pb.dims(2)
    x = pb.param("f32", [t, c])
    pb.output(pb.reduce("argmax", x, 0, dtype="i64"))
    pb.output(pb.reduce("min", x, 0))
    pb.output(pb.reduce("max", x, 0))
    pat = pb.build()
    hd = ctx.register(pat)
    assert hd.info["template"] == "col_reduce"
    rng = np.random.default_rng(4)
    for T, C in ((1, 5), (200, 33), (5000, 257), (3, 4096)):
        x = rng.normal(size=(T, C)).astype(np.float32)
        x[rng.integers(0, T, size=C), np.arange(C)] = 7.0
        x[rng.integers(0, T, size=C), np.arange(C)] = 7.0
        for v in (None, "col_3stage_vec", "col_strip_vec", "col_strip_scalar"):
            compare(ctx, pat, [T, C], [torch.from_numpy(x)], "col argmax", force=v, handle=hd)


# ---------------------------------------------------------------- generic patterns
def test_elementwise_op_zoo_fp32(ctx):
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("f32", [n])          # any sign
    p = pb.param("f32", [n])          # positive
    for oc in ("neg", "abs", "exp", "tanh", "sigmoid", "erf"):
        pb.output(pb.op(oc, x))
    for oc in ("log", "sqrt", "rsqrt", "rcp"):
        pb.output(pb.op(oc, p))
    for oc in ("add", "sub", "mul", "div", "max", "min"):
        pb.output(pb.op(oc, x, p))
    pb.output(pb.op("pow", p, x))
    pb.output(pb.op("select", pb.op("gt", x, p), x, p))
    pb.output(pb.cast(pb.op("mul", x, pb.const(8.0)), "i32"))   # exact product: same truncation on both sides
    pb.output(pb.op("le", x, pb.const(0.25)))
    pat = pb.build()
    g = torch.Generator().manual_seed(1)
    for N in (1, 1000, 100003):
        x = torch.randn(N, generator=g) * 2.0
        p = torch.rand(N, generator=g) * 3.0 + 0.05
        compare(ctx, pat, [N], [x, p], "op zoo")


def test_outer_sum_and_rank3_column_reduce(ctx):
    pb = PatternBuilder()
    n, m = pb.dims(2)
    x = pb.param("f32", [n])
    y = pb.param("f16", [m])
    pb.output(pb.op("add", pb.broadcast(x, [n, m], [0]), pb.broadcast(pb.cast(y, "f32"), [n, m], [1])))
    pat = pb.build()
    g = torch.Generator().manual_seed(2)
    for N, M in ((1, 1), (37, 129), (300, 5)):
        compare(ctx, pat, [N, M], [torch.randn(N, generator=g), torch.randn(M, generator=g).half()], "outer sum")
    # [B, T, C] reduced over T with a per-(b,c) epilogue and a per-channel scale
    pb = PatternBuilder()
    b, t, c = pb.dims(3)
    x = pb.param("f32", [b, t, c])
    w = pb.param("f32", [c])
    xs = pb.op("mul", x, pb.broadcast(w, [b, t, c], [2]))
    s = pb.reduce("sum", xs, 1)
    mean = pb.op("div", s, pb.dim_size(t))
    pb.output(mean)
    pb.output(pb.op("sub", xs, pb.broadcast(mean, [b, t, c], [0, 2])))
    pat = pb.build()
    hd = ctx.register(pat)
    assert hd.info["template"] == "col_reduce"
    for B, T, C in ((1, 1, 1), (3, 50, 17), (2, 700, 256), (70, 9, 8)):
        ins = [torch.randn(B, T, C, generator=g), torch.randn(C, generator=g)]
        for v in (None, "col_3stage_vec", "col_3stage_scalar", "col_strip_vec", "col_strip_scalar", "col_2stage_vec", "col_2stage_scalar"):
            compare(ctx, pat, [B, T, C], ins, "rank3 col", force=v, handle=hd)


def test_row_outputs_and_logsumexp(ctx):
    """Per-row outputs next to a full output; f16 storage."""
    pb = PatternBuilder()
    t, h = pb.dims(2)
    x = pb.param("f16", [t, h])
    xf = pb.cast(x, "f32")
    m = pb.reduce("max", xf, 1)
    e = pb.op("exp", pb.op("sub", xf, pb.broadcast(m, [t, h], [0])))
    s = pb.reduce("sum", e, 1)
    lse = pb.op("add", m, pb.op("log", s))
    pb.output(lse)
    pb.output(pb.cast(pb.op("sub", xf, pb.broadcast(lse, [t, h], [0])), "f16"))
    pat = pb.build()
    hd = ctx.register(pat)
    g = torch.Generator().manual_seed(3)
    for T, H in ((1, 1), (50, 33), (7, 3000), (2, 40000)):
        compare(ctx, pat, [T, H], [(torch.randn(T, H, generator=g) * 3).half()], "log-softmax", handle=hd)


def test_softmax_backward_and_layernorm_with_second_output(ctx):
    """Two adjacent variants of the benchmark patterns: the backward of a row softmax (one row
    reduction over a product of two inputs, dx = y * (dy - sum(dy * y))) and add + bias + LayerNorm
    that also emits the pre-normalisation sum as a second bf16 output."""
    pb = PatternBuilder("softmax_bwd")
    t, h = pb.dims(2)
    y = pb.cast(pb.param("bf16", [t, h]), "f32")
    dy = pb.cast(pb.param("bf16", [t, h]), "f32")
    dot = pb.reduce("sum", pb.op("mul", dy, y), 1)
    pb.output(pb.cast(pb.op("mul", y, pb.op("sub", dy, pb.broadcast(dot, [t, h], [0]))), "bf16"))
    pat = pb.build()
    hd = ctx.register(pat)
    assert hd.info["template"] == "row_reduce" and hd.info["n_phases"] == 1
    g = torch.Generator().manual_seed(4)
    for T, H in ((3, 7), (50, 1000), (9, 5739), (2, 20000)):
        probs = torch.softmax(torch.randn(T, H, generator=g), dim=1).bfloat16()
        compare(ctx, pat, [T, H], [probs, torch.randn(T, H, generator=g).bfloat16()], "softmax backward", handle=hd)

    pb = PatternBuilder("ln_two_outputs")
    t, h = pb.dims(2)
    x = pb.cast(pb.param("bf16", [t, h]), "f32")
    r = pb.cast(pb.param("bf16", [t, h]), "f32")
    b = pb.param("f32", [h]); gam = pb.param("f32", [h]); beta = pb.param("f32", [h])
    col = lambda v: pb.broadcast(v, [t, h], [1])
    row = lambda v: pb.broadcast(v, [t, h], [0])
    v = pb.op("add", pb.op("add", x, r), col(b))
    pb.output(pb.cast(v, "bf16"))
    mean = pb.op("div", pb.reduce("sum", v, 1), pb.dim_size(h))
    d = pb.op("sub", v, row(mean))
    var = pb.op("div", pb.reduce("sum", pb.op("mul", d, d), 1), pb.dim_size(h))
    n = pb.op("mul", d, row(pb.op("rsqrt", pb.op("add", var, pb.const(1e-5)))))
    pb.output(pb.cast(pb.op("add", pb.op("mul", n, col(gam)), col(beta)), "bf16"))
    pat = pb.build()
    hd = ctx.register(pat)
    assert hd.info["n_outputs"] == 2 and hd.info["n_phases"] == 2
    for T, H in ((5, 8), (40, 768), (7, 4099)):
        ins = [torch.randn(T, H, generator=g).bfloat16(), torch.randn(T, H, generator=g).bfloat16(),
               torch.randn(H, generator=g), 1 + 0.1 * torch.randn(H, generator=g), 0.1 * torch.randn(H, generator=g)]
        compare(ctx, pat, [T, H], ins, "LayerNorm with the sum as second output", handle=hd)


def test_flat_fusion_by_tensor_size_equality(ctx):
    pb = PatternBuilder()
    a, b, c, d = pb.dims(4)
    x = pb.param("f32", [a, b])
    z = pb.param("f32", [c, d])
    pb.output(pb.op("exp", x))
    pb.output(pb.op("mul", z, pb.const(3.0)))
    pb.numel_eq(x, z)
    pat = pb.build()
    g = torch.Generator().manual_seed(4)
    compare(ctx, pat, [6, 50, 20, 15], [torch.randn(6, 50, generator=g), torch.randn(20, 15, generator=g)], "flat")


# ---------------------------------------------------------------- device-side error paths and counters
def test_launch_errors_and_stats(ctx):
    from paper_2103_05288_amd import DiscError
    cfg = CONFIGS["C3"]
    pat = cfg.pattern()
    h = ctx.register(pat)
    dims = [100, 64]
    ins = [t.cuda() for t in cfg.inputs(dims, seed=1)]
    outs = alloc_outputs(pat, dims, "cuda")
    big = [20000, 300]                   # partials of the chunks go through the workspace
    ins_b = [t.cuda() for t in cfg.inputs(big, seed=2)]
    with pytest.raises(DiscError) as e:
        h.launch(big, ins_b, alloc_outputs(pat, big, "cuda"), workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == "WORKSPACE"
    with pytest.raises(DiscError) as e:
        h.launch(dims, ins[:0], outs)
    assert e.value.status == "INVALID_ARG"
    before = ctx.stats()
    ws = torch.empty(ctx.workspace_bytes(h.id, dims), dtype=torch.uint8, device="cuda")
    h.launch(dims, ins, outs, workspace=ws)
    torch.cuda.synchronize()
    after = ctx.stats()
    assert after["launch_calls"] == before["launch_calls"] + 1
    assert after["device_launches"] == before["device_launches"] + 1      # small: the single-launch version
    assert after["compile_events"] == before["compile_events"]
    h.launch(big, ins_b, alloc_outputs(pat, big, "cuda"),
             workspace=torch.empty(ctx.workspace_bytes(h.id, big), dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert ctx.stats()["device_launches"] == after["device_launches"] + 2   # partial, finish + epilogue
    ctx.force_variant(V("col_3stage_vec"))
    try:
        h.launch(big, ins_b, alloc_outputs(pat, big, "cuda"),
                 workspace=torch.empty(ctx.workspace_bytes(h.id, big), dtype=torch.uint8, device="cuda"))
    finally:
        ctx.force_variant(-1)
    torch.cuda.synchronize()
    assert ctx.stats()["device_launches"] == after["device_launches"] + 5   # partial, finish, epilogue
    # zero rows: success, nothing launched
    c0 = CONFIGS["C0"]
    p0 = c0.pattern()
    h0 = ctx.register(p0)
    n = ctx.stats()["device_launches"]
    h0.launch([0, 768], [torch.empty(0, 768, device="cuda"), torch.empty(768, device="cuda"), torch.empty(0, 768, device="cuda")],
              [torch.empty(0, 768, device="cuda")])
    assert ctx.stats()["device_launches"] == n


def test_util_kernels(ctx):
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    ctx.util_copy(dst, src, src.numel() * 4)
    ctx.util_empty_launch()
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


# ---------------------------------------------------------------- single-shape modules (gap-to-static comparison)
@pytest.mark.parametrize("cfg_name,dims", [
    ("C0", [37, 768]), ("C1", [2, 3, 77]), ("C2", [33, 1021]), ("C2", [700, 4096]), ("C3", [700, 1024]), ("C3", [5000, 300]),
    ("C4", [41, 1000]), ("C4", [300, 5739]), ("C4", [5, 12289]), ("C4", [3, 30000]),
])
def test_single_shape_module_matches_oracle_and_generic(ctx, cfg_name, dims):
    cfg = CONFIGS[cfg_name]
    pat = cfg.pattern()
    ins = cfg.inputs(dims, seed=9)
    hs = ctx.register_static(pat, dims)
    got = run_gpu(hs, pat, dims, ins)
    want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
    for k, (g, w) in enumerate(zip(got, want)):
        assert_close(g, w, f"static {cfg_name} dims={dims} out{k}")
    # (not compared bit for bit with the shape-generic module: the two may run with different grids,
    # and rows of several wavefronts are summed in an order that depends on the block's row count)
    from paper_2103_05288_amd import DiscError
    with pytest.raises(DiscError) as e:
        other = list(dims)
        other[0] += 1
        run_gpu(hs, pat, other, cfg.inputs(other, seed=9))
    assert e.value.status == "SHAPE"


def test_byte_offsets_beyond_32_bits(ctx):
    """A 1-D tensor whose byte size exceeds 4 GiB while its slot count still fits the 32-bit slot
    index, and a row-reduce whose single row is that long (streaming version): element offsets
    inside a row must be scaled to bytes in 64 bits."""
    n = (1 << 30) + 12345                      # 4 GiB + of fp32
    pb = PatternBuilder()
    d = pb.dim()
    x = pb.param("f32", [d])
    pb.output(pb.op("add", pb.op("mul", x, pb.const(2.0)), pb.const(1.0)))
    pat = pb.build()
    h = ctx.register(pat)
    assert h.plan([n])["index_bits"] == 32
    xs = torch.empty(n, dtype=torch.float32, device="cuda")
    step = 1 << 20
    for s in range(0, n, 1 << 26):             # value = index mod 2^20, exact in fp32
        e = min(n, s + (1 << 26))
        xs[s:e] = (torch.arange(s, e, device="cuda", dtype=torch.int64) % step).to(torch.float32)
    out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    h.launch([n], [xs], [out])
    torch.cuda.synchronize()
    g = torch.Generator().manual_seed(3)
    idx = torch.cat([torch.arange(0, 4096), torch.arange(n - 4096, n), torch.randint(0, n, (200000,), generator=g),
                     torch.arange((1 << 30) - 2048, (1 << 30) + 2048)]).cuda()
    want = (idx % step).to(torch.float32) * 2.0 + 1.0
    assert torch.equal(out[idx], want)
    assert not torch.isnan(out[:: 4099]).any()
    del out
    # one row of the same length: row max (streaming version, three passes would be needed for an
    # epilogue; a reduce-only pattern keeps the test at two tensors)
    pb = PatternBuilder()
    t, hh = pb.dims(2)
    x2 = pb.param("f32", [t, hh])
    pb.output(pb.reduce("max", x2, 1))
    pb.output(pb.reduce("min", x2, 1))
    pat2 = pb.build()
    h2 = ctx.register(pat2)
    assert h2.plan([1, n])["variant_name"] == "row_stream_vec"
    xs[n - 7] = 5.0e6                          # a maximum near the far end of the row
    xs[(1 << 30) + 5] = -3.0                   # a minimum just past the 4 GiB byte offset
    outs = [torch.empty(1, dtype=torch.float32, device="cuda") for _ in range(2)]
    h2.launch([1, n], [xs.view(1, n)], outs)
    torch.cuda.synchronize()
    assert outs[0].item() == 5.0e6 and outs[1].item() == -3.0


def test_launches_can_be_captured_in_a_graph(ctx):
    """disc_launch enqueues kernels and nothing else (no allocation, no synchronisation, no memset),
    so a caller may record it into a HIP graph: row-reduce, three-launch column-reduce and loop
    patterns captured once, replayed with new input contents, every replay checked against the
    oracle (with the program's own eager work and synchronisations between the replays)."""
    jobs = []
    for name, dims in (("C2", [300, 1024]), ("C3", [3000, 1024]), ("C0", [77, 768]), ("C4", [50, 5739])):
        cfg = CONFIGS[name]
        pat = cfg.pattern()
        h = ctx.register(pat)
        ins = [t.cuda() for t in cfg.inputs(dims, seed=31)]
        outs = alloc_outputs(pat, dims, "cuda")
        ws = torch.empty(max(16, ctx.workspace_bytes(h.id, dims)), dtype=torch.uint8, device="cuda")
        h.launch(dims, ins, outs, workspace=ws)          # warm: occupancy queries, module functions
        jobs.append((name, cfg, pat, h, dims, ins, outs, ws))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for name, cfg, pat, h, dims, ins, outs, ws in jobs:
                h.launch(dims, ins, outs, workspace=ws, stream=side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        fresh = {}
        for name, cfg, pat, h, dims, ins, outs, ws in jobs:
            new = cfg.inputs(dims, seed=100 + replay)
            for dst, src in zip(ins, new):
                dst.copy_(src.cuda())                     # eager work between the replays
            for o in outs:
                o.fill_(float("nan")) if o.dtype.is_floating_point else o.zero_()
            fresh[name] = new
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, cfg, pat, h, dims, ins, outs, ws in jobs:
            want = oracle_run(pat, dims, [to_oracle_input(t) for t in fresh[name]])[0]
            for k, (g, w) in enumerate(zip(outs, want)):
                assert_close(g.cpu(), w, f"graph replay {replay} {name} out{k}")
