"""Host-side logic through the C ABI, no GPU needed: exports, checker, fusion decision, planner,
error paths.  A host-only context (device -1) still runs the whole registration path including
the one device compile for gfx950 (hipRTC cross-compiles without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2103_05288_amd import Context, DiscError, VARIANTS, lib_path, load_library
from workloads import PatternBuilder
from workloads.configs import CONFIGS, algorithmic_bytes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
V = {n: i for i, n in enumerate(VARIANTS)}


@pytest.fixture(scope="module")
def ctx():
    c = Context(-1)
    yield c
    c.close()


@pytest.fixture(scope="module")
def handles(ctx):
    return {n: ctx.register(cfg.pattern()) for n, cfg in CONFIGS.items()}


def expect(code, fn, *a, **k):
    with pytest.raises(DiscError) as e:
        fn(*a, **k)
    assert e.value.status == code, (e.value.status, e.value.message)
    return e.value.message


# ------------------------------------------------------------------ boundary
def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "disc.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(disc_[a-z_]+)\s*\(", body))
    assert {"disc_create", "disc_register_pattern", "disc_launch", "disc_plan"} <= declared
    lib = ctypes.CDLL(lib_path())
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in disc.h but not exported"
    assert load_library() is not None


def test_one_compile_per_pattern_and_pattern_cache(ctx, handles):
    kinds = {n: h.info["template"] for n, h in handles.items()}
    assert kinds == {"C0": "loop", "C1": "row_reduce", "C2": "row_reduce", "C3": "col_reduce", "C4": "row_reduce"}
    before = ctx.stats()
    for n, cfg in CONFIGS.items():
        again = ctx.register(cfg.pattern())          # same op sequence: answered from the cache
        assert again.id == handles[n].id
        assert again.info["compile_events"] == 1
    after = ctx.stats()
    assert after["compile_events"] == before["compile_events"]
    assert after["pattern_cache_hits"] == before["pattern_cache_hits"] + len(CONFIGS)
    # planning at many shapes never compiles
    for t in (1, 7, 1000, 99999):
        handles["C4"].plan([t, 333])
    assert ctx.stats()["compile_events"] == after["compile_events"]


def test_generated_source_is_exposed(handles):
    src = handles["C4"].source
    assert "struct Pat" in src and "k_row_vec_nv2w" in src and "row_reg_body" in src


# ------------------------------------------------------------------ constraint closure
def test_dim_classes_from_op_semantics(ctx, handles):
    assert handles["C1"].info["n_dim_classes"] == 3
    # Add: operands and result have the same shape -> symbolic dims get merged
    pb = PatternBuilder()
    d = pb.dims(6)
    x = pb.param("f32", [d[0], d[1]])
    r = pb.param("f32", [d[2], d[3]])
    pb.output(pb.op("add", x, r, dims=[d[4], d[5]]))
    h = ctx.register(pb.build())
    cls = h.info["dim_class"]
    assert cls[0] == cls[2] == cls[4] and cls[1] == cls[3] == cls[5] and cls[0] != cls[1]
    assert h.plan([5, 7, 5, 7, 5, 7])["n_launches"] == 1
    msg = expect("CONSTRAINT", h.plan, [5, 7, 6, 7, 5, 7])
    assert "registered as equal" in msg


def test_static_sizes(ctx):
    pb = PatternBuilder()
    t = pb.dim()
    x = pb.param("f32", [t, pb.static(3)])
    y = pb.param("f32", [t, pb.static(4)])
    pb.output(pb.op("add", x, y))
    assert "static sizes" in expect("BAD_PATTERN", ctx.register, pb.build())
    pb = PatternBuilder()
    t, h = pb.dims(2)
    x = pb.param("f32", [t, h])
    y = pb.param("f32", [t, pb.static(16)])
    pb.output(pb.op("add", x, y))
    hd = ctx.register(pb.build())
    assert hd.plan([9, 16])["n_launches"] == 1
    assert "static size" in expect("CONSTRAINT", hd.plan, [9, 17])


def _two_chains(constraint=None):
    """Two element-wise chains on tensors whose shapes are unrelated in the op list (what is left
    of a framework Split after lowering): fusible only with an injected constraint."""
    pb = PatternBuilder()
    a, b, c, d = pb.dims(4)
    x = pb.param("f32", [a, b])
    z = pb.param("f32", [c, d])
    o1 = pb.output(pb.op("exp", x))
    o2 = pb.output(pb.op("neg", z))
    if constraint == "dim":
        pb.dim_eq(x, 0, z, 0)
        pb.dim_eq(x, 1, z, 1)
    elif constraint == "numel":
        pb.numel_eq(x, z)
    return pb.build(), (o1, o2)


def test_caller_constraints_enable_fusion(ctx):
    msg = expect("UNFUSIBLE", ctx.register, _two_chains()[0])
    assert "DIM_EQ" in msg and "NUMEL_EQ" in msg
    h = ctx.register(_two_chains("dim")[0])
    assert h.info["template"] == "loop" and h.info["n_outputs"] == 2 and h.info["n_dim_classes"] == 2
    assert h.info["n_collapsed"] == 1                      # [a,b] collapses to one flat group
    expect("CONSTRAINT", h.plan, [4, 5, 4, 6])
    hn = ctx.register(_two_chains("numel")[0])             # tensor-size equality: fused over a flat index
    assert hn.info["template"] == "loop" and hn.info["n_collapsed"] == 1
    assert hn.plan([4, 6, 3, 8])["inner"] == 24
    # the registered tensor-size equality is part of the launch-time shape calculation: dims that
    # contradict it are refused before anything could run over the smaller tensor
    msg = expect("CONSTRAINT", hn.plan, [4, 6, 5, 1])
    assert "registered as equal in size" in msg
    expect("CONSTRAINT", hn.ctx.workspace_bytes, hn.id, [4, 6, 23, 1])
    # (the advisor's case: a rank-1 tensor tied to a rank-2 one)
    pb = PatternBuilder()
    a, b, c = pb.dims(3)
    x = pb.param("f32", [a, b])
    z = pb.param("f32", [c])
    pb.output(pb.op("exp", x))
    pb.output(pb.op("neg", z))
    pb.numel_eq(x, z)
    h1 = ctx.register(pb.build())
    assert h1.plan([4, 6, 24])["inner"] == 24
    expect("CONSTRAINT", h1.plan, [4, 6, 5])


# ------------------------------------------------------------------ fusion decision
def test_unfusible_patterns(ctx):
    # reductions over different axes
    pb = PatternBuilder()
    t, h = pb.dims(2)
    x = pb.param("f32", [t, h])
    pb.output(pb.reduce("max", x, 0))
    pb.output(pb.reduce("sum", x, 1))
    assert "floating-point sum" in expect("UNFUSIBLE", ctx.register, pb.build())
    # (a SUM over the rows next to row reductions is fused: tests/test_row_col_sums.py)
    pb = PatternBuilder()
    b, t, h = pb.dims(3)
    x = pb.param("f32", [b, t, h])
    pb.output(pb.reduce("sum", x, 0))
    pb.output(pb.reduce("sum", x, 1))
    assert "different axes" in expect("UNFUSIBLE", ctx.register, pb.build())
    # a row result consumed along the other axis of a square iteration space
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("f32", [n, n])
    m = pb.reduce("max", x, 1)
    pb.output(pb.op("sub", x, pb.broadcast(m, [n, n], [1])))
    assert "other axes" in expect("UNFUSIBLE", ctx.register, pb.build())
    # a column reduction feeding a second reduction needs another pass over the tensor
    pb = PatternBuilder()
    t, h = pb.dims(2)
    x = pb.param("f32", [t, h])
    mean = pb.op("div", pb.reduce("sum", x, 0), pb.dim_size(t))
    d = pb.op("sub", x, pb.broadcast(mean, [t, h], [1]))
    pb.output(pb.reduce("sum", pb.op("mul", d, d), 0))
    assert "second pass" in expect("UNFUSIBLE", ctx.register, pb.build())


def test_broadcast_contexts_and_collapse(ctx, handles):
    # C1: [B, NH, S, S] with a [B,1,1,S] mask collapses to [B] x [NH*S] x [S]
    assert handles["C1"].info["n_collapsed"] == 3
    p = handles["C1"].plan([8, 12, 100])
    assert p["rows"] == 8 * 12 * 100 and p["inner"] == 100
    # outer sum x[i] + y[j]: one operand per axis, nothing collapses
    pb = PatternBuilder()
    n, m = pb.dims(2)
    x = pb.param("f32", [n])
    y = pb.param("f32", [m])
    pb.output(pb.op("add", pb.broadcast(x, [n, m], [0]), pb.broadcast(y, [n, m], [1])))
    h = ctx.register(pb.build())
    assert h.info["n_collapsed"] == 2
    # a pure element-wise rank-4 pattern collapses to one flat dim
    pb = PatternBuilder()
    d = pb.dims(4)
    x = pb.param("bf16", d)
    pb.output(pb.cast(pb.op("tanh", pb.cast(x, "f32")), "bf16"))
    h = ctx.register(pb.build())
    assert h.info["n_collapsed"] == 1 and h.plan([2, 3, 4, 5])["inner"] == 120


@pytest.mark.parametrize("case", ["forward_ref", "rank5", "bool_arith", "no_output", "bad_axis", "bcast_order",
                                  "argmax_dtype", "output_dtype"])
def test_bad_patterns(ctx, case):
    from workloads.pattern import Op, Pattern
    p = Pattern(n_dims=2)
    if case == "forward_ref":
        p.ops = [Op("param", "f32", (), (0,)), Op("neg", "f32", (2,), (0,)), Op("output", "f32", (1,), (0,))]
    elif case == "rank5":
        lib = load_library()
        from paper_2103_05288_amd.binding import disc_op, disc_constraint
        ops = (disc_op * 1)()
        ops[0].opcode, ops[0].dtype, ops[0].rank = 0, 0, 5
        pid = ctypes.c_int32()
        rc = lib.disc_register_pattern(ctx.h, ops, 1, (disc_constraint * 1)(), 0, ctypes.byref(pid))
        assert rc == -2 and b"static rank" in lib.disc_last_error(ctx.h)
        return
    elif case == "bool_arith":
        p.ops = [Op("param", "bool", (), (0,)), Op("add", "f32", (0, 0), (0,)), Op("output", "f32", (1,), (0,))]
    elif case == "no_output":
        p.ops = [Op("param", "f32", (), (0,))]
    elif case == "bad_axis":
        p.ops = [Op("param", "f32", (), (0, 1)), Op("reduce_sum", "f32", (0,), (0,), (2,)), Op("output", "f32", (1,), (0,))]
    elif case == "bcast_order":
        p.ops = [Op("param", "f32", (), (0, 1)), Op("broadcast", "f32", (0,), (0, 1), (1, 0)), Op("output", "f32", (1,), (0, 1))]
    elif case == "argmax_dtype":
        p.ops = [Op("param", "f32", (), (0, 1)), Op("reduce_argmax", "f32", (0,), (0,), (1,)), Op("output", "f32", (1,), (0,))]
    elif case == "output_dtype":
        p.ops = [Op("param", "f32", (), (0,)), Op("output", "bf16", (0,), (0,))]
    expect("BAD_PATTERN", ctx.register, p)


# ------------------------------------------------------------------ runtime flow (planner)
def test_row_schedule_selection(handles):
    h = handles["C4"]
    short = h.plan([1000, 64])
    assert short["variant_name"] == "row_reg_vec" and short["lanes_per_row"] < 64      # several rows per wavefront
    mid = h.plan([1000, 1024])
    assert mid["variant_name"] == "row_reg_vec" and mid["n_launches"] == 1
    long_ = h.plan([100, 8192])
    assert long_["variant_name"] == "row_reg_vec" and long_["lanes_per_row"] == 512     # wavefronts cooperate via LDS
    assert long_["block"][0][0] == 512 and long_["slots_per_lane"] == 2
    assert long_["lanes_per_row"] * long_["slots_per_lane"] * long_["vec_width"] >= 8192
    huge = h.plan([10, 100000])
    assert huge["variant_name"] == "row_stream_vec"                                    # does not fit registers
    for p in (short, mid, huge):
        assert p["grid"][0][0] >= 1 and p["block"][0][0] == 256
    assert h.plan([7, 3])["vec_width"] in (1, 8)
    forced = h.plan([1000, 1024], V["row_reg_scalar"])
    assert forced["vec_width"] == 1 and forced["variant_name"] == "row_reg_scalar"
    expect("INVALID_ARG", h.plan, [1000, 1024], V["loop_vec"])
    expect("INVALID_ARG", h.plan, [10, 100000], V["row_reg_vec"])


def test_row_schedule_capacity_steps(handles):
    """Lanes per row x slots per lane: the least capacity among {2, 3} x power of two that holds the
    row; blocks above 256 threads only for the two longest classes; staged kernel versions (_s) as
    long as the row vectors fit the LDS budget.  A ragged end is taken as single elements (and the
    row then only needs capacity for its whole slots) when the row has at least 8 lanes and the
    block 256 threads."""
    h = handles["C4"]                     # bf16, 8 elements per slot
    cases = {                             # H -> (lanes per row, slots per lane, block)
        64: (4, 2, 256), 65: (4, 3, 256), 97: (8, 2, 256), 105: (8, 2, 256), 512: (32, 2, 256), 513: (32, 2, 256),
        1024: (64, 2, 256), 1100: (64, 3, 256), 1537: (64, 3, 256), 1543: (64, 3, 256), 1545: (128, 2, 256),
        3000: (128, 3, 256), 4096: (256, 2, 256), 5739: (256, 3, 256), 6145: (256, 3, 256), 6151: (256, 3, 256),
        6153: (512, 2, 512), 8192: (512, 2, 512),
        8200: (512, 3, 512), 12289: (1024, 2, 1024), 16385: (1024, 2, 1024), 16393: (1024, 3, 1024), 24576: (1024, 3, 1024),
    }
    for H, (G, nv, block) in cases.items():
        p = h.plan([50, H])
        assert (p["lanes_per_row"], p["slots_per_lane"], p["block"][0][0]) == (G, nv, block), (H, p)
        tail = H % 8 != 0 and G >= 8 and (block == 256 or nv <= 2) and G * nv * 8 >= H - H % 8 and p["kernels"][0].endswith("_t")
        assert G * nv * 8 >= (H - H % 8 if tail else H)
        want = "k_row_vec_nv%d%s" % (max(nv, 2 if block > 256 else 1), "w" if block > 256 else "")
        name = p["kernels"][0]
        assert not name.endswith("_nt")                       # a small launch: its result may be wanted from cache
        # rows in blocks of 256 threads take a version without ragged-tail paths: _e when they are
        # whole slots, _t (whole slots + single elements) when they have at least 8 lanes
        # (blocks above 256 threads: a _t version of the two-slot kernel only)
        even = ("_t" if H % 8 != 0 and nv <= 2 else "") if block != 256 else "_e" if H % 8 == 0 else "_t" if G >= 8 else ""
        assert name.endswith(want + "_s" + even) or name.endswith(want + even), (H, p["kernels"])
        # the non-temporal version: launches of 64 MiB or more whose rows start and end on 16-byte
        # boundaries, 128 elements or more, blocks of 256 threads
        big = h.plan([(80 << 20) // (5 * H) + 1, H])["kernels"][0]
        assert big.endswith("_nt") == (H % 8 == 0 and H >= 128 and block == 256), (H, big)
        assert (big[:-3] + "_e" if big.endswith("_nt") else big) == name
    assert h.plan([50, 24577])["variant_name"] == "row_stream_vec"
    # below 512 elements the non-temporal version needs rows of whole 128-byte lines in every operand
    assert [h.plan([200000, H])["kernels"][0].endswith("_nt") for H in (128, 200, 360, 384, 504, 512, 520)] == \
        [True, False, False, True, False, True, True]
    # C4 stages a float32 row vector: 4 bytes x H must fit 48 KiB
    assert h.plan([50, 8192])["kernels"][0].endswith("_s") and h.plan([50, 8192])["lds_bytes"][0] >= 4 * 8192
    assert not h.plan([50, 16385])["kernels"][0].endswith("_s") and h.plan([50, 16385])["lds_bytes"][0] == 0
    # scalar versions: at most two slots per lane, never staged
    p = h.plan([50, 100], V["row_reg_scalar"])
    assert p["slots_per_lane"] <= 2 and not p["kernels"][0].endswith("_s")


def test_aligned_slots_of_ragged_rows_plan(handles):
    """Ragged rows in the versions that take the row's ends as single elements (_t): when the rows
    start off dword boundaries (odd lengths of 2-byte elements), with aligned bases and at least 14
    lanes per row, the vector slots are put on the tensor's 16-byte boundaries,
    which needs a grid that gives a lane group rows of one alignment only -- (grid x rows per block x
    row length) a multiple of the vector width.  Otherwise the grid stays odd, so that every block
    meets all alignments."""
    h4 = handles["C4"]
    for H in (513, 1023, 1026, 1100, 2047, 4095, 5739, 6145):
        T = (200 << 20) // H
        p = h4.plan([T, H])
        assert p["kernels"][0].endswith("_t"), (H, p["kernels"])
        rpb = p["block"][0][0] // p["lanes_per_row"]
        if H % 2 == 1:        # rows of bf16 elements that start off dword boundaries: shifted
            assert (p["grid"][0][0] * rpb * H) % 8 == 0, (H, p["grid"])
        else:                 # dword-aligned rows run at full rate as they are
            assert p["grid"][0][0] % 2 == 1, (H, p["grid"])
        q = h4.plan([T, H], inputs=[4098, 4096, 4096, 4096], outputs=[4096])      # one base off a slot boundary
        assert q["kernels"][0].endswith("_t") and q["grid"][0][0] % 2 == 1, (H, q["grid"])
    # too few rows for such a grid: the plain _t launch
    p = h4.plan([5, 5739])
    assert p["kernels"][0].endswith("_t") and p["grid"][0][0] == 5


def test_single_shape_registration(ctx, handles):
    """The same op list compiled for one shape: a pattern of its own per shape, only that shape's kernel
    versions in the module, its extents and launch plan as constants; other dims are refused."""
    pat = CONFIGS["C4"].pattern()
    before = ctx.stats()
    a = ctx.register_static(pat, [30000, 2048])
    b = ctx.register_static(pat, [300, 2049])
    again = ctx.register_static(pat, [30000, 2048])
    after = ctx.stats()
    assert a.id != b.id and again.id == a.id and a.id != handles["C4"].id
    assert after["compile_events"] == before["compile_events"] + 2 and after["pattern_cache_hits"] == before["pattern_cache_hits"] + 1
    # 2048-wide rows plan the non-temporal version; its plain sibling stays for misaligned operands
    assert a.info["compile_events"] == 1 and a.info["n_variants"] == 2 and a.info["compile_ms"] > 0
    assert b.info["n_variants"] == 1
    generic = handles["C4"].plan([30000, 2048])
    pa = a.plan([30000, 2048])
    for k in ("variant_name", "lanes_per_row", "slots_per_lane", "vec_width", "block", "lds_bytes", "algorithmic_bytes"):
        assert pa[k] == generic[k], k
    assert pa["kernels"][0].split("_k_")[1] == generic["kernels"][0].split("_k_")[1]
    src = a.source
    assert "A.inner = 2048LL;" in src and "A.rows = 30000LL;" in src and "rp.G = 128;" in src
    assert src.count('extern "C" __global__') == 2 and b.source.count('extern "C" __global__') == 1
    assert "A.inner = 2049LL;" in b.source
    expect("SHAPE", a.plan, [30000, 2049])
    expect("SHAPE", a.plan, [30001, 2048])
    expect("INVALID_ARG", a.plan, [30000, 2048], V["row_reg_scalar"])
    # a column reduce keeps its three entry points; a small one its single strip kernel
    c3 = CONFIGS["C3"].pattern()
    big = ctx.register_static(c3, [5000, 1024])
    small = ctx.register_static(c3, [100, 1024])
    assert big.info["n_variants"] == 2 and small.info["n_variants"] == 1      # partial + finish-and-epilogue; one strip kernel
    assert "rp.nchunk = " in big.source and "A.mid = 5000LL;" in big.source
    # nothing to launch, nothing to specialise
    expect("SHAPE", ctx.register_static, pat, [0, 64])
    expect("INVALID_ARG", ctx.register_static, pat, [])
    expect("INVALID_ARG", ctx.register_static, pat, [1, 2, 3])


def test_loop_and_index_width_selection(ctx, handles):
    h = handles["C0"]
    p = h.plan([300, 768])
    assert p["variant_name"] == "loop_vec" and p["index_bits"] == 32 and p["vec_width"] == 4
    assert p["algorithmic_bytes"] == algorithmic_bytes(CONFIGS["C0"].pattern(), [300, 768])
    assert h.plan([300, 5])["variant_name"] == "loop_scalar"      # padding a 5-wide row to 8 wastes too much
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("bf16", [n])
    pb.output(pb.cast(pb.op("neg", pb.cast(x, "f32")), "bf16"))
    big = ctx.register(pb.build())
    assert big.plan([1 << 20])["index_bits"] == 32
    assert big.plan([1 << 35])["index_bits"] == 64
    expect("INVALID_ARG", big.plan, [1 << 35], V["loop_vec"])


def test_col_reduce_plan_and_workspace(ctx, handles):
    h = handles["C3"]
    # the usual case: two launches, the second finishes and applies the epilogue
    p = h.plan([65536, 1024])
    assert p["variant_name"] == "col_2stage_vec" and p["n_launches"] == 2 and p["mid"] == 65536
    assert p["kernels"][0].endswith("k_col_partial_vec") and p["kernels"][1].endswith("k_col_epi2_vec_nt")
    assert p["workspace_bytes"] > 0 and ctx.workspace_bytes(h.id, [65536, 1024]) == p["workspace_bytes"]
    assert 1 < p["grid"][0][1] <= 32                              # the reduced axis is cut into a few chunks
    assert p["grid"][0][0] * p["grid"][0][1] >= 512               # ... on narrow column tiles: the chip is filled
    assert p["grid"][1][0] == p["grid"][0][0] and p["grid"][1][1] > p["grid"][0][1]
    assert h.plan([3000, 1024])["kernels"][1].endswith("k_col_epi2_vec")      # small launches keep plain stores
    # a long and narrow reduced axis needs more chunks than the second launch can merge per block:
    # the separate finish launch stays
    q = h.plan([2000000, 8])
    assert q["variant_name"] == "col_3stage_vec" and q["n_launches"] == 3 and q["grid"][0][1] > 32
    assert q["kernels"][1].endswith("k_col_finish")
    f3 = h.plan([65536, 1024], V["col_3stage_vec"])
    assert f3["n_launches"] == 3 and f3["workspace_bytes"] > p["workspace_bytes"]
    assert h.plan([1, 1024], V["col_3stage_vec"])["grid"][0][1] == 1
    assert h.plan([1, 1024], V["col_2stage_vec"])["grid"][0][1] == 1
    assert ctx.workspace_bytes(handles["C4"].id, [10, 10]) == 0
    # up to about a million elements: one launch, a block per strip of columns, no workspace
    s = h.plan([512, 1024])
    assert s["variant_name"] == "col_strip_vec" and s["n_launches"] == 1 and s["kernels"][0].endswith("k_col_strip_vec")
    assert s["grid"][0][0] * s["lanes_per_row"] * s["vec_width"] >= 1024 and s["grid"][0][0] >= 32
    assert s["workspace_bytes"] == 0                       # reduce results stay in registers
    assert h.plan([1025, 1024])["variant_name"] == "col_2stage_vec"
    assert h.plan([7, 5])["variant_name"] == "col_strip_scalar"
    forced = h.plan([300, 1024], V["col_3stage_scalar"])
    assert forced["variant_name"] == "col_3stage_scalar" and forced["n_launches"] == 3
    assert h.plan([70000, 1024], V["col_strip_vec"])["n_launches"] == 1
    expect("INVALID_ARG", h.plan, [300, 1024], V["row_reg_vec"])


def test_degenerate_shapes_and_errors(ctx, handles):
    assert handles["C0"].plan([0, 768])["n_launches"] == 0
    assert handles["C4"].plan([0, 64])["n_launches"] == 0
    expect("EMPTY_REDUCE", handles["C4"].plan, [5, 0])
    expect("EMPTY_REDUCE", handles["C3"].plan, [0, 1024])
    assert handles["C3"].plan([5, 0])["n_launches"] == 0
    expect("SHAPE", handles["C0"].plan, [-1, 768])
    expect("SHAPE", handles["C0"].plan, [1 << 40, 1 << 40])
    expect("INVALID_ARG", handles["C0"].plan, [1, 2, 3])
    expect("INVALID_ARG", ctx.plan, 12345, [1, 2])
    expect("INVALID_ARG", ctx.force_variant, 99)
    # a host-only context cannot launch
    expect("INVALID_ARG", handles["C0"].launch, [1, 768], [1, 2, 3], [4], stream=0)


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: any other --gpus value ends with a message, before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


# ------------------------------------------------------------------ code generation corner cases
def test_negative_constants_and_integer_ops_compile(ctx):
    """NEG / ABS of negative literals (float and integer) and integer arithmetic of both widths go
    through the one device compile (a '-' pasted in front of a negative literal would not)."""
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("f32", [n])
    xi = pb.param("i32", [n])
    xl = pb.param("i64", [n])
    pb.output(pb.op("add", x, pb.op("neg", pb.const(-1.5)), dims=[n]))
    pb.output(pb.op("mul", x, pb.op("abs", pb.const(-2.0)), dims=[n]))
    pb.output(pb.op("add", xi, pb.op("abs", pb.const(-3.0, "i32")), dims=[n]))
    pb.output(pb.op("sub", xl, pb.op("neg", pb.const(-7.0, "i64")), dims=[n]))
    pb.output(pb.op("div", pb.op("mul", xi, xi), pb.op("max", pb.op("abs", xi), pb.const(1.0, "i32"), dims=[n])))
    pb.output(pb.cast(pb.op("mul", pb.cast(pb.cast(x, "bf16"), "f32"), x), "f16"))
    h = ctx.register(pb.build())
    assert h.info["compile_events"] == 1 and h.info["template"] == "loop"
    src = h.source
    assert "disc::from_f32<__bf16>" in src          # the mid-chain cast rounds
    assert "(disc::u32)" in src and "(disc::u64)" in src   # integer arithmetic wraps


# ------------------------------------------------------------------ the launch path allocates nothing
def test_launch_path_makes_no_heap_allocation(tmp_path):
    """1000 distinct shapes per benchmark pattern through disc_plan / disc_workspace_bytes (the launch
    path without the enqueue) under a counting allocator: no allocation, so no strings, maps or
    vectors are built per call -- the host flow is tables filled at registration (Section 4.2.3).
    The counting program is C++ (tests/cpp/plan_alloc_count.cpp) because the allocator of the whole
    process has to be interposed."""
    import struct
    import subprocess
    import numpy as np
    from paper_2103_05288_amd.binding import marshal_pattern
    from workloads import extras
    exe = tmp_path / "plan_alloc_count"
    subprocess.run(["g++", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-o", str(exe),
                    os.path.join(ROOT, "tests", "cpp", "plan_alloc_count.cpp"), lib_path(),
                    "-Wl,-rpath," + os.path.dirname(lib_path()), "-Wl,-rpath,/opt/rocm/lib"], check=True)
    rng = np.random.default_rng(5)
    files = []
    pats = {n: cfg.pattern() for n, cfg in CONFIGS.items()}
    pats["LNB"] = extras.layernorm_backward_graph()
    pats["LSE"] = extras.logsumexp_with_total_and_amax()
    for name, pat in pats.items():
        ops, n_ops, cs, n_cs = marshal_pattern(pat)
        nd = pat.n_dims
        shapes = set()
        while len(shapes) < 1000:
            if name == "C1":
                shapes.add((int(rng.integers(1, 9)), int(rng.integers(1, 13)), int(rng.integers(1, 2000))))
            else:
                shapes.add(tuple(int(2 ** rng.uniform(0, 17)) for _ in range(nd)))
        path = tmp_path / f"{name}.pat"
        with open(path, "wb") as f:
            f.write(struct.pack("<iii", n_ops, n_cs, nd))
            f.write(bytes(ops))
            if n_cs:
                f.write(bytes(cs)[: n_cs * 20])
            f.write(struct.pack("<i", len(shapes)))
            for s in sorted(shapes):
                f.write(struct.pack("<%dq" % nd, *s))
        files.append(str(path))
    r = subprocess.run([str(exe)] + files, capture_output=True, text=True)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.count("allocations=0") == len(files)
    # the same driver with the library's host sources under ASan + UBSan: registration (checker,
    # code generation, the device compile) and 1000 plans per pattern, error paths included
    from paper_2103_05288_amd.build import build_sanitized_driver
    san = build_sanitized_driver(str(tmp_path / "plan_sanitized"), os.path.join(ROOT, "tests", "cpp", "plan_alloc_count.cpp"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([san] + files, capture_output=True, text=True, env=env)
    print(r.stdout[-2000:], r.stderr[-4000:])
    assert r.returncode == 0, r.stdout + r.stderr
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


# ------------------------------------------------------------------ outputs whose size depends on the data
def test_compaction_patterns_checker_and_plan(ctx):
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("i32", [n])
    keep = pb.ne_prev(x)
    pb.output(pb.compact(x, keep))
    pb.output(pb.compact_rank(keep))
    pb.output(pb.compact_count(keep))
    h = ctx.register(pb.build())
    assert h.info["template"] == "compact" and h.info["compile_events"] == 1 and h.info["n_outputs"] == 3
    p = h.plan([100000])
    assert p["variant_name"] == "compact_vec" and p["n_launches"] == 3
    assert [k.split("k_compact_")[1] for k in p["kernels"]] == ["count_vec", "scan", "scatter_vec"]
    assert p["grid"][1] == [1, 1, 1] and p["block"][1][0] == 1024
    tile = 256 * 4 * p["vec_width"]
    assert p["grid"][0][0] == -(-100000 // tile) and p["workspace_bytes"] == 8 * p["grid"][0][0]
    assert h.plan([0])["n_launches"] == 1 and h.plan([0])["kernels"][0].endswith("k_compact_scan")   # the count is still delivered
    assert h.plan([5], V["compact_scalar"])["vec_width"] == 1
    expect("INVALID_ARG", h.plan, [5], V["loop_vec"])
    # value and predicate share one length by the op's shape propagation: checked at launch
    pb = PatternBuilder()
    a, b = pb.dims(2)
    x = pb.param("f32", [a])
    k = pb.op("gt", pb.param("f32", [b]), pb.const(0.0), dims=[b])
    pb.output(pb.compact(x, k))
    h2 = ctx.register(pb.build())
    assert h2.info["n_dim_classes"] == 1 and h2.plan([7, 7])["n_launches"] == 3
    expect("CONSTRAINT", h2.plan, [7, 8])
    # a second predicate; a compaction result used further; a reduction beside it
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("f32", [n])
    k1 = pb.op("gt", x, pb.const(0.0), dims=[n])
    k2 = pb.op("lt", x, pb.const(0.0), dims=[n])
    pb.output(pb.compact(x, k1))
    pb.output(pb.compact(x, k2))
    assert "share one predicate" in expect("UNFUSIBLE", ctx.register, pb.build())
    pb = PatternBuilder()
    n = pb.dim()
    x = pb.param("f32", [n])
    y = pb.compact(x, pb.op("gt", x, pb.const(0.0), dims=[n]))
    pb.output(pb.op("exp", y))
    assert "only feed OUTPUTs" in expect("UNFUSIBLE", ctx.register, pb.build())
    pb = PatternBuilder()
    t, hh = pb.dims(2)
    x = pb.param("f32", [t, hh])
    pb.output(pb.reduce("sum", x, 1))
    xx = pb.param("f32", [t])
    pb.output(pb.compact(xx, pb.op("gt", xx, pb.const(0.0), dims=[t])))
    expect("UNFUSIBLE", ctx.register, pb.build())
