"""GPU parity over the row-reduce schedules: every class of (lanes per row, slots per lane), ragged
tails of every length, row counts that leave the last block partly filled, rows of several
wavefronts whose slot grid turns from row to row, the staged (LDS) and unstaged kernel versions,
and the streaming version behind the longest register-resident class."""
import os

import numpy as np
import pytest
import torch

from oracle import run as oracle_run
from workloads import PatternBuilder
from workloads.configs import CONFIGS
from tests.util import assert_close, run_gpu, to_oracle_input
from paper_2103_05288_amd import VARIANTS

pytestmark = pytest.mark.gpu

# row lengths chosen around the capacity steps 2 * 2^k and 3 * 2^k slots of 8 elements, plus ragged
# tails 1..7 past a slot boundary
ROW_LENGTHS = [1, 3, 7, 8, 9, 15, 17, 31, 33, 47, 63, 65, 97, 100, 127, 128, 129, 191, 200, 255, 256, 257, 385, 511, 513,
               768, 770, 1023, 1024, 1025, 1100, 1537, 2047, 2048, 2049, 3000, 3073, 4096, 4097, 5739, 6144, 6145, 8191,
               8193, 12289, 16386, 20003, 24576, 24577]


@pytest.fixture(scope="module")
def ctx():
    from paper_2103_05288_amd import Context
    c = Context(0)
    yield c
    c.close()


def check(ctx, cfg_name, dims, seed, handle=None):
    cfg = CONFIGS[cfg_name]
    pat = cfg.pattern()
    h = handle or ctx.register(pat)
    ins = cfg.inputs(dims, seed=seed)
    got = run_gpu(h, pat, dims, ins)
    want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
    plan = h.plan(dims)
    for k, (g, w) in enumerate(zip(got, want)):
        assert_close(g, w, f"{cfg_name} dims={dims} out{k} G={plan['lanes_per_row']} nv={plan['slots_per_lane']} "
                           f"kernel={plan['kernels'][0]}")
    return plan


@pytest.mark.parametrize("cfg_name", ["C2", "C4"])
def test_every_capacity_class_and_tail(ctx, cfg_name):
    h = ctx.register(CONFIGS[cfg_name].pattern())
    seen = set()
    suffixes = set()
    for i, H in enumerate(ROW_LENGTHS):
        T = 1 + (i * 5) % 23            # 1 .. 23 rows: every residue of rows per block shows up
        plan = check(ctx, cfg_name, [T, H], seed=100 + i, handle=h)
        seen.add((plan["variant_name"], plan["lanes_per_row"], plan["slots_per_lane"]))
        name = plan["kernels"][0]
        suffixes.add(name.rsplit("_", 1)[1] if name.rsplit("_", 1)[1] in ("e", "t", "nt") else "")
        # a ragged end on at least 8 lanes in a block of 256 threads is taken as single elements (_t)
        if plan["variant_name"] == "row_reg_vec" and plan["block"][0][0] == 256:
            assert name.endswith("_t") == (H % 8 != 0 and plan["lanes_per_row"] >= 8), (H, name)
    assert {"", "e", "t"} <= suffixes
    lanes = {g for v, g, n in seen if v == "row_reg_vec"}
    assert {4, 8, 16, 32, 64, 128, 256, 512, 1024} <= lanes
    assert {n for v, g, n in seen if v == "row_reg_vec"} >= {1, 2, 3}
    assert any(v == "row_stream_vec" for v, g, n in seen)
    # large launches of rows that start and end on 16-byte boundaries run the non-temporal versions
    rows = lambda H: (100 << 20) // (4 * H)
    assert all(h.plan([rows(H), H])["kernels"][0].endswith("_nt") for H in (128, 768, 2048, 6144))
    assert not any(h.plan([rows(H), H])["kernels"][0].endswith("_nt") for H in (64, 127, 2047, 8192))
    assert not any(h.plan([5, H])["kernels"][0].endswith("_nt") for H in (128, 768, 2048, 6144))


@pytest.mark.parametrize("cfg_name", ["C2", "C4"])
def test_many_rows_per_block_and_turning_grid(monkeypatch, cfg_name):
    """Enough rows that blocks walk several of them (the software pipeline runs past its first row)
    and, for rows of several wavefronts, the slot grid keeps turning.  One round of resident blocks
    keeps the row counts this needs small."""
    from paper_2103_05288_amd import Context
    c = Context(0)
    c.test_option("row_rounds", 1)
    try:
        h = c.register(CONFIGS[cfg_name].pattern())
        for H, T in [(127, 70001), (1100, 9001), (2047, 6000), (3001, 5003), (5739, 6007), (8190, 4500), (20003, 700)]:
            plan = check(c, cfg_name, [T, H], seed=H, handle=h)
            rows_per_block = plan["block"][0][0] // plan["lanes_per_row"]
            assert T > plan["grid"][0][0] * rows_per_block, (H, T, plan["grid"], rows_per_block)
    finally:
        c.close()


def test_non_temporal_versions_any_alignment(monkeypatch):
    """The non-temporal kernel versions forced wherever they exist (rows of whole slots, also small
    launches and short rows that the host rule would leave to the plain versions), and the host rule
    with operands that are not 16-byte aligned: it must fall back to a plain version."""
    from paper_2103_05288_amd import Context
    c = Context(0)
    c.test_option("non_temporal", 1)
    try:
        for cfg_name in ("C2", "C4"):
            h = c.register(CONFIGS[cfg_name].pattern())
            for H, T in [(8, 40), (127, 300), (1000, 77), (2047, 500), (3000, 2003), (6144, 300), (72, 5000)]:
                plan = check(c, cfg_name, [T, H], seed=H + 2, handle=h)
                # (the non-temporal versions are built for rows of whole slots: 8 elements here)
                assert plan["kernels"][0].endswith("_nt") == (H % 8 == 0), plan["kernels"]
        # the loop-fusion kernel and the epilogue of a column reduce have such versions too
        plan = check(c, "C0", [300, 768], seed=9)
        assert plan["kernels"][0].endswith("k_loop_vec_nt"), plan["kernels"]
        plan = check(c, "C3", [3000, 1024], seed=10)
        assert plan["kernels"][-1].endswith("k_col_epi2_vec_nt"), plan["kernels"]
        c.force_variant(VARIANTS.index("col_3stage_vec"))
        check(c, "C3", [3000, 1024], seed=10)
        c.force_variant(-1)
        plan = c.register(CONFIGS["C3"].pattern()).plan([3000, 1024], VARIANTS.index("col_3stage_vec"))
        assert plan["kernels"][-1].endswith("k_col_epi_vec_nt"), plan["kernels"]
    finally:
        c.close()
    c = Context(0)
    try:
        # host rule for the loop kernels: large launches only
        h0 = c.register(CONFIGS["C0"].pattern())
        assert h0.plan([20000, 768])["kernels"][0].endswith("_nt") and not h0.plan([300, 768])["kernels"][0].endswith("_nt")
        # one real launch above the size threshold under the host rule (C2: 6 bytes per element)
        plan = check(c, "C2", [14000, 1024], seed=21)
        assert plan["kernels"][0].endswith("_nt"), plan["kernels"]
        cfg = CONFIGS["C4"]
        pat = cfg.pattern()
        h = c.register(pat)
        dims = [33, 1024]
        ins = cfg.inputs(dims, seed=3)
        want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
        dev = []
        for t in ins:                       # every operand 2 bytes (bf16) or 1 byte past a 16-byte boundary
            flat = torch.empty(t.numel() + 16, dtype=t.dtype, device="cuda")
            view = flat[1:1 + t.numel()].view(t.shape)
            view.copy_(t)
            dev.append(view)
        out_flat = torch.zeros(dims[0] * dims[1] + 16, dtype=torch.bfloat16, device="cuda")
        out = out_flat[1:1 + dims[0] * dims[1]].view(dims)
        # the rule at a size where it applies: aligned (or no) pointers take the version, these do not
        big = [20000, 1024]
        assert h.plan(big)["kernels"][0].endswith("_nt")
        assert not h.plan(big, inputs=[t.data_ptr() for t in dev], outputs=[out.data_ptr()])["kernels"][0].endswith("_nt")
        h.launch(dims, dev, [out])
        torch.cuda.synchronize()
        assert_close(out.cpu(), want[0], "misaligned bases")
        assert float(out_flat[0]) == 0.0 and float(out_flat[-1]) == 0.0
    finally:
        c.close()


def test_unstaged_versions(monkeypatch):
    """The same shapes with LDS staging switched off: the kernel versions that read row vectors from
    global memory in every slot."""
    from paper_2103_05288_amd import Context
    c = Context(0)
    c.test_option("stage_row_vectors", 0)
    try:
        for cfg_name in ("C2", "C4"):
            h = c.register(CONFIGS[cfg_name].pattern())
            for H, T in [(9, 40), (127, 300), (1100, 77), (3001, 2003), (8190, 600), (20003, 40)]:
                plan = check(c, cfg_name, [T, H], seed=H + 1, handle=h)
                assert not plan["kernels"][0].endswith("_s") and plan["lds_bytes"][0] == 0
    finally:
        c.close()


def test_ragged_pieces_every_storage_width(ctx):
    """One pattern with 1-, 2- and 4-byte operands and outputs of each width, so the ragged tail of a
    row moves through the power-of-two pieces of every vector type; the last row ends the tensors, so
    its tail cannot be over-read."""
    pb = PatternBuilder("widths")
    T, H = pb.dims(2)
    a = pb.param("bf16", [T, H])
    b = pb.param("f32", [T, H])
    m = pb.param("bool", [T, H])
    a32 = pb.cast(a, "f32")
    s = pb.reduce("max", pb.op("mul", a32, b), 1)      # a max: no accumulated rounding to cancel against
    y = pb.op("select", m, b, pb.op("add", a32, pb.broadcast(s, [T, H], [0])), dims=[T, H])
    pb.output(y)                                        # f32
    pb.output(pb.cast(y, "f16"))                        # 2 bytes
    pb.output(pb.op("gt", y, pb.const(0.0), dims=[T, H]))   # bool, 1 byte
    pat = pb.build()
    h = ctx.register(pat)
    rng = np.random.default_rng(5)
    for H_ in list(range(1, 18)) + [63, 127, 129, 250, 1001, 4099]:
        for T_ in (1, 5):
            ins = [torch.from_numpy(rng.standard_normal((T_, H_)).astype(np.float32)).to(torch.bfloat16),
                   torch.from_numpy(rng.standard_normal((T_, H_)).astype(np.float32)),
                   torch.from_numpy((rng.random((T_, H_)) < 0.3).astype(np.uint8))]
            got = run_gpu(h, pat, [T_, H_], ins)
            want = oracle_run(pat, [T_, H_], [to_oracle_input(t) for t in ins])[0]
            # the comparison output flips where y is within rounding of zero: compare it only away from 0
            y64 = np.asarray(want[0])
            safe = np.abs(y64) > 1e-4
            assert_close(got[0], want[0], f"widths f32 dims={[T_, H_]}")
            assert_close(got[1], want[1], f"widths f16 dims={[T_, H_]}")
            assert np.array_equal(got[2].numpy()[safe] != 0, np.asarray(want[2])[safe] != 0), [T_, H_]


def test_odd_rows_of_two_byte_elements_any_base_alignment():
    """Rows of an odd number of 2-byte elements start alternately on and two bytes off a dword
    boundary.  A pattern with 2-byte and 1-byte full-size operands and results, an fp32 row vector
    (staged in LDS or not), a sum, a max and an argmax per row; guard cells around every result show
    that nothing is written outside, with bases on a 16-byte boundary and one element past it."""
    from paper_2103_05288_amd import Context
    pb = PatternBuilder("odd_rows")
    T, H = pb.dims(2)
    x = pb.param("bf16", [T, H])
    m = pb.param("bool", [T, H])
    g = pb.param("f32", [H])
    x32 = pb.cast(x, "f32")
    v = pb.op("mul", x32, pb.broadcast(g, [T, H], [1]))
    mx = pb.reduce("max", v, 1)
    am = pb.reduce("argmax", v, 1)
    e = pb.op("exp", pb.op("sub", v, pb.broadcast(mx, [T, H], [0])))
    s = pb.reduce("sum", e, 1)
    y = pb.op("select", m, x32, pb.op("div", e, pb.broadcast(s, [T, H], [0])), dims=[T, H])
    pb.output(pb.cast(y, "bf16"))
    pb.output(pb.cast(pb.op("add", y, v), "f16"))
    pb.output(pb.op("gt", v, pb.const(0.25), dims=[T, H]))
    pb.output(am)
    pb.output(s)
    pat = pb.build()
    rng = np.random.default_rng(11)
    out_dt = [torch.bfloat16, torch.float16, torch.bool, torch.int32, torch.float32]

    def run(c, h, dims, ins, skew):
        """Launch with every full-size tensor `skew` elements past a 16-byte boundary and guards around the results."""
        T_, H_ = dims
        dev = []
        for t in ins:
            if t.dim() == 2:
                flat = torch.zeros(t.numel() + 32, dtype=t.dtype, device="cuda")
                view = flat[16 + skew:16 + skew + t.numel()].view(t.shape)
                view.copy_(t)
                dev.append(view)
            else:
                dev.append(t.cuda())
        flats, outs = [], []
        for dt, full in zip(out_dt, (True, True, True, False, False)):
            n = T_ * H_ if full else T_
            flat = torch.full((n + 32,), 1, dtype=dt, device="cuda")
            flats.append(flat)
            outs.append(flat[16 + skew:16 + skew + n].view((T_, H_) if full else (T_,)))
        h.launch(dims, dev, outs)
        torch.cuda.synchronize()
        for f, o in zip(flats, outs):
            fc = f.cpu()
            assert bool((fc[:16 + skew] == 1).all()) and bool((fc[16 + skew + o.numel():] == 1).all()), f"guard cells dims={dims} skew={skew}"
        return [o.cpu() for o in outs]

    for stage in (1, 0):
        c = Context(0)
        c.test_option("stage_row_vectors", stage)
        c.test_option("row_rounds", 1)
        try:
            h = c.register(pat)
            shapes = [(2, 5), (3, 9), (5, 33), (64, 127), (1001, 129), (7, 511), (300, 1023), (33, 1025), (4100, 3001),
                      (6000, 4095), (9, 6143), (2500, 8191), (5, 24575), (70001, 127)]
            for T_, H_ in shapes:
                ins = [torch.from_numpy(rng.standard_normal((T_, H_)).astype(np.float32)).to(torch.bfloat16),
                       torch.from_numpy((rng.random((T_, H_)) < 0.3)),
                       torch.from_numpy((0.5 + rng.random(H_)).astype(np.float32))]
                print(f"[odd rows] stage={stage} dims={[T_, H_]}", flush=True)
                want = oracle_run(pat, [T_, H_], [to_oracle_input(t) for t in ins])[0]
                v64 = np.asarray(ins[0].float().numpy(), dtype=np.float64) * np.asarray(ins[2].numpy(), dtype=np.float64)[None, :]
                for skew in (0, 1):          # bf16 / f16 tensors: dword aligned, then two bytes off
                    got = run(c, h, [T_, H_], ins, skew)
                    what = f"odd rows dims={[T_, H_]} stage={stage} skew={skew}"
                    assert_close(got[0], want[0], what + " out0")
                    assert_close(got[1], want[1], what + " out1")
                    safe = np.abs(v64 - 0.25) > 1e-5
                    assert np.array_equal(got[2].numpy()[safe], np.asarray(want[2])[safe] != 0), what + " out2"
                    # argmax: the position may differ only where two products tie to fp32 rounding
                    ga = got[3].numpy().astype(np.int64)
                    wa = np.asarray(want[3]).astype(np.int64)
                    rows_ = np.arange(T_)
                    assert np.all((ga >= 0) & (ga < H_)), what
                    assert np.all(np.abs(v64[rows_, ga] - v64[rows_, wa]) <= 1e-6 * np.abs(v64[rows_, wa])), what + " argmax"
                    assert_close(got[4], want[4], what + " out4")
        finally:
            c.close()


def test_single_element_ends_in_fp32_and_f16_patterns(ctx):
    """The versions that take the ragged ends of a row as single elements, at other vector widths
    than the benchmark patterns': an fp32 softmax (4 elements per slot, up to 3 single elements at
    either end -- fp32 rows always start on dword boundaries, so they are never shifted) and an f16
    one with a row-group mask (8 per slot; odd rows are shifted), at seeded random row lengths."""
    rng = np.random.default_rng(23)
    for dt, tdt in (("f32", torch.float32), ("f16", torch.float16)):
        pb = PatternBuilder("softmax_" + dt)
        B, S, H = pb.dims(3)
        x = pb.param(dt, [B, S, H])
        m = pb.param(dt, [B, pb.static(1), H])
        v = pb.op("add", pb.cast(x, "f32"), pb.cast(pb.broadcast(m, [B, S, H], [0, 1, 2]), "f32"))
        mx = pb.reduce("max", v, 2)
        e = pb.op("exp", pb.op("sub", v, pb.broadcast(mx, [B, S, H], [0, 1])))
        s = pb.reduce("sum", e, 2)
        pb.output(pb.cast(pb.op("div", e, pb.broadcast(s, [B, S, H], [0, 1])), dt))
        pb.output(mx)
        pat = pb.build()
        h = ctx.register(pat)
        seen_t = 0
        for _ in range(14):
            Hh = int(rng.integers(33, 3000))
            Bb, Ss = int(rng.integers(1, 4)), int(rng.integers(1, 300))
            dims = [Bb, Ss, Hh]
            xs = torch.from_numpy(rng.standard_normal((Bb, Ss, Hh)).astype(np.float32)).to(tdt)
            ms = torch.from_numpy((rng.random((Bb, 1, Hh)) < 0.2).astype(np.float32) * -50.0).to(tdt)
            got = run_gpu(h, pat, dims, [xs, ms])
            want = oracle_run(pat, dims, [to_oracle_input(xs), to_oracle_input(ms)])[0]
            plan = h.plan(dims)
            seen_t += plan["kernels"][0].endswith("_t")
            for k, (g, w) in enumerate(zip(got, want)):
                assert_close(g, w, f"softmax {dt} dims={dims} out{k} kernel={plan['kernels'][0]}")
        assert seen_t >= 5
