"""Outputs whose size depends on the input values (Section 2: Unique-style ops) on the GPU against the
oracle: Unique of a sorted tensor (values, the index of every element, the count), and compaction by a
predicate that a fused chain computes.  Index and integer outputs bit-exact; the part of an output
buffer beyond the data-dependent length must stay untouched; the count arrives in device memory."""
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


def unique_sorted(dtype):
    pb = PatternBuilder("unique_sorted")
    n = pb.dim()
    x = pb.param(dtype, [n])
    keep = pb.ne_prev(x)
    pb.output(pb.compact(x, keep))
    pb.output(pb.compact_rank(keep, "i32"))
    pb.output(pb.compact_count(keep, "i64"))
    return pb.build()


def filtered():
    """keep = tanh(x) * w > thr; outputs: x + 1 (bf16), w as i32, the slots (i64), the count (i32)."""
    pb = PatternBuilder("filter")
    n = pb.dim()
    x = pb.param("bf16", [n])
    w = pb.param("f32", [n])
    thr = pb.param("f32", [])
    xf = pb.cast(x, "f32")
    keep = pb.op("gt", pb.op("mul", pb.op("tanh", xf), w), thr, dims=[n])
    pb.output(pb.compact(pb.cast(pb.op("add", xf, pb.const(1.0), dims=[n]), "bf16"), keep))
    pb.output(pb.compact(pb.cast(w, "i32"), keep))
    pb.output(pb.compact_rank(keep, "i64"))
    pb.output(pb.compact_count(keep, "i32"))
    return pb.build()


def check(ctx, pat, dims, ins, what, force=None):
    from paper_2103_05288_amd import VARIANTS
    h = ctx.register(pat)
    if force:
        ctx.force_variant(VARIANTS.index(force))
    try:
        got = run_gpu(h, pat, dims, ins)                  # outputs are poisoned first (NaN / -7)
    finally:
        ctx.force_variant(-1)
    want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
    counts = [int(np.asarray(w)) for w, o in zip(want, pat.outputs) if pat.ops[pat.ops[o].ins[0]].opcode == "compact_count"]
    for k, (g, w, o) in enumerate(zip(got, want, pat.outputs)):
        oc = pat.ops[pat.ops[o].ins[0]].opcode
        w = np.asarray(w)
        if oc == "compact":
            n = w.shape[0]
            assert not counts or counts[0] == n
            head, tail = g[:n], g[n:]
            if g.dtype.is_floating_point:
                assert_close(head, w, f"{what} dims={dims} out{k}")
                assert bool(torch.isnan(tail).all()), f"{what} dims={dims} out{k}: written beyond the data-dependent length"
            else:
                assert np.array_equal(head.numpy().astype(np.int64), w.astype(np.int64)), f"{what} dims={dims} out{k}"
                assert bool((tail == -7).all()), f"{what} dims={dims} out{k}: written beyond the data-dependent length"
        else:
            assert np.array_equal(g.numpy().astype(np.int64).reshape(w.shape), w.astype(np.int64)), f"{what} dims={dims} out{k} ({oc})"
    return h


@pytest.mark.parametrize("dtype", ["i32", "i64", "f32"])
def test_unique_of_sorted_tensor(ctx, dtype):
    pat = unique_sorted(dtype)
    tdt = {"i32": torch.int32, "i64": torch.int64, "f32": torch.float32}[dtype]
    g = torch.Generator().manual_seed(11)
    # ragged sizes around the tile sizes (256 lanes x 4 slots x 2 or 4 elements), one element, long runs, no repeats
    for n, spread in ((1, 3), (2, 1), (7, 2), (2047, 50), (2048, 5), (2049, 100000), (4095, 7), (4096, 900), (4097, 3), (5000, 1),
                      (100003, 300), (1 << 20, 40000)):
        x = torch.sort(torch.randint(-spread, spread + 1, (n,), generator=g, dtype=torch.int64)).values
        if dtype == "i64":
            x = x * 3000000007            # beyond 32 bits
        print(f"[unique] {dtype} n={n} spread={spread}", flush=True)
        check(ctx, pat, [n], [x.to(tdt)], f"unique {dtype}")
    # all equal (one value kept) and strictly increasing (everything kept)
    check(ctx, pat, [3000], [torch.full((3000,), 5, dtype=tdt)], "all equal")
    check(ctx, pat, [3000], [torch.arange(3000, dtype=tdt)], "all distinct")
    check(ctx, pat, [3000], [torch.arange(3000, dtype=tdt)], "all distinct, scalar version", force="compact_scalar")
    assert ctx.pattern_info(ctx.register(pat).id)["compile_events"] == 1


def test_compaction_by_a_fused_predicate(ctx):
    pat = filtered()
    g = torch.Generator().manual_seed(12)
    for n in (1, 100, 4097, 70001, 300000):
        x = (torch.randn(n, generator=g) * 2).to(torch.bfloat16)
        w = torch.round(torch.randn(n, generator=g) * 4)
        # none kept, all kept, about half, few (products are exact multiples of tanh: no near-ties with the thresholds)
        for thr in (1e9, -1e9, 0.0, 3.3):
            print(f"[filter] n={n} thr={thr}", flush=True)
            check(ctx, pat, [n], [x, w, torch.tensor(thr)], f"filter thr={thr}")
    check(ctx, pat, [4097], [x[:4097], w[:4097], torch.tensor(0.0)], "filter scalar version", force="compact_scalar")


def test_empty_input_still_delivers_the_count(ctx):
    pat = unique_sorted("i32")
    h = ctx.register(pat)
    outs = [torch.full((16,), -7, dtype=torch.int32, device="cuda"), torch.full((16,), -7, dtype=torch.int32, device="cuda"),
            torch.full((1,), -7, dtype=torch.int64, device="cuda")]
    ws = torch.empty(max(16, ctx.workspace_bytes(h.id, [0])), dtype=torch.uint8, device="cuda")
    h.launch([0], [torch.zeros(16, dtype=torch.int32, device="cuda")], outs, workspace=ws)
    torch.cuda.synchronize()
    assert int(outs[2][0]) == 0 and bool((outs[0] == -7).all()) and bool((outs[1] == -7).all())
    # the same call twice gives the same bits (no atomics anywhere)
    x = torch.sort(torch.randint(0, 1000, (50000,), generator=torch.Generator().manual_seed(1))).values.to(torch.int32)
    a = run_gpu(h, pat, [50000], [x])
    b = run_gpu(h, pat, [50000], [x])
    assert all(torch.equal(p, q) for p, q in zip(a, b))
