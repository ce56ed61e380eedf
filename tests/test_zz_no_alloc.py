"""disc_launch_static_scratch (the entry point for callers that cannot allocate) against disc_launch
with a caller's workspace: same kernels, so the outputs must agree bit for bit -- two calls in a
row, the second with a smaller input (what the first call left in the array must not matter) --
and against the oracle to the usual bar.  Shapes beyond the array's size are refused."""
import pytest
import torch

from oracle import run as oracle_run
from workloads import extras
from workloads.configs import CONFIGS, TORCH_DTYPE
from tests.util import alloc_outputs, assert_close, run_gpu, to_oracle_input

pytestmark = pytest.mark.gpu

SCRATCH_BYTES = 16 << 20


@pytest.fixture(scope="module")
def ctx():
    from paper_2103_05288_amd import Context
    c = Context(0)
    yield c
    c.close()


def _both_ways(ctx, h, pat, dims, ins, what):
    dev = [t.cuda().contiguous() for t in ins]
    ref = run_gpu(h, pat, dims, ins)                       # disc_launch with a torch workspace
    outs = alloc_outputs(pat, dims, "cuda")
    for o in outs:
        o.fill_(float("nan")) if o.dtype.is_floating_point else o.fill_(-7)
    torch.cuda.synchronize()
    ctx.launch_static_scratch(h.id, dims, dev, outs)
    torch.cuda.synchronize()
    for k, (a, b) in enumerate(zip(outs, ref)):
        assert torch.equal(a.cpu().view(torch.uint8), b.view(torch.uint8)), f"{what} dims={dims} out{k}: differs from disc_launch"
    want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
    for k, (g, w) in enumerate(zip(outs, want)):
        assert_close(g.cpu(), w, f"{what} dims={dims} out{k}")


def test_static_scratch_matches_disc_launch_twice_second_smaller(ctx):
    # column reduce through three launches (partials and reduce results live in the scratch array)
    cfg = CONFIGS["C3"]
    pat = cfg.pattern()
    h = ctx.register(pat)
    for dims in ([5000, 1024], [2500, 1024], [4097, 1333]):
        assert h.plan(dims)["workspace_bytes"] > 0 and h.plan(dims)["n_launches"] >= 2
        print(f"[static scratch] C3 dims={dims}", flush=True)
        _both_ways(ctx, h, pat, dims, cfg.inputs(dims, seed=dims[0]), "C3")
    # row reduce that carries column sums (LayerNorm backward): partial rows in the scratch array
    pat = extras.layernorm_backward_graph()
    h = ctx.register(pat)
    g = torch.Generator().manual_seed(3)
    for dims in ([3000, 512], [700, 200]):
        x = torch.randn(dims, generator=g).to(torch.bfloat16)
        dy = torch.randn(dims, generator=g).to(torch.bfloat16)
        gam = torch.randn(dims[1], generator=g)
        assert h.plan(dims)["workspace_bytes"] > 0
        print(f"[static scratch] LayerNorm backward dims={dims}", flush=True)
        dev = [t.cuda() for t in (x, dy, gam)]
        ref = run_gpu(h, pat, dims, [x, dy, gam])
        outs = alloc_outputs(pat, dims, "cuda")
        ctx.launch_static_scratch(h.id, dims, dev, outs)
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(zip(outs, ref)):
            assert torch.equal(a.cpu().view(torch.uint8), b.view(torch.uint8)), f"LN backward dims={dims} out{k}"
    # a pattern without scratch memory goes straight through
    cfg = CONFIGS["C4"]
    pat = cfg.pattern()
    h = ctx.register(pat)
    _both_ways(ctx, h, pat, [37, 777], cfg.inputs([37, 777], seed=1), "C4")


def test_static_scratch_refuses_what_does_not_fit(ctx):
    from paper_2103_05288_amd import DiscError
    pat = extras.layernorm_backward_graph()
    h = ctx.register(pat)
    dims = [1 << 20, 8192]                      # ~1000 partial rows x 8192 columns x 2 sums x 4 bytes > 16 MiB
    need = h.plan(dims)["workspace_bytes"]
    assert need > SCRATCH_BYTES
    # nothing is dereferenced before the size check: tiny stand-in tensors are enough
    t = torch.zeros(16, device="cuda")
    with pytest.raises(DiscError) as e:
        ctx.launch_static_scratch(h.id, dims, [t, t, t], [t, t, t])
    assert e.value.status == "WORKSPACE" and "DISC_STATIC_SCRATCH_BYTES" in e.value.message
