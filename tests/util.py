"""Helpers shared by the tests: comparator bars and the GPU / oracle drivers."""
import numpy as np
import torch

from workloads.configs import TORCH_DTYPE

# Parity bars, element-wise.
#  fp32 outputs:        |gpu - oracle| <= 1e-5 |oracle| + 1e-6
#  f16 / bf16 outputs:  the value is computed in fp32 (same 1e-5 / 1e-6 bar on the arithmetic) and then
#                       rounded ONCE to the storage type, which alone costs up to half a unit in the last
#                       place of that type:  |gpu - oracle| <= 0.5 ulp_T(x) + 1e-5 |oracle| + 1e-6.
#                       For f16 (half ulp <= 2^-11 |x|) this is inside the "rel 2e-3" bar; for bf16 the
#                       rounding alone reaches 2^-8 |x| = 3.9e-3 |x|, so no correctly rounded bf16 result can
#                       meet a blanket 2e-3: the bar keeps the arithmetic at the fp32 tolerance and adds
#                       exactly the unavoidable storage rounding, element by element.
#  integer outputs:     bit-exact
RTOL, ATOL = 1e-5, 1e-6
MANT_BITS = {"f16": (10, -14), "bf16": (7, -126)}    # explicit mantissa bits, minimum normal exponent


def ulp(x: np.ndarray, kind: str) -> np.ndarray:
    bits, emin = MANT_BITS[kind]
    ax = np.abs(x)
    e = np.floor(np.log2(np.where(ax > 0, ax, 1.0)))
    e = np.maximum(e, emin)
    return np.exp2(e - bits)


def to_oracle_input(t: torch.Tensor) -> np.ndarray:
    """Storage tensor -> numpy array the oracle takes (every f16/bf16 value is exact in float64)."""
    t = t.detach().cpu()
    if t.dtype in (torch.float16, torch.bfloat16, torch.float32):
        return t.to(torch.float64).numpy()
    return t.numpy()


def alloc_outputs(pattern, dims, device):
    outs = []
    for i in pattern.outputs:
        op = pattern.ops[i]
        outs.append(torch.empty(pattern.shape_of(i, dims), dtype=TORCH_DTYPE[op.dtype], device=device))
    return outs


def run_gpu(handle, pattern, dims, inputs, device="cuda", poison=True, workspace=None):
    # an empty operand still needs an address (the ABI refuses null pointers): any allocation will do
    dev_in = [t.to(device).contiguous() if t.numel() else torch.zeros(16, dtype=t.dtype, device=device) for t in inputs]
    outs = alloc_outputs(pattern, dims, device)
    if poison:
        for o in outs:
            if o.dtype.is_floating_point:
                o.fill_(float("nan"))
            else:
                o.fill_(-7 if o.dtype != torch.uint8 else 255)
    if workspace is None:
        need = handle.ctx.workspace_bytes(handle.id, dims)
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=device)
    handle.launch(dims, dev_in, outs, workspace=workspace)
    torch.cuda.synchronize()
    return [o.cpu() for o in outs]


def assert_close(got: torch.Tensor, want: np.ndarray, what: str = ""):
    if not got.dtype.is_floating_point:
        g = got.numpy().astype(np.int64)
        w = np.asarray(want).astype(np.int64)
        assert g.shape == w.shape, (what, g.shape, w.shape)
        bad = np.nonzero(g != w)
        assert bad[0].size == 0, f"{what}: {bad[0].size} index mismatches, first at {[b[0] for b in bad]}"
        return
    g = got.to(torch.float64).numpy()
    w = np.asarray(want, dtype=np.float64)
    assert g.shape == w.shape, (what, g.shape, w.shape)
    err = np.abs(g - w)
    lim = RTOL * np.abs(w) + ATOL
    if got.dtype in (torch.float16, torch.bfloat16):
        kind = "f16" if got.dtype == torch.float16 else "bf16"
        lim = lim + 0.5 * ulp(np.maximum(np.abs(g), np.abs(w)), kind)
    bad = ~(err <= lim)          # NaN-safe: a NaN on either side fails
    if bad.any():
        idx = np.unravel_index(np.argmax(np.where(bad, err - lim, -np.inf)), g.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {g.size} elements outside the {got.dtype} bar; "
                             f"worst at {tuple(int(i) for i in idx)}: gpu={g[idx]!r} oracle={w[idx]!r} "
                             f"err={err[idx]:.3e} limit={lim[idx]:.3e}")
