"""The five benchmark configurations: op lists, seeded shape draws, seeded values.

Each configuration stands in for a memory-bound sub-graph of the paper's
workloads (Table 1: Transformer / BERT / Seq2seq / ASR / TTS with varying
sequence length; Section 2 on the neglect of dynamic shapes): bias+GELU,
masked attention softmax, residual+LayerNorm, a column reduction with a
broadcast epilogue and a long mixed chain.  The paper's own models, weights and
data are not public; everything here is synthetic and seeded.

Only descriptions live here: the op lists say WHAT is computed, the draws say
at which runtime shapes, the fillers produce input values.  No arithmetic of
the method itself (no fused expression, no reduction) is implemented here.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, List, Sequence

import numpy as np
import torch

from .pattern import Pattern, PatternBuilder

TORCH_DTYPE = {
    "f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16,
    "i32": torch.int32, "i64": torch.int64, "bool": torch.uint8,
}
DTYPE_BYTES = {"f32": 4, "f16": 2, "bf16": 2, "i32": 4, "i64": 8, "bool": 1}


# --------------------------------------------------------------------------
# op lists
# --------------------------------------------------------------------------
def c0_pattern() -> Pattern:
    """y = gelu_tanh(x + b) + r, fp32; x, r: [T,H], b: [H]."""
    pb = PatternBuilder("c0_bias_gelu_residual")
    T, H = pb.dims(2)
    x = pb.param("f32", [T, H])
    b = pb.param("f32", [H])
    r = pb.param("f32", [T, H])
    u = pb.op("add", x, pb.broadcast(b, [T, H], [1]))
    c0 = pb.const(0.7978845608028654)      # sqrt(2/pi)
    c1 = pb.const(0.044715)
    u3 = pb.op("mul", pb.op("mul", u, u), u)
    z = pb.op("mul", c0, pb.op("add", u, pb.op("mul", c1, u3)), dims=[T, H])
    one = pb.const(1.0)
    half = pb.const(0.5)
    g = pb.op("mul", pb.op("mul", half, u, dims=[T, H]), pb.op("add", one, pb.op("tanh", z), dims=[T, H]))
    y = pb.op("add", g, r)
    pb.output(y)
    return pb.build()


def c1_pattern() -> Pattern:
    """softmax over the last axis of x*0.125 + mask; x: [B,NH,S,S] f16, mask: [B,1,1,S] f16."""
    pb = PatternBuilder("c1_masked_softmax")
    B, NH, S = pb.dims(3)
    full = [B, NH, S, S]
    x = pb.param("f16", full)
    mask = pb.param("f16", [B, pb.static(1), pb.static(1), S])
    xf = pb.cast(x, "f32")
    mf = pb.cast(mask, "f32")
    a = pb.op("add", pb.op("mul", xf, pb.const(0.125)), pb.broadcast(mf, full, [0, 1, 2, 3]))
    m = pb.reduce("max", a, 3)
    e = pb.op("exp", pb.op("sub", a, pb.broadcast(m, full, [0, 1, 2])))
    s = pb.reduce("sum", e, 3)
    y = pb.op("div", e, pb.broadcast(s, full, [0, 1, 2]))
    pb.output(pb.cast(y, "f16"))
    return pb.build()


def c2_pattern() -> Pattern:
    """LayerNorm(x + r + bias) * gamma + beta over the last axis; all bf16 storage."""
    pb = PatternBuilder("c2_residual_bias_layernorm")
    T, H = pb.dims(2)
    x = pb.param("bf16", [T, H])
    r = pb.param("bf16", [T, H])
    b = pb.param("bf16", [H])
    gamma = pb.param("bf16", [H])
    beta = pb.param("bf16", [H])
    f = lambda v: pb.cast(v, "f32")
    row = lambda v: pb.broadcast(v, [T, H], [0])     # [T] -> [T,H]
    col = lambda v: pb.broadcast(v, [T, H], [1])     # [H] -> [T,H]
    v = pb.op("add", pb.op("add", f(x), f(r)), col(f(b)))
    hs = pb.dim_size(H)
    mu = pb.op("div", pb.reduce("sum", v, 1), hs)
    d = pb.op("sub", v, row(mu))
    var = pb.op("div", pb.reduce("sum", pb.op("mul", d, d), 1), hs)
    rstd = pb.op("rsqrt", pb.op("add", var, pb.const(1e-5)))
    n = pb.op("mul", d, row(rstd))
    y = pb.op("add", pb.op("mul", n, col(f(gamma))), col(f(beta)))
    pb.output(pb.cast(y, "bf16"))
    return pb.build()


def c3_pattern() -> Pattern:
    """sum[c] = sum_t x[t,c]; mean = sum / T; y = x - mean; fp32; three outputs."""
    pb = PatternBuilder("c3_colsum_mean_center")
    T, C = pb.dims(2)
    x = pb.param("f32", [T, C])
    s = pb.reduce("sum", x, 0)
    mean = pb.op("div", s, pb.dim_size(T))
    y = pb.op("sub", x, pb.broadcast(mean, [T, C], [1]))
    pb.output(s)
    pb.output(mean)
    pb.output(y)
    return pb.build()


def c4_pattern() -> Pattern:
    """The mixed 12-op chain (cast, two broadcasts, row max, sub, exp, row sum, div,
    select, rsqrt-scaled residual, cast back); bf16 in / out."""
    pb = PatternBuilder("c4_mixed12")
    T, H = pb.dims(2)
    x = pb.param("bf16", [T, H])
    mask = pb.param("bool", [T, H])
    bH = pb.param("f32", [H])
    cT = pb.param("f32", [T, pb.static(1)])
    row = lambda v: pb.broadcast(v, [T, H], [0])
    x32 = pb.cast(x, "f32")                                   # 1 cast
    a = pb.op("add", x32, pb.broadcast(bH, [T, H], [1]))      # 2 + [H]
    b = pb.op("add", a, pb.broadcast(cT, [T, H], [0, 1]))     # 3 + [T,1]
    m = pb.reduce("max", b, 1)                                # 4 row max
    c = pb.op("sub", b, row(m))                               # 5
    e = pb.op("exp", c)                                       # 6
    s = pb.reduce("sum", e, 1)                                # 7 row sum
    p = pb.op("div", e, row(s))                               # 8
    q = pb.op("select", mask, pb.const(0.0), p, dims=[T, H])  # 9 true -> zeroed
    w = pb.op("rsqrt", s)                                     # 10
    y32 = pb.op("add", q, pb.op("mul", x32, row(w)))          # 11 scaled residual
    pb.output(pb.cast(y32, "bf16"))                           # 12 cast back
    return pb.build()


# --------------------------------------------------------------------------
# seeded shape draws (numpy default_rng: reproducible on any machine)
# --------------------------------------------------------------------------
def _log_uniform_int(rng, lo: int, hi: int, n: int) -> np.ndarray:
    u = rng.uniform(math.log2(lo), math.log2(hi), size=n)
    return np.clip(np.rint(2.0 ** u), lo, hi).astype(np.int64)


def c0_calls(seed: int = 1000, n: int = 8) -> List[List[int]]:
    rng = np.random.default_rng(seed)
    return [[int(t), 768] for t in rng.integers(1, 513, size=n)]


def c1_calls(seed: int = 1001, n: int = 32) -> List[List[int]]:
    rng = np.random.default_rng(seed)
    return [[8, 12, int(s)] for s in rng.integers(16, 513, size=n)]


def c2_calls(seed: int = 1002, n_per_h: int = 16) -> List[List[int]]:
    rng = np.random.default_rng(seed)
    calls = []
    for h in (768, 1024, 4096):
        for _ in range(n_per_h):
            calls.append([int(rng.integers(1, 513, size=64).sum()), h])
    return calls


def c3_calls(seed: int = 1003, n: int = 200) -> List[List[int]]:
    rng = np.random.default_rng(seed)
    return [[int(t), 1024] for t in _log_uniform_int(rng, 1, 65536, n)]


def c4_calls(seed: int = 1004, n: int = 1000) -> List[List[int]]:
    rng = np.random.default_rng(seed)
    ts = _log_uniform_int(rng, 1, 1 << 20, n)
    hs = _log_uniform_int(rng, 64, 8192, n)
    return [[int(t), int(h)] for t, h in zip(ts, hs)]


# --------------------------------------------------------------------------
# seeded values
# --------------------------------------------------------------------------
def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, dtype, g, device, mean=0.0, std=1.0):
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(mean, std, generator=g)
    return t.to(dtype)


def c0_inputs(dims: Sequence[int], seed: int, device="cpu"):
    T, H = dims
    g = _gen(seed, device)
    return [_randn((T, H), torch.float32, g, device),
            _randn((H,), torch.float32, g, device, 0.0, 0.02),
            _randn((T, H), torch.float32, g, device)]


def c1_inputs(dims: Sequence[int], seed: int, device="cpu"):
    B, NH, S = dims
    g = _gen(seed, device)
    x = _randn((B, NH, S, S), torch.float16, g, device)
    # key-padding mask from per-batch valid lengths L_b ~ U{1..S}: 0 on valid keys, -1e4 after
    lens = torch.randint(1, S + 1, (B,), generator=g, device=device)
    keys = torch.arange(S, device=device).view(1, 1, 1, S)
    mask = torch.where(keys < lens.view(B, 1, 1, 1), 0.0, -1.0e4).to(torch.float16)
    return [x, mask]


def c2_inputs(dims: Sequence[int], seed: int, device="cpu"):
    T, H = dims
    g = _gen(seed, device)
    bf = torch.bfloat16
    return [_randn((T, H), bf, g, device), _randn((T, H), bf, g, device),
            _randn((H,), bf, g, device),
            _randn((H,), bf, g, device, 1.0, 0.1), _randn((H,), bf, g, device, 0.0, 0.1)]


def c3_inputs(dims: Sequence[int], seed: int, device="cpu"):
    T, C = dims
    g = _gen(seed, device)
    x = torch.empty((T, C), dtype=torch.float32, device=device)
    x.uniform_(-1.0, 1.0, generator=g)
    return [x]


def c4_inputs(dims: Sequence[int], seed: int, device="cpu"):
    T, H = dims
    g = _gen(seed, device)
    x = _randn((T, H), torch.bfloat16, g, device)
    mask = (torch.rand((T, H), generator=g, device=device) < 0.1).to(torch.uint8)
    bH = _randn((H,), torch.float32, g, device)
    cT = _randn((T, 1), torch.float32, g, device)
    return [x, mask, bH, cT]


# --------------------------------------------------------------------------
# algorithmic bytes: every distinct input byte read once + every output byte
# written once (what the fused method itself has to move)
# --------------------------------------------------------------------------
def algorithmic_bytes(pattern: Pattern, dims: Sequence[int]) -> int:
    total = 0
    for i, op in enumerate(pattern.ops):
        if op.opcode in ("param", "output"):
            n = 1
            for s in pattern.shape_of(i, dims):
                n *= s
            total += n * DTYPE_BYTES[op.dtype]
    return total


@dataclass(frozen=True)
class Config:
    name: str
    pattern: Callable[[], Pattern]
    calls: Callable[..., List[List[int]]]
    inputs: Callable[..., list]


CONFIGS = {
    "C0": Config("C0", c0_pattern, c0_calls, c0_inputs),
    "C1": Config("C1", c1_pattern, c1_calls, c1_inputs),
    "C2": Config("C2", c2_pattern, c2_calls, c2_inputs),
    "C3": Config("C3", c3_pattern, c3_calls, c3_inputs),
    "C4": Config("C4", c4_pattern, c4_calls, c4_inputs),
}
