#!/usr/bin/env python3
"""Benchmark of the shape-generic fusion kernels on one MI355X.

One "step" = one pass of the whole hot path over the five benchmark configurations' dynamic-shape
sweeps (C0 8 calls, C1 32, C2 48, C3 200, C4 1000; every call a different runtime shape, every
pattern compiled once).  Inputs are resident in HBM before the timed region starts.

  value = algorithmic bytes of one step / wall time of one step            (GB/s)

Algorithmic bytes = every input read once + every output written once.  The JSON line also carries
the roofline of the dominant kernel (the C4 row-reduce version that moves the most bytes), a CPU
baseline (the unfused fp64 oracle timed on a bounded sample of the same workload) and per-config
detail.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from workloads.configs import CONFIGS, TORCH_DTYPE, algorithmic_bytes  # noqa: E402

PEAK_HBM_GBPS = 8000.0


def _fill_normal(buf: torch.Tensor, seed: int, chunk: int = 1 << 27):
    g = torch.Generator(device=buf.device)
    g.manual_seed(seed)
    flat = buf.view(-1)
    for a in range(0, flat.numel(), chunk):
        b = min(flat.numel(), a + chunk)
        tmp = torch.empty(b - a, dtype=torch.float32, device=buf.device)
        tmp.normal_(0.0, 1.0, generator=g)
        flat[a:b] = tmp.to(buf.dtype)
        del tmp


class Arena:
    """A flat pre-filled device buffer; tensors for a call are views at a rotating offset so that
    consecutive calls do not re-read what the previous call left in cache."""

    def __init__(self, numel: int, dtype, device, fill, seed):
        self.buf = torch.empty(numel, dtype=dtype, device=device)
        self.pos = 0
        self.align = 256 // self.buf.element_size()
        if fill == "normal":
            _fill_normal(self.buf, seed)
        elif fill == "uniform":
            g = torch.Generator(device=device)
            g.manual_seed(seed)
            self.buf.uniform_(-1.0, 1.0, generator=g)
        elif fill == "mask":
            g = torch.Generator(device=device)
            g.manual_seed(seed)
            chunk = 1 << 28
            for a in range(0, numel, chunk):
                b = min(numel, a + chunk)
                self.buf[a:b] = (torch.rand(b - a, device=device, generator=g) < 0.1).to(dtype)

    def take(self, shape, shift=0):
        """`shift` elements past the 256-byte aligned position: deliberately misaligned operands."""
        n = int(np.prod(shape))
        if self.pos + n + shift > self.buf.numel():
            self.pos = 0
        v = self.buf[self.pos + shift:self.pos + shift + n].view(*shape)
        self.pos += (n + shift + self.align - 1) // self.align * self.align
        return v


class Sweep:
    """All calls of one configuration with their device tensors bound."""

    def __init__(self, name, ctx, device):
        self.name = name
        self.cfg = CONFIGS[name]
        self.pattern = self.cfg.pattern()
        self.handle = ctx.register(self.pattern)
        self.calls = self.cfg.calls()
        self.bytes = [algorithmic_bytes(self.pattern, d) for d in self.calls]
        self.bound = []          # (dims, inputs, outputs, workspace)
        self.device = device
        self._bind(ctx)

    def _bind(self, ctx):
        dev = self.device
        pat = self.pattern
        in_shapes = lambda d: [pat.shape_of(i, d) for i in pat.params]
        out_shapes = lambda d: [pat.shape_of(i, d) for i in pat.outputs]
        n_in, n_out = len(pat.params), len(pat.outputs)
        # one arena per tensor slot, sized for twice the largest call (so the offset can rotate)
        max_in = [max(int(np.prod(in_shapes(d)[k])) for d in self.calls) for k in range(n_in)]
        max_out = [max(int(np.prod(out_shapes(d)[k])) for d in self.calls) for k in range(n_out)]
        sum_in = [sum(int(np.prod(in_shapes(d)[k])) for d in self.calls) for k in range(n_in)]
        arenas_in = []
        for k, pi in enumerate(pat.params):
            dt = TORCH_DTYPE[pat.ops[pi].dtype]
            numel = min(sum_in[k] + 4096 * len(self.calls), 2 * max_in[k] + 4096)
            fill = "mask" if pat.ops[pi].dtype == "bool" else ("uniform" if self.name == "C3" else "normal")
            arenas_in.append(Arena(numel, dt, dev, fill, seed=1000 + 17 * k + 101 * int(self.name[1:])))
        arenas_out = [Arena(2 * max_out[k] + 4096, TORCH_DTYPE[pat.ops[oi].dtype], dev, None, 0)
                      for k, oi in enumerate(pat.outputs)]
        ws_need = max(ctx.workspace_bytes(self.handle.id, d) for d in self.calls)
        self.workspace = torch.empty(max(ws_need, 256), dtype=torch.uint8, device=dev)
        self.bound_shifted = []
        # second pass over the same arenas: every operand and result one element past its 256-byte
        # aligned position (the labelled misaligned-bases sweep)
        for shift in (0, 1):
            rng = np.random.default_rng(4242)
            for a in arenas_in + arenas_out:
                a.pos = 0
            for d in self.calls:
                ins = [arenas_in[k].take(s, shift) for k, s in enumerate(in_shapes(d))]
                if self.name == "C1":
                    # real key-padding mask (0 / -1e4) from per-batch valid lengths
                    B, NH, S = d
                    lens = torch.from_numpy(rng.integers(1, S + 1, size=B)).to(dev)
                    keys = torch.arange(S, device=dev).view(1, 1, 1, S)
                    ins[1] = torch.where(keys < lens.view(B, 1, 1, 1), 0.0, -1.0e4).to(torch.float16).contiguous()
                if self.name == "C0":
                    ins[1] = ins[1] * 0.02
                if self.name == "C2":
                    ins[3] = (ins[3].float() * 0.1 + 1.0).to(ins[3].dtype)
                    ins[4] = (ins[4].float() * 0.1).to(ins[4].dtype)
                outs = [arenas_out[k].take(s, shift) for k, s in enumerate(out_shapes(d))]
                (self.bound if shift == 0 else self.bound_shifted).append((d, ins, outs))
        # arguments marshalled once per call site; the timed loop is one C call per launch
        self.calls_bound = [self.handle.bind(d, ins, outs, workspace=self.workspace) for d, ins, outs in self.bound]
        self.calls_shifted = [self.handle.bind(d, ins, outs, workspace=self.workspace) for d, ins, outs in self.bound_shifted]

    def bind_streams(self, streams):
        """The same calls dealt out round-robin over several streams (independent requests may
        overlap their ramp-up and drain); every stream gets a workspace of its own."""
        ws = [torch.empty_like(self.workspace) for _ in streams]
        self.calls_multi = [self.handle.bind(d, ins, outs, workspace=ws[i % len(streams)], stream=streams[i % len(streams)].cuda_stream)
                            for i, (d, ins, outs) in enumerate(self.bound)]
        self._multi_keep = ws

    def run_all_multi(self):
        for c in self.calls_multi:
            c()

    def run_all(self):
        for c in self.calls_bound:
            c()

    def run_all_shifted(self):
        for c in self.calls_shifted:
            c()

    def run_one(self, i):
        self.calls_bound[i]()

    def timed_calls(self):
        """Per-call device time inside a back-to-back sweep: one event between consecutive launches on
        the launch stream, one synchronisation at the end."""
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(self.calls_bound) + 1)]
        evs[0].record()
        for i, c in enumerate(self.calls_bound):
            c()
            evs[i + 1].record()
        evs[-1].synchronize()
        return [evs[i].elapsed_time(evs[i + 1]) * 1e-3 for i in range(len(self.calls_bound))]


def time_events(fn, stream=None):
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    a.record()
    fn()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) * 1e-3


# Hot shapes for the gap-to-static comparison (Section 5.3 of the paper: shape-generic kernels reach
# 85 % of static-shape ones on average): the same pattern registered shape-generic and compiled for
# the one shape (extents and launch plan as compile-time constants, only that shape's kernel version).
GAP_SHAPES = {
    "C0": [[512, 768]],
    "C1": [[8, 12, 384], [8, 12, 505]],
    "C2": [[16384, 1024], [4096, 4096], [9000, 768]],
    "C3": [[65536, 1024], [300, 1024]],
    "C4": [[65536, 2048], [46773, 5739], [200000, 127], [16384, 8192]],
}


def gap_to_static(ctx, names, dev):
    from workloads.configs import CONFIGS, TORCH_DTYPE, algorithmic_bytes
    rows = []
    for name in names:
        cfg = CONFIGS[name]
        pat = cfg.pattern()
        generic = ctx.register(pat)                      # cache hit: registered by the sweep already
        for dims in GAP_SHAPES.get(name, []):
            ins = cfg.inputs(dims, seed=77, device=dev)
            outs_g = [torch.empty(pat.shape_of(o, dims), dtype=TORCH_DTYPE[pat.ops[o].dtype], device=dev) for o in pat.outputs]
            outs_s = [torch.empty_like(o) for o in outs_g]
            ws = torch.empty(max(16, ctx.workspace_bytes(generic.id, dims)), dtype=torch.uint8, device=dev)
            static = ctx.register_static(pat, dims)
            cg = generic.bind(dims, ins, outs_g, workspace=ws)
            cs = static.bind(dims, ins, outs_s, workspace=ws)

            def rate(call):
                call()
                torch.cuda.synchronize()
                t = min(time_events(lambda: [call() for _ in range(10)]) for _ in range(3)) / 10
                return algorithmic_bytes(pat, dims) / t / 1e9
            g, s = rate(cg), rate(cs)
            diff = max(float((a.double() - b.double()).abs().max()) if a.numel() else 0.0 for a, b in zip(outs_g, outs_s))
            rows.append({"cfg": name, "dims": dims, "generic_GBps": round(g, 1), "static_GBps": round(s, 1),
                         "generic_over_static": round(g / s, 4), "static_compile_ms": round(static.info["compile_ms"], 1),
                         "max_abs_diff_outputs": diff, "kernel": generic.plan(dims)["kernels"][0]})
            del ins, outs_g, outs_s, ws
    ratios = [r["generic_over_static"] for r in rows]
    return {"shapes": rows, "mean_generic_over_static": round(float(np.mean(ratios)), 4) if ratios else None,
            "min": min(ratios) if ratios else None, "max": max(ratios) if ratios else None,
            "static_compiles": len(rows),
            "note": "static = the same op list compiled for that one shape (a module per shape); generic = the one "
                    "shape-generic module used by the whole sweep"}


def graph_replay(sweeps):
    """The same launches recorded once into a HIP graph per configuration and replayed: what is left
    when the host's per-call work (shape calculation, version selection, the launch call) and the
    dispatch gaps between dependent launches are taken out.  Not the headline: a recorded graph has
    its shapes fixed, which is what the method exists to avoid; the figure only shows how much of
    the small-call configurations is launch latency."""
    out = {}
    side = torch.cuda.Stream()
    for sw in sweeps:
        calls = [sw.handle.bind(d, ins, outs, workspace=sw.workspace, stream=side.cuda_stream) for d, ins, outs in sw.bound]
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for c in calls:
                    c()
        torch.cuda.current_stream().wait_stream(side)
        graph.replay()
        torch.cuda.synchronize()
        t = min(time_events(graph.replay) for _ in range(3))
        out[sw.name] = {"sweep_ms": round(t * 1e3, 4), "GBps_sweep": round(sum(sw.bytes) / t / 1e9, 1)}
        del graph
    return out


def next_rows(ctx, dev):
    """Secondary figures, outside the headline value: the op-graph path and the indexing functions
    on inputs (slice, pad, transpose) at one large shape each; effective rate = bytes of the
    graph's / pattern's inputs and outputs, each once, over the device time of one call."""
    from workloads.configs import TORCH_DTYPE
    from workloads.extras import (gelu_backward_bias_gradient, heads_softmax, layernorm_backward_graph,
                                  logsumexp_with_total_and_amax, padded_softmax, pure_transpose, qkv_split, unique_of_sorted)

    def io_bytes(pat, dims):
        n = 0
        for v in list(pat.params) + list(pat.outputs):
            n += int(np.prod(pat.shape_of(v, dims))) * torch.empty(0, dtype=TORCH_DTYPE[pat.ops[v].dtype]).element_size()
        return n

    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    rows = {}
    # ~1 GB of operands and results per call: nothing of a call survives in the 256 MB memory-side cache
    cases = [("graph_layernorm_backward", layernorm_backward_graph(), [131072, 1024], True),
             ("gelu_backward_bias_gradient", gelu_backward_bias_gradient(), [131072, 1024], False),
             ("logsumexp_total_amax", logsumexp_with_total_and_amax(), [262144, 2048], False),
             ("slice_qkv_split", qkv_split(), [131072, 1024, 3072, 1024, 2048], False),
             ("pad_softmax_minus_inf", padded_softmax(), [131072, 2000, 24, 2048], False),
             ("transpose_heads_softmax", heads_softmax(), [128, 1024, 16, 128], False),
             ("transpose_tile_bf16", pure_transpose("bf16", (1, 0)), [16384, 16384], False)]
    for name, pat, dims, is_graph in cases:
        ins = [torch.randn(pat.shape_of(pi, dims), device=dev, generator=gen).to(TORCH_DTYPE[pat.ops[pi].dtype]) for pi in pat.params]
        outs = [torch.empty(pat.shape_of(o, dims), dtype=TORCH_DTYPE[pat.ops[o].dtype], device=dev) for o in pat.outputs]
        if is_graph:
            h = ctx.register_graph(pat)
            ws = torch.empty(max(16, h.workspace_bytes(dims)), dtype=torch.uint8, device=dev)
            call = lambda: h.launch(dims, ins, outs, workspace=ws)
            extra = {"patterns": h.info["n_patterns"], "planned_buffers": h.info["n_buffers"], "workspace_bytes": int(ws.numel()),
                     "kernel_prefixes": ["disc_p%d_" % p for p in h.info["pattern_id"][:h.info["n_patterns"]]]}
        else:
            h = ctx.register(pat)
            ws = torch.empty(max(16, ctx.workspace_bytes(h.id, dims)), dtype=torch.uint8, device=dev)
            call = h.bind(dims, ins, outs, workspace=ws)
            extra = {"kernels": h.plan(dims)["kernels"], "template": h.info["template"]}
        call()
        torch.cuda.synchronize()
        t = min(time_events(lambda: [call() for _ in range(10)]) for _ in range(3)) / 10
        rows[name] = dict({"dims": dims, "io_bytes": io_bytes(pat, dims), "us": round(t * 1e6, 2),
                           "GBps": round(io_bytes(pat, dims) / t / 1e9, 1)}, **extra)
        del ins, outs, ws
    # an output whose size depends on the data: Unique of a sorted tensor (about one value in sixteen
    # is new).  Bytes = the input, the index of every element, and what was actually kept.
    pat = unique_of_sorted("i32")
    n = 1 << 27
    x = torch.sort(torch.randint(0, n // 16, (n,), device=dev, generator=gen, dtype=torch.int32)).values
    outs = [torch.empty(n, dtype=torch.int32, device=dev), torch.empty(n, dtype=torch.int32, device=dev),
            torch.zeros(1, dtype=torch.int64, device=dev)]
    h = ctx.register(pat)
    ws = torch.empty(max(16, ctx.workspace_bytes(h.id, [n])), dtype=torch.uint8, device=dev)
    call = h.bind([n], [x], outs, workspace=ws)
    call()
    torch.cuda.synchronize()
    kept = int(outs[2][0])
    t = min(time_events(lambda: [call() for _ in range(10)]) for _ in range(3)) / 10
    moved = 4 * n + 4 * n + 4 * kept + 8
    rows["unique_of_sorted_i32"] = {"dims": [n], "kept": kept, "io_bytes": moved, "us": round(t * 1e6, 2),
                                    "GBps": round(moved / t / 1e9, 1), "kernels": h.plan([n])["kernels"], "template": h.info["template"],
                                    "expected_traffic_over_io_bytes": round((8 * n + 4 * n + 4 * kept) / moved, 3),
                                    "note": "three launches; the input is read twice (count pass, scatter pass)"}
    del x, outs, ws
    return rows


def mix_ceiling(ctx, dev):
    """The practical ceiling for the row kernels' traffic mix: streaming probes that move 3 bytes read :
    2 written per element with one 1-byte stream (the 12-op pattern) and 4 : 2 (residual + LayerNorm)
    and do next to no arithmetic, plain and non-temporal, swept over the grid size and the bytes in
    flight per lane.  The best rate of each mix is what the fused kernels are compared with."""
    n = 1 << 27                                   # elements of 2 bytes: 256 MB per 2-byte stream
    a = torch.zeros(n, dtype=torch.int16, device=dev)
    b = torch.zeros(n, dtype=torch.int16, device=dev)
    m = torch.zeros(n, dtype=torch.uint8, device=dev)
    out = torch.empty(n, dtype=torch.int16, device=dev)
    res = {}
    for kind, name, bytes_per_elem in ((0, "read3_write2_with_byte_stream", 5), (1, "read4_write2", 6)):
        rows = []
        for nt in (0, 1):
            for u in (1, 2, 4, 8):
                for bpc in (2, 4, 8, 16, 32):
                    call = lambda: ctx.util_mix(kind, nt, u, bpc, out, a, m if kind == 0 else b, n)
                    call()
                    torch.cuda.synchronize()
                    t = min(time_events(call) for _ in range(3))
                    rows.append({"non_temporal": nt, "slots_in_flight": u, "blocks_per_cu": bpc,
                                 "GBps": round(bytes_per_elem * n / t / 1e9, 1)})
        best = max(rows, key=lambda r: r["GBps"])
        best_plain = max((r for r in rows if not r["non_temporal"]), key=lambda r: r["GBps"])
        res[name] = {"best": best, "best_plain": best_plain, "configs_tried": len(rows),
                     "worst_GBps": min(r["GBps"] for r in rows)}
    del a, b, m, out
    return res


def accuracy_report(sweeps, rows_per_call=48, calls_per_cfg=4):
    """16-bit outputs against the oracle on sampled rows, outside the timed region: the largest
    relative error with no absolute term (over |oracle| > 1e-3) and the fraction of those elements
    beyond 2e-3 -- the literal bar of the benchmark spec, which a correctly rounded bf16 value can
    miss by itself (half a unit in the last place of bf16 is up to 2^-8 = 3.9e-3 of the value)."""
    from oracle import run as oracle_run
    out = {}
    for sw in sweeps:
        pat = sw.pattern
        kinds = {pat.ops[o].dtype for o in pat.outputs}
        if not (kinds & {"f16", "bf16"}):
            continue
        order = np.argsort(sw.bytes)
        picks = [int(order[int(q * (len(order) - 1))]) for q in np.linspace(0.35, 1.0, calls_per_cfg)]
        worst, n_all, n_bad, worst_ulp = 0.0, 0, 0, 0.0
        for i in picks:
            d, ins, outs = sw.bound[i]
            sw.run_one(i)
            torch.cuda.synchronize()
            lead = d[0]
            lo = max(0, lead // 2 - rows_per_call // 2)
            hi = min(lead, lo + rows_per_call) if sw.name != "C1" else min(lead, lo + 1)
            sub, dims = [], list(d)
            dims[0] = hi - lo
            for t, pi in zip(ins, pat.params):
                op = pat.ops[pi]
                t = t[lo:hi] if (len(op.dims) >= 1 and op.dims[0] == 0) else t
                t = t.cpu()
                sub.append(t.to(torch.float64).numpy() if t.dtype.is_floating_point else t.numpy())
            want = oracle_run(pat, dims, sub)[0]
            for o_t, w, oi in zip(outs, want, pat.outputs):
                if pat.ops[oi].dtype not in ("f16", "bf16"):
                    continue
                g = o_t[lo:hi].cpu().to(torch.float64).numpy()
                sel = np.abs(w) > 1e-3
                rel = np.abs(g - w)[sel] / np.abs(w)[sel]
                if rel.size:
                    worst = max(worst, float(rel.max()))
                    n_all += int(rel.size)
                    n_bad += int((rel > 2e-3).sum())
                    bits = 7 if pat.ops[oi].dtype == "bf16" else 10
                    ulp = np.exp2(np.floor(np.log2(np.abs(w)[sel])) - bits)
                    worst_ulp = max(worst_ulp, float((np.abs(g - w)[sel] / ulp).max()))
        out[sw.name] = {"storage": sorted(kinds & {"f16", "bf16"})[0], "calls_checked": len(picks), "elements": n_all,
                        "max_rel_err_atol0": float("%.3e" % worst), "fraction_beyond_2e-3": float("%.3e" % (n_bad / max(1, n_all))),
                        "max_err_in_ulps_of_storage": round(worst_ulp, 3)}
    return out


def cpu_baseline(sweeps, budget_s=20.0):
    """Oracle (as it stands) on a bounded sample of the sweep: per configuration the calls in order of
    element count, smallest first, none above 256 MiB, until that configuration's share of the time
    budget is used; row-independent patterns are evaluated in row chunks on a thread pool (numpy
    releases the GIL inside ufuncs)."""
    from oracle import run as oracle_run
    cores = min(os.cpu_count() or 1, 16)
    pool = ThreadPoolExecutor(max_workers=cores)
    total_bytes, total_s, n_calls = 0, 0.0, 0
    per_cfg_budget = budget_s / len(sweeps)
    detail = {}
    for sw in sweeps:
        pat = sw.pattern
        used, b, n = 0.0, 0, 0
        order = np.argsort([int(np.prod(d)) for d in sw.calls])      # small shapes first: bounded work
        for i in order:
            d, ins, _ = sw.bound[i]
            if sw.bytes[i] > (1 << 28):
                continue
            host = [t.cpu() for t in ins]
            host = [t.to(torch.float64).numpy() if t.dtype.is_floating_point else t.numpy() for t in host]
            t0 = time.perf_counter()
            rows = d[0]
            row_split = sw.name in ("C0", "C2", "C4") and rows >= 2 * cores
            if row_split:
                # rows are independent: same results as one call, evaluated chunk by chunk
                bounds = np.linspace(0, rows, cores + 1).astype(int)
                def work(k):
                    lo, hi = bounds[k], bounds[k + 1]
                    if hi <= lo:
                        return None
                    # slice the operands whose leading axis is the row dim (symbolic dim 0)
                    sub = [h[lo:hi] if (len(pat.ops[pi].dims) >= 1 and pat.ops[pi].dims[0] == 0) else h
                           for h, pi in zip(host, pat.params)]
                    return oracle_run(pat, [hi - lo] + list(d[1:]), sub)[0]
                list(pool.map(work, range(cores)))
            else:
                oracle_run(pat, d, host)
            dt = time.perf_counter() - t0
            used += dt
            b += sw.bytes[i]
            n += 1
            if used > per_cfg_budget:
                break
        detail[sw.name] = {"calls": n, "seconds": round(used, 3), "GBps": round(b / used / 1e9, 4) if used > 0 else None}
        total_bytes += b
        total_s += used
        n_calls += n
    pool.shutdown()
    return {"value": round(total_bytes / total_s / 1e9, 4), "unit": "GB/s", "cores": cores, "host_cpu_count": os.cpu_count(),
            "kind": "oracle",
            "sample": f"{n_calls} smallest-first calls of the C0-C4 sweeps (<= 256 MiB each), ~{budget_s:.0f} s of CPU work; "
                      "C0/C2/C4 row-chunked over a thread pool, C1/C3 one numpy call",
            "per_config": detail}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--configs", default="C0,C1,C2,C3,C4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gap-to-static", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true")
    ap.add_argument("--next-rows-only", action="store_true",
                    help="time the secondary workloads alone (plus the plain copy the traffic counters are scaled by) "
                         "and print them as one JSON line; what the profiles of those kernels are taken from")
    ap.add_argument("--streams", type=int, default=1, help="streams the calls of the timed step are dealt out over")
    ap.add_argument("--cpu-budget", type=float, default=20.0)
    ap.add_argument("--dump-calls", default="", help="write per-call dims / bytes / device time as JSON lines")
    ap.add_argument("--one-call", default="", metavar="CFG:DIMS",
                    help="launch ONE call of one configuration a few times (e.g. C4:65536,4096) and print its plan and "
                         "rate as one JSON line; what the per-kernel counter passes under profiles/ are taken from")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    from paper_2103_05288_amd import Context
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ctx = Context(0)
    if args.one_call:
        name, dims_s = args.one_call.split(":")
        dims = [int(x) for x in dims_s.split(",")]
        cfg = CONFIGS[name]
        pat = cfg.pattern()
        h = ctx.register(pat)
        ins = cfg.inputs(dims, seed=3, device="cuda")
        outs = [torch.empty(pat.shape_of(o, dims), dtype=TORCH_DTYPE[pat.ops[o].dtype], device=dev) for o in pat.outputs]
        ws = torch.empty(max(16, ctx.workspace_bytes(h.id, dims)), dtype=torch.uint8, device=dev)
        call = h.bind(dims, ins, outs, workspace=ws)
        call()
        torch.cuda.synchronize()
        t = min(time_events(call) for _ in range(3))
        plan = h.plan(dims)
        print(json.dumps({"mode": "one_call", "config": name, "dims": dims, "kernels": plan["kernels"],
                          "grid": plan["grid"][:plan["n_launches"]], "block": plan["block"][:plan["n_launches"]],
                          "lanes_per_row": plan["lanes_per_row"], "slots_per_lane": plan["slots_per_lane"],
                          "launches": 4, "us": round(t * 1e6, 2),
                          "GBps": round(algorithmic_bytes(pat, dims) / t / 1e9, 1)}))
        return
    if args.next_rows_only:
        n_copy = 1 << 30
        src = torch.zeros(n_copy, dtype=torch.uint8, device=dev)
        dst = torch.empty(n_copy, dtype=torch.uint8, device=dev)
        ctx.util_copy(dst, src, n_copy)
        torch.cuda.synchronize()
        t_copy = min(time_events(lambda: [ctx.util_copy(dst, src, n_copy) for _ in range(10)]) for _ in range(3)) / 10
        del src, dst
        print(json.dumps({"mode": "next_rows_only", "copy_ceiling_GBps": round(2 * n_copy / t_copy / 1e9, 1),
                          "next_rows": next_rows(ctx, dev)}))
        return
    names = [n for n in args.configs.split(",") if n]
    t_setup = time.perf_counter()
    sweeps = [Sweep(n, ctx, dev) for n in names]
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup

    streams = [torch.cuda.Stream() for _ in range(args.streams)] if args.streams > 1 else []
    for sw in sweeps:
        if streams:
            sw.bind_streams(streams)

    def step():
        for sw in sweeps:
            sw.run_all_multi() if streams else sw.run_all()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    step_bytes = sum(sum(sw.bytes) for sw in sweeps)
    ms_per_step = wall / args.steps * 1e3
    value = step_bytes / (wall / args.steps) / 1e9

    # ---- per-config and per-call device times (HIP events on the launch stream), after the timed region
    per_cfg = {}
    dominant = None
    for sw in sweeps:
        sw.run_all()
        torch.cuda.synchronize()
        t_cfg = min(time_events(sw.run_all) for _ in range(3))
        per_call = [min(a, b) for a, b in zip(sw.timed_calls(), sw.timed_calls())]
        plans = [sw.handle.plan(d) for d in sw.calls]
        if args.dump_calls:
            with open(args.dump_calls, "a") as f:
                for d, b, t, pl in zip(sw.calls, sw.bytes, per_call, plans):
                    f.write(json.dumps({"cfg": sw.name, "dims": d, "bytes": b, "us": round(t * 1e6, 2), "G": pl["lanes_per_row"],
                                        "nv": pl["slots_per_lane"], "grid": pl["grid"][0][0] if pl["grid"] else 0,
                                        "variant": pl["variant_name"]}) + "\n")
        by_kernel = {}
        for i, pl in enumerate(plans):
            key = "+".join(pl["kernels"])          # entry-point symbols, as rocprofv3 shows them
            e = by_kernel.setdefault(key, {"launches": 0, "bytes": 0, "seconds": 0.0})
            e["launches"] += 1
            e["bytes"] += sw.bytes[i]
            e["seconds"] += per_call[i]
        long_rows = [i for i, pl in enumerate(plans) if pl["inner"] >= 1024]
        big = [i for i in range(len(sw.calls)) if sw.bytes[i] >= (32 << 20)]
        gb = lambda idx: (sum(sw.bytes[i] for i in idx) / max(1e-12, sum(per_call[i] for i in idx)) / 1e9) if idx else None
        sw.run_all_shifted()
        torch.cuda.synchronize()
        t_shift = min(time_events(sw.run_all_shifted) for _ in range(3))
        n_launch = [pl["n_launches"] for pl in plans]
        per_cfg[sw.name] = {
            "calls": len(sw.calls), "bytes": sum(sw.bytes), "sweep_ms": round(t_cfg * 1e3, 4),
            "device_launches": int(sum(n_launch)),
            "GBps_sweep_misaligned_bases": round(sum(sw.bytes) / t_shift / 1e9, 1),
            "GBps_sweep": round(sum(sw.bytes) / t_cfg / 1e9, 1),
            "GBps_sum_of_calls": round(gb(list(range(len(sw.calls)))), 1),
            "GBps_rows_ge_1024": None if gb(long_rows) is None else round(gb(long_rows), 1),
            "GBps_calls_ge_32MiB": None if gb(big) is None else round(gb(big), 1),
            "median_call_us": round(float(np.median(per_call)) * 1e6, 2),
            "compile_events": sw.handle.ctx.pattern_info(sw.handle.id)["compile_events"],
            "compile_ms": round(sw.handle.info["compile_ms"], 1),
            "kernels": {k: {"launches": v["launches"], "GBps": round(v["bytes"] / v["seconds"] / 1e9, 1),
                            "avg_us": round(v["seconds"] / v["launches"] * 1e6, 2)} for k, v in by_kernel.items()},
        }
        if sw.name == "C4" or dominant is None:
            k, v = max(by_kernel.items(), key=lambda kv: kv[1]["bytes"])
            dominant = (sw.name, k, v)

    # ---- practical ceiling (plain 16-byte copy, 1 GiB) and launch floor
    n_copy = 1 << 30
    src = torch.empty(n_copy, dtype=torch.uint8, device=dev)
    dst = torch.empty(n_copy, dtype=torch.uint8, device=dev)
    src.zero_()
    ctx.util_copy(dst, src, n_copy)
    torch.cuda.synchronize()
    t_copy = min(time_events(lambda: [ctx.util_copy(dst, src, n_copy) for _ in range(10)]) for _ in range(3)) / 10
    copy_gbps = 2 * n_copy / t_copy / 1e9
    ctx.util_copy(dst, src, n_copy, non_temporal=True)
    torch.cuda.synchronize()
    t_copy_nt = min(time_events(lambda: [ctx.util_copy(dst, src, n_copy, non_temporal=True) for _ in range(10)]) for _ in range(3)) / 10
    copy_nt_gbps = 2 * n_copy / t_copy_nt / 1e9
    del src, dst
    ctx.util_empty_launch()
    torch.cuda.synchronize()
    t_empty = time_events(lambda: [ctx.util_empty_launch() for _ in range(1000)]) / 1000
    st = ctx.stats()
    host_us = st["host_launch_ns"] / max(1, st["launch_calls"]) / 1e3     # includes waiting for queue space
    plan_us = st["host_plan_ns"] / max(1, st["launch_calls"]) / 1e3
    # the same with an empty queue: a tiny call of the first sweep, synchronised every 32 launches
    sw0 = sweeps[0]
    small = min(range(len(sw0.calls)), key=lambda i: sw0.bytes[i])
    s0 = ctx.stats()
    for i in range(2048):
        sw0.calls_bound[small]()
        if i % 32 == 31:
            torch.cuda.synchronize()
    s1 = ctx.stats()
    host_idle_us = (s1["host_launch_ns"] - s0["host_launch_ns"]) / 2048 / 1e3

    # latency-adjusted bound: a call cannot finish faster than its launches' fixed cost t0 plus its
    # bytes at the peak rate; t0 = the measured back-to-back cost of an empty launch
    for sw in sweeps:
        pc = per_cfg[sw.name]
        plans = [sw.handle.plan(d) for d in sw.calls]
        bound_s = sum(pl["n_launches"] * t_empty + b / (PEAK_HBM_GBPS * 1e9) for pl, b in zip(plans, sw.bytes))
        pc["latency_adjusted_bound_GBps"] = round(sum(sw.bytes) / bound_s / 1e9, 1)
        pc["frac_of_latency_adjusted_bound"] = round(pc["GBps_sweep"] / pc["latency_adjusted_bound_GBps"], 4)
    mix = mix_ceiling(ctx, dev)
    mix_best = {"C4": mix["read3_write2_with_byte_stream"]["best"]["GBps"], "C2": mix["read4_write2"]["best"]["GBps"]}

    dom_name, dom_kernel, dom = dominant
    achieved = dom["bytes"] / dom["seconds"] / 1e9
    # measured HBM traffic per launch of that kernel over the same sweep (rocprofv3 FETCH_SIZE / WRITE_SIZE,
    # scaled by what the counters read for the plain copy kernel): recorded under profiles/
    traffic, traffic_commit = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        rec = tj.get(dom_kernel)
        traffic = rec["bytes_per_launch"] if rec else None
        traffic_commit = tj.get("_commit")
    roofline = {"bound": "hbm", "kernel": f"{dom_name}:{dom_kernel}", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBPS,
                "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBPS, 4), "traffic": traffic,
                "launches": dom["launches"], "avg_launch_us": round(dom["seconds"] / dom["launches"] * 1e6, 2),
                "bytes_per_launch": int(dom["bytes"] / dom["launches"]),
                "traffic_source": "profiles/traffic.json (rocprofv3 FETCH_SIZE / WRITE_SIZE passes over this command)"
                                  + (f" at commit {traffic_commit}" if traffic_commit else ""),
                "frac_of_copy_ceiling": round(achieved / copy_gbps, 4),
                "mix_ceiling_GBps": mix_best.get(dom_name),
                "frac_of_mix_ceiling": round(achieved / mix_best[dom_name], 4) if dom_name in mix_best else None}

    out = {
        "metric": "effective HBM GB/s over the dynamic-shape sweep (C0-C4), one compile per pattern",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "+".join(names) + " dynamic-shape sweeps: " +
                   ", ".join(f"{sw.name} {len(sw.calls)} calls" for sw in sweeps),
                   "bytes_per_step": step_bytes, "calls_per_step": sum(len(sw.calls) for sw in sweeps),
                   "storage": "f32 / f16 / bf16 / bool tensors, fp32 arithmetic, f64 accumulation of fp32 column sums"},
        "pct_of_peak": round(100 * value / PEAK_HBM_GBPS, 2),
        "roofline": roofline,
        "copy_ceiling_GBps": round(copy_gbps, 1),
        "copy_nt_ceiling_GBps": round(copy_nt_gbps, 1),
        "mix_ceiling": mix,
        "rows_ge_1024_vs_mix_ceiling": {n: round(per_cfg[n]["GBps_rows_ge_1024"] / mix_best[n], 4)
                                        for n in mix_best if n in per_cfg and per_cfg[n]["GBps_rows_ge_1024"]},
        "accuracy_16bit_outputs": accuracy_report(sweeps),
        "empty_launch_us": round(t_empty * 1e6, 2),
        "host_launch_us_per_call": round(host_idle_us, 2), "host_plan_us_per_call": round(plan_us, 3),
        "host_launch_us_per_call_queue_full": round(host_us, 2),
        "kernels_compiled_per_pattern": {sw.name: per_cfg[sw.name]["compile_events"] for sw in sweeps},
        "per_config": per_cfg,
        "setup_s": round(setup_s, 1),
    }
    if not args.no_gap_to_static:
        out["gap_to_static"] = gap_to_static(ctx, names, dev)
    if not args.no_next_rows:
        out["next_rows"] = next_rows(ctx, dev)
        out["graph_replay"] = graph_replay(sweeps)
        if not streams:
            # the same step with its (independent) calls dealt out over four streams: ramp-up and
            # drain of consecutive kernels overlap.  A secondary figure; the headline, the roofline
            # object and the profiles are all single-stream.
            four = [torch.cuda.Stream() for _ in range(4)]
            for sw in sweeps:
                sw.bind_streams(four)
            for sw in sweeps:
                sw.run_all_multi()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                for sw in sweeps:
                    sw.run_all_multi()
            torch.cuda.synchronize()
            w4 = (time.perf_counter() - t0) / args.steps
            out["multi_stream"] = {"streams": 4, "value": round(step_bytes / w4 / 1e9, 1), "ms_per_step": round(w4 * 1e3, 3)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(sweeps, args.cpu_budget)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
