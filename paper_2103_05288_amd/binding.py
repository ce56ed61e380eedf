"""ctypes binding of libdisc.so: same names as the C ABI, marshalling only.

There is no CPU fallback: if the library is missing, importing this module's
``load_library`` raises; if no GPU is present, launches return an error code.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))

MAX_RANK, MAX_DIMS = 4, 16

DTYPE_IDS = {"f32": 0, "f16": 1, "bf16": 2, "i32": 3, "i64": 4, "bool": 5}
_OPCODES = ("param", "const", "dim_size", "neg", "abs", "exp", "log", "tanh", "sqrt", "rsqrt", "rcp",
            "sigmoid", "erf", "add", "sub", "mul", "div", "max", "min", "pow", "lt", "le", "gt", "ge",
            "eq", "ne", "select", "cast", "broadcast", "reduce_sum", "reduce_max", "reduce_min",
            "reduce_argmax", "output", "slice", "pad", "transpose", "ne_prev", "compact", "compact_count", "compact_rank")
OPCODE_IDS = {n: i for i, n in enumerate(_OPCODES)}
VARIANTS = ("loop_vec", "loop_vec_i64", "loop_scalar", "loop_scalar_i64", "row_reg_vec", "row_reg_scalar",
            "row_stream_vec", "row_stream_scalar", "col_3stage_vec", "col_3stage_scalar", "col_strip_vec",
            "col_strip_scalar", "transpose_tile", "col_2stage_vec", "col_2stage_scalar",
            "compact_vec", "compact_scalar")
STATUS = {0: "OK", -1: "INVALID_ARG", -2: "BAD_PATTERN", -3: "UNFUSIBLE", -4: "CONSTRAINT", -5: "WORKSPACE",
          -6: "COMPILE", -7: "HIP", -8: "SHAPE", -9: "EMPTY_REDUCE", -10: "INTERNAL"}
TEST_OPTIONS = {"non_temporal": 0, "stage_row_vectors": 1, "row_rounds": 2, "align_row_slots": 3}
TEMPLATES = ("loop", "row_reduce", "col_reduce", "transpose", "compact")


class disc_op(C.Structure):
    _fields_ = [("opcode", C.c_int32), ("dtype", C.c_int32), ("in_", C.c_int32 * 3), ("rank", C.c_int32),
                ("dim", C.c_int32 * MAX_RANK), ("axis_map", C.c_int32 * MAX_RANK), ("fconst", C.c_double)]


class disc_constraint(C.Structure):
    _fields_ = [("kind", C.c_int32), ("a_value", C.c_int32), ("a_axis", C.c_int32),
                ("b_value", C.c_int32), ("b_axis", C.c_int32)]


class disc_pattern_info_t(C.Structure):
    _fields_ = [("template_kind", C.c_int32), ("n_dims", C.c_int32), ("n_inputs", C.c_int32),
                ("n_outputs", C.c_int32), ("compile_events", C.c_int32), ("n_variants", C.c_int32),
                ("n_phases", C.c_int32), ("vec_width", C.c_int32), ("n_collapsed", C.c_int32),
                ("n_dim_classes", C.c_int32), ("dim_class", C.c_int32 * MAX_DIMS), ("compile_ms", C.c_double)]


MAX_GRAPH_PATTERNS = 64
MAX_OPS = 256


class disc_graph_info_t(C.Structure):
    _fields_ = [("n_dims", C.c_int32), ("n_inputs", C.c_int32), ("n_outputs", C.c_int32), ("n_patterns", C.c_int32),
                ("n_intermediates", C.c_int32), ("n_buffers", C.c_int32), ("pattern_id", C.c_int32 * MAX_GRAPH_PATTERNS),
                ("pattern_ops", C.c_int32 * MAX_GRAPH_PATTERNS), ("group_of_op", C.c_int32 * MAX_OPS)]


class disc_plan_t(C.Structure):
    _fields_ = [("variant", C.c_int32), ("n_launches", C.c_int32), ("index_bits", C.c_int32),
                ("vec_width", C.c_int32), ("lanes_per_row", C.c_int32), ("slots_per_lane", C.c_int32),
                ("reg_slots", C.c_int32), ("grid", (C.c_uint32 * 3) * 3), ("block", (C.c_uint32 * 3) * 3),
                ("lds_bytes", C.c_uint32 * 3), ("kernel", (C.c_char * 48) * 3), ("rows", C.c_int64), ("inner", C.c_int64), ("mid", C.c_int64),
                ("algorithmic_bytes", C.c_int64), ("workspace_bytes", C.c_size_t)]


class disc_stats_t(C.Structure):
    _fields_ = [("patterns_registered", C.c_int64), ("pattern_cache_hits", C.c_int64),
                ("compile_events", C.c_int64), ("launch_calls", C.c_int64), ("device_launches", C.c_int64),
                ("variant_count", C.c_int64 * len(VARIANTS)), ("host_plan_ns", C.c_int64),
                ("host_launch_ns", C.c_int64)]


class DiscError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"DISC_ERR_{STATUS.get(code, code)}: {message}")
        self.code = code
        self.status = STATUS.get(code, str(code))
        self.message = message


EXPORTS = ("disc_create", "disc_destroy", "disc_last_error", "disc_register_pattern", "disc_register_pattern_static",
           "disc_pattern_info",
           "disc_pattern_source", "disc_workspace_bytes", "disc_plan", "disc_launch", "disc_force_variant", "disc_test_option",
           "disc_static_scratch_init", "disc_launch_static_scratch",
           "disc_get_stats", "disc_util_copy", "disc_util_copy_nt", "disc_util_empty_launch", "disc_util_mix", "disc_register_graph", "disc_graph_info",
           "disc_graph_workspace_bytes", "disc_graph_launch")

_lib = None


def lib_path() -> str:
    return os.path.join(HERE, "libdisc.so")


def load_library():
    """Load libdisc.so.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2103_05288_amd.build` "
                          "(or __graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(path)
    vp, i32p, i64p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    lib.disc_create.argtypes = [C.POINTER(vp), C.c_int]
    lib.disc_destroy.argtypes = [vp]
    lib.disc_destroy.restype = None
    lib.disc_last_error.argtypes = [vp]
    lib.disc_last_error.restype = C.c_char_p
    lib.disc_register_pattern.argtypes = [vp, C.POINTER(disc_op), C.c_int, C.POINTER(disc_constraint), C.c_int, i32p]
    lib.disc_register_pattern_static.argtypes = [vp, C.POINTER(disc_op), C.c_int, C.POINTER(disc_constraint), C.c_int,
                                                 i64p, C.c_int, i32p]
    lib.disc_pattern_info.argtypes = [vp, C.c_int32, C.POINTER(disc_pattern_info_t)]
    lib.disc_pattern_source.argtypes = [vp, C.c_int32]
    lib.disc_pattern_source.restype = C.c_char_p
    lib.disc_workspace_bytes.argtypes = [vp, C.c_int32, i64p, C.c_int, C.POINTER(C.c_size_t)]
    lib.disc_plan.argtypes = [vp, C.c_int32, i64p, C.c_int, C.POINTER(vp), C.POINTER(vp), C.c_int, C.POINTER(disc_plan_t)]
    lib.disc_launch.argtypes = [vp, C.c_int32, i64p, C.c_int, C.POINTER(vp), C.c_int, C.POINTER(vp), C.c_int,
                                vp, C.c_size_t, vp]
    lib.disc_register_graph.argtypes = [vp, C.POINTER(disc_op), C.c_int, C.POINTER(disc_constraint), C.c_int, i32p]
    lib.disc_graph_info.argtypes = [vp, C.c_int32, C.POINTER(disc_graph_info_t)]
    lib.disc_graph_workspace_bytes.argtypes = [vp, C.c_int32, i64p, C.c_int, C.POINTER(C.c_size_t)]
    lib.disc_graph_launch.argtypes = [vp, C.c_int32, i64p, C.c_int, C.POINTER(vp), C.c_int, C.POINTER(vp), C.c_int,
                                      vp, C.c_size_t, vp]
    lib.disc_force_variant.argtypes = [vp, C.c_int]
    lib.disc_static_scratch_init.argtypes = [vp]
    lib.disc_launch_static_scratch.argtypes = [vp, C.c_int32, i64p, C.c_int, C.POINTER(vp), C.c_int, C.POINTER(vp), C.c_int, vp]
    lib.disc_test_option.argtypes = [vp, C.c_int, C.c_int]
    lib.disc_get_stats.argtypes = [vp, C.POINTER(disc_stats_t)]
    lib.disc_util_copy.argtypes = [vp, vp, vp, C.c_size_t, vp]
    lib.disc_util_copy_nt.argtypes = [vp, vp, vp, C.c_size_t, vp]
    lib.disc_util_empty_launch.argtypes = [vp, vp]
    lib.disc_util_mix.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, vp, C.c_size_t, vp]
    _lib = lib
    return lib


def marshal_pattern(pattern):
    """workloads.Pattern-like object (ops with string opcodes) -> C arrays."""
    ops = (disc_op * len(pattern.ops))()
    for i, o in enumerate(pattern.ops):
        c = ops[i]
        c.opcode = OPCODE_IDS[o.opcode]
        c.dtype = DTYPE_IDS[o.dtype]
        for k in range(3):
            c.in_[k] = o.ins[k] if k < len(o.ins) else -1
        c.rank = len(o.dims)
        for k in range(MAX_RANK):
            c.dim[k] = o.dims[k] if k < len(o.dims) else 0
            c.axis_map[k] = o.axis_map[k] if k < len(o.axis_map) else 0
        c.fconst = o.fconst
    cs = (disc_constraint * max(1, len(pattern.constraints)))()
    for i, (kind, av, aa, bv, ba) in enumerate(pattern.constraints):
        cs[i].kind, cs[i].a_value, cs[i].a_axis, cs[i].b_value, cs[i].b_axis = kind, av, aa, bv, ba
    return ops, len(pattern.ops), cs, len(pattern.constraints)


class BoundCall:
    """One disc_launch with its arguments marshalled once: calling it is a single C call.
    Keeps the tensors alive; the pointers must stay valid for as long as it is used."""

    def __init__(self, ctx: "Context", pid: int, dims, inputs, outputs, workspace, workspace_bytes, stream):
        self._keep = (list(inputs), list(outputs), workspace)
        self._fn = ctx.lib.disc_launch
        self._ctx = ctx
        self._args = (ctx.h, pid, (C.c_int64 * max(1, len(dims)))(*[int(d) for d in dims]), len(dims),
                      (C.c_void_p * max(1, len(inputs)))(*[_ptr(t) for t in inputs]), len(inputs),
                      (C.c_void_p * max(1, len(outputs)))(*[_ptr(t) for t in outputs]), len(outputs),
                      C.c_void_p(_ptr(workspace)) if workspace is not None else C.c_void_p(),
                      C.c_size_t(workspace_bytes), C.c_void_p(stream))

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != 0:
            self._ctx._check(rc)


class PatternHandle:
    def __init__(self, ctx: "Context", pid: int):
        self.ctx, self.id = ctx, pid
        self.info = ctx.pattern_info(pid)

    def bind(self, dims, inputs, outputs, workspace=None, stream: Optional[int] = None) -> BoundCall:
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        wsb = workspace.numel() * workspace.element_size() if workspace is not None else 0
        return BoundCall(self.ctx, self.id, dims, inputs, outputs, workspace, wsb, stream)

    def launch(self, dims, inputs, outputs, **kw):
        return self.ctx.launch(self.id, dims, inputs, outputs, **kw)

    def plan(self, dims, force_variant: int = -1, inputs=None, outputs=None):
        return self.ctx.plan(self.id, dims, force_variant, inputs, outputs)

    @property
    def source(self) -> str:
        return self.ctx.pattern_source(self.id)


class GraphHandle:
    """An op graph cut into fusion patterns (disc_register_graph)."""

    def __init__(self, ctx: "Context", gid: int, n_ops: int):
        self.ctx, self.id, self.n_ops = ctx, gid, n_ops

    @property
    def info(self) -> dict:
        g = disc_graph_info_t()
        self.ctx._check(self.ctx.lib.disc_graph_info(self.ctx.h, self.id, C.byref(g)))
        d = {k: getattr(g, k) for k in ("n_dims", "n_inputs", "n_outputs", "n_patterns", "n_intermediates", "n_buffers")}
        d["pattern_id"] = list(g.pattern_id)[: g.n_patterns]
        d["pattern_ops"] = list(g.pattern_ops)[: g.n_patterns]
        d["group_of_op"] = list(g.group_of_op)[: self.n_ops]
        return d

    def workspace_bytes(self, dims) -> int:
        arr, n = self.ctx._dims(dims)
        out = C.c_size_t(0)
        self.ctx._check(self.ctx.lib.disc_graph_workspace_bytes(self.ctx.h, self.id, arr, n, C.byref(out)))
        return int(out.value)

    def launch(self, dims, inputs: Sequence, outputs: Sequence, workspace=None, workspace_bytes: int = 0,
               stream: Optional[int] = None):
        arr, n = self.ctx._dims(dims)
        ins = (C.c_void_p * max(1, len(inputs)))(*[_ptr(t) for t in inputs])
        outs = (C.c_void_p * max(1, len(outputs)))(*[_ptr(t) for t in outputs])
        ws = C.c_void_p(_ptr(workspace)) if workspace is not None else C.c_void_p()
        if workspace is not None and not workspace_bytes and hasattr(workspace, "numel"):
            workspace_bytes = workspace.numel() * workspace.element_size()
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self.ctx._check(self.ctx.lib.disc_graph_launch(self.ctx.h, self.id, arr, n, ins, len(inputs), outs, len(outputs),
                                                       ws, C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def _ptr(t) -> int:
    return int(t.data_ptr()) if hasattr(t, "data_ptr") else int(t)


class Context:
    """One disc_ctx.  device=-1 gives a host-only context (checker, planner, device compile)."""

    def __init__(self, device: int = 0):
        self.lib = load_library()
        self.h = C.c_void_p()
        rc = self.lib.disc_create(C.byref(self.h), int(device))
        if rc != 0:
            raise DiscError(rc, "disc_create failed (no such HIP device?)")
        self.device = device

    def close(self):
        if self.h:
            self.lib.disc_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != 0:
            raise DiscError(rc, self.lib.disc_last_error(self.h).decode(errors="replace"))

    def register(self, pattern) -> PatternHandle:
        ops, n_ops, cs, n_cs = marshal_pattern(pattern)
        pid = C.c_int32(-1)
        self._check(self.lib.disc_register_pattern(self.h, ops, n_ops, cs, n_cs, C.byref(pid)))
        return PatternHandle(self, pid.value)

    def register_graph(self, pattern) -> GraphHandle:
        """An op list that need not be one fusible pattern: cut into patterns, buffers planned."""
        ops, n_ops, cs, n_cs = marshal_pattern(pattern)
        gid = C.c_int32(-1)
        self._check(self.lib.disc_register_graph(self.h, ops, n_ops, cs, n_cs, C.byref(gid)))
        return GraphHandle(self, gid.value, n_ops)

    def register_static(self, pattern, dims) -> PatternHandle:
        """The pattern compiled for this one shape only (single-shape module)."""
        ops, n_ops, cs, n_cs = marshal_pattern(pattern)
        arr, n = self._dims(dims)
        pid = C.c_int32(-1)
        self._check(self.lib.disc_register_pattern_static(self.h, ops, n_ops, cs, n_cs, arr, n, C.byref(pid)))
        return PatternHandle(self, pid.value)

    def pattern_info(self, pid: int) -> dict:
        info = disc_pattern_info_t()
        self._check(self.lib.disc_pattern_info(self.h, pid, C.byref(info)))
        d = {k: getattr(info, k) for k, _ in info._fields_ if k != "dim_class"}
        d["dim_class"] = list(info.dim_class)[: info.n_dims]
        d["template"] = TEMPLATES[info.template_kind]
        return d

    def pattern_source(self, pid: int) -> str:
        s = self.lib.disc_pattern_source(self.h, pid)
        return s.decode() if s else ""

    @staticmethod
    def _dims(dims):
        arr = (C.c_int64 * max(1, len(dims)))(*[int(d) for d in dims])
        return arr, len(dims)

    def workspace_bytes(self, pid: int, dims) -> int:
        arr, n = self._dims(dims)
        out = C.c_size_t(0)
        self._check(self.lib.disc_workspace_bytes(self.h, pid, arr, n, C.byref(out)))
        return out.value

    def plan(self, pid: int, dims, force_variant: int = -1, inputs=None, outputs=None) -> dict:
        """The launch plan for these dims; with inputs / outputs (tensors or device addresses) the
        plan is the one a launch with exactly these operands takes."""
        arr, n = self._dims(dims)
        p = disc_plan_t()
        ins = (C.c_void_p * max(1, len(inputs)))(*[_ptr(t) for t in inputs]) if inputs is not None else None
        outs = (C.c_void_p * max(1, len(outputs)))(*[_ptr(t) for t in outputs]) if outputs is not None else None
        self._check(self.lib.disc_plan(self.h, pid, arr, n, ins, outs, int(force_variant), C.byref(p)))
        d = {k: getattr(p, k) for k, _ in p._fields_ if k not in ("grid", "block", "lds_bytes", "kernel")}
        d["kernels"] = [bytes(p.kernel[i]).split(b"\0")[0].decode() for i in range(p.n_launches)]
        d["grid"] = [list(g) for g in p.grid][: p.n_launches]
        d["block"] = [list(b) for b in p.block][: p.n_launches]
        d["lds_bytes"] = list(p.lds_bytes)[: p.n_launches]
        d["variant_name"] = VARIANTS[p.variant] if 0 <= p.variant < len(VARIANTS) else None
        return d

    def force_variant(self, variant: int):
        self._check(self.lib.disc_force_variant(self.h, int(variant)))

    def test_option(self, name: str, value: int):
        """Tests only: override one host rule (see disc_test_option in disc.h)."""
        self._check(self.lib.disc_test_option(self.h, TEST_OPTIONS[name], int(value)))

    def launch(self, pid: int, dims, inputs: Sequence, outputs: Sequence, workspace=None,
               workspace_bytes: int = 0, stream: Optional[int] = None):
        """inputs / outputs: torch tensors (their data_ptr is passed) or raw device addresses."""
        arr, n = self._dims(dims)
        ins = (C.c_void_p * max(1, len(inputs)))(*[_ptr(t) for t in inputs])
        outs = (C.c_void_p * max(1, len(outputs)))(*[_ptr(t) for t in outputs])
        ws = C.c_void_p(_ptr(workspace)) if workspace is not None else C.c_void_p()
        if workspace is not None and not workspace_bytes and hasattr(workspace, "numel"):
            workspace_bytes = workspace.numel() * workspace.element_size()
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self._check(self.lib.disc_launch(self.h, pid, arr, n, ins, len(inputs), outs, len(outputs), ws,
                                         C.c_size_t(workspace_bytes), C.c_void_p(stream)))

    def launch_static_scratch(self, pid: int, dims, inputs: Sequence, outputs: Sequence, stream: Optional[int] = None):
        """disc_launch_static_scratch: no workspace argument, nothing allocated (the library's own
        fixed device array serves as scratch memory)."""
        arr, n = self._dims(dims)
        ins = (C.c_void_p * max(1, len(inputs)))(*[_ptr(t) for t in inputs])
        outs = (C.c_void_p * max(1, len(outputs)))(*[_ptr(t) for t in outputs])
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self._check(self.lib.disc_launch_static_scratch(self.h, pid, arr, n, ins, len(inputs), outs, len(outputs),
                                                        C.c_void_p(stream)))

    def stats(self) -> dict:
        s = disc_stats_t()
        self._check(self.lib.disc_get_stats(self.h, C.byref(s)))
        d = {k: getattr(s, k) for k, _ in s._fields_ if k != "variant_count"}
        d["variant_count"] = {VARIANTS[i]: s.variant_count[i] for i in range(len(VARIANTS)) if s.variant_count[i]}
        return d

    def util_copy(self, dst, src, nbytes: int, stream: Optional[int] = None, non_temporal: bool = False):
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        fn = self.lib.disc_util_copy_nt if non_temporal else self.lib.disc_util_copy
        self._check(fn(self.h, C.c_void_p(_ptr(dst)), C.c_void_p(_ptr(src)),
                                            C.c_size_t(nbytes), C.c_void_p(stream)))

    def util_mix(self, kind: int, non_temporal: bool, slots_in_flight: int, blocks_per_cu: int, out, a, b_or_mask, n_elems: int,
                 stream: Optional[int] = None):
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self._check(self.lib.disc_util_mix(self.h, int(kind), int(bool(non_temporal)), int(slots_in_flight), int(blocks_per_cu),
                                           C.c_void_p(_ptr(out)), C.c_void_p(_ptr(a)), C.c_void_p(_ptr(b_or_mask)),
                                           C.c_size_t(n_elems), C.c_void_p(stream)))

    def util_empty_launch(self, stream: Optional[int] = None):
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self._check(self.lib.disc_util_empty_launch(self.h, C.c_void_p(stream)))
