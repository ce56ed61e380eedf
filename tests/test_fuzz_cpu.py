"""The C ABI never throws, aborts or hangs on a malformed pattern: random op lists and single-field
mutations of the benchmark patterns through disc_register_pattern and disc_register_graph on a
host-only context.  Every call must come back with a status; a status of 0 must leave a pattern
whose plan can be asked for."""
import ctypes as C

import numpy as np
import pytest

from workloads.configs import CONFIGS


@pytest.fixture(scope="module")
def hctx():
    from paper_2103_05288_amd import Context
    c = Context(device=-1)
    yield c
    c.close()


def _random_ops(rng, n):
    from paper_2103_05288_amd.binding import disc_op
    ops = (disc_op * n)()
    for i in range(n):
        o = ops[i]
        o.opcode = int(rng.integers(-2, 40))
        o.dtype = int(rng.integers(-1, 8))
        for k in range(3):
            o.in_[k] = int(rng.integers(-3, n + 3))
        o.rank = int(rng.integers(-1, 7))
        for k in range(4):
            o.dim[k] = int(rng.integers(-6, 20))
            o.axis_map[k] = int(rng.integers(-4, 20))
        o.fconst = float(rng.normal())
    return ops


def test_random_garbage_is_refused_with_a_status(hctx):
    from paper_2103_05288_amd.binding import disc_constraint
    rng = np.random.default_rng(2024)
    lib, h = hctx.lib, hctx.h
    ok = 0
    for case in range(3000):
        n = int(rng.integers(1, 12))
        ops = _random_ops(rng, n)
        ncs = int(rng.integers(0, 3))
        cs = (disc_constraint * max(1, ncs))()
        for j in range(ncs):
            cs[j].kind = int(rng.integers(-1, 3))
            cs[j].a_value, cs[j].b_value = int(rng.integers(-2, n + 2)), int(rng.integers(-2, n + 2))
            cs[j].a_axis, cs[j].b_axis = int(rng.integers(-2, 6)), int(rng.integers(-2, 6))
        pid = C.c_int32(-5)
        fn = lib.disc_register_pattern if case % 2 == 0 else lib.disc_register_graph
        rc = fn(h, ops, n, cs, ncs, C.byref(pid))
        assert -9 <= rc <= 0
        if rc == 0:
            ok += 1
        else:
            assert pid.value == -1 and len(lib.disc_last_error(h)) > 0
    assert ok < 300          # random lists are almost never patterns


@pytest.mark.parametrize("name", ["C3", "C1"])
def test_single_field_mutations(hctx, name):
    from paper_2103_05288_amd.binding import marshal_pattern
    pat = CONFIGS[name].pattern()
    rng = np.random.default_rng(7 + len(name))
    lib, h = hctx.lib, hctx.h
    statuses = {}
    for case in range(24):
        ops, n, cs, ncs = marshal_pattern(pat)
        i = int(rng.integers(0, n))
        field = ["opcode", "dtype", "in0", "in1", "rank", "dim0", "dim1", "axis0"][int(rng.integers(0, 8))]
        o = ops[i]
        if field == "opcode":
            o.opcode = int(rng.integers(0, 38))
        elif field == "dtype":
            o.dtype = int(rng.integers(0, 6))
        elif field == "in0":
            o.in_[0] = int(rng.integers(-1, n))
        elif field == "in1":
            o.in_[1] = int(rng.integers(-1, n))
        elif field == "rank":
            o.rank = int(rng.integers(0, 5))
        elif field == "dim0":
            o.dim[0] = int(rng.integers(-4, 4))
        elif field == "dim1":
            o.dim[1] = int(rng.integers(-4, 4))
        else:
            o.axis_map[0] = int(rng.integers(-2, 4))
        pid = C.c_int32(-5)
        fn = lib.disc_register_pattern if case % 3 else lib.disc_register_graph
        rc = fn(h, ops, n, cs, ncs, C.byref(pid))
        assert -9 <= rc <= 0
        statuses[rc] = statuses.get(rc, 0) + 1
        if rc == 0 and case % 3:
            # whatever was accepted can be planned (or refuses the shape with a status)
            nd = hctx.pattern_info(pid.value)["n_dims"]
            try:
                hctx.plan(pid.value, [5] * nd)
            except Exception as e:                       # DiscError only
                assert type(e).__name__ == "DiscError"
    assert len(statuses) >= 2


def test_plan_with_extreme_dims(hctx):
    """The launch path without the enqueue, over sizes from 0 to 2^40 and negative ones: a plan or
    a status, never a crash; a plan's grid and block stay within the device limits."""
    from paper_2103_05288_amd import DiscError
    from tests.test_slice import qkv_split, softmax_of_window
    from tests.test_pad import padded_softmax, pad_scale
    from tests.test_transpose import heads_softmax, pure_transpose
    pats = [CONFIGS[n].pattern() for n in ("C0", "C1", "C3")] + [qkv_split(), softmax_of_window(), padded_softmax(), pad_scale(),
                                                               heads_softmax(), pure_transpose("bf16", (0, 2, 1))]
    values = [0, 1, 2, 3, 7, 8, 64, 1000, 4099, 1 << 16, 1 << 20, (1 << 31) - 1, 1 << 31, 1 << 33, 1 << 40, -1]
    rng = np.random.default_rng(99)
    planned = refused = 0
    for pat in pats:
        h = hctx.register(pat)
        nd = h.info["n_dims"]
        for _ in range(300):
            dims = [values[int(rng.integers(0, len(values)))] for _ in range(nd)]
            try:
                p = h.plan(dims)
            except DiscError as e:
                assert e.status in ("SHAPE", "EMPTY_REDUCE", "CONSTRAINT", "INVALID_ARG"), (pat.name, dims, e)
                refused += 1
                continue
            planned += 1
            for l in range(p["n_launches"]):
                gx, gy, gz = p["grid"][l]
                assert 1 <= gx < (1 << 31) and 1 <= gy <= 65535 and 1 <= gz <= 65535, (pat.name, dims, p["grid"])
                assert 64 <= p["block"][l][0] <= 1024 and p["lds_bytes"][l] <= 160 * 1024
    assert planned > 200 and refused > 200


def test_graph_workspace_with_extreme_dims(hctx):
    from paper_2103_05288_amd import DiscError
    from tests.test_graph import chain_graph, layernorm_backward_graph
    values = [0, 1, 7, 1000, 1 << 20, (1 << 31) - 1, 1 << 33, 1 << 40, 1 << 62, -1]
    rng = np.random.default_rng(5)
    for make in (lambda: chain_graph(4), layernorm_backward_graph):
        g = hctx.register_graph(make())
        got = refused = 0
        for _ in range(200):
            dims = [values[int(rng.integers(0, len(values)))] for _ in range(2)]
            try:
                ws = g.workspace_bytes(dims)
                assert 0 <= ws < (1 << 63)
                got += 1
            except DiscError as e:
                assert e.status in ("SHAPE", "EMPTY_REDUCE", "INVALID_ARG"), (dims, e)
                refused += 1
        assert got > 20 and refused > 20
