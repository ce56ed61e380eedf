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
