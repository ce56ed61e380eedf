"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle import run as oracle_run
from workloads.configs import CONFIGS
from tests.util import assert_close, run_gpu, to_oracle_input

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2103_05288_amd import Context
    c = Context(0)
    yield c
    c.close()


def check(ctx, cfg_name, dims, seed, handle=None, force=None):
    cfg = CONFIGS[cfg_name]
    pat = cfg.pattern()
    h = handle or ctx.register(pat)
    ins = cfg.inputs(dims, seed)
    if force is not None:
        ctx.force_variant(force)
    try:
        got = run_gpu(h, pat, dims, ins)
    finally:
        ctx.force_variant(-1)
    want = oracle_run(pat, dims, [to_oracle_input(t) for t in ins])[0]
    for k, (g, w) in enumerate(zip(got, want)):
        assert_close(g, w, f"{cfg_name} dims={dims} out{k} force={force}")
    return h


SMALL = {
    "C0": [[1, 768], [7, 768], [300, 768], [33, 5], [5, 1], [129, 771]],
    "C1": [[2, 3, 16], [2, 3, 17], [1, 2, 64], [2, 1, 131], [1, 1, 512], [1, 1, 1]],
    "C2": [[5, 768], [64, 1024], [3, 4096], [17, 100], [9, 3], [2, 9000]],
    "C3": [[1, 1024], [100, 1024], [5000, 1024], [37, 100], [300, 7], [64, 3000], [2, 1]],
    "C4": [[1, 64], [37, 64], [100, 777], [3, 8192], [1000, 65], [5, 9], [2, 20000]],
}


@pytest.mark.parametrize("cfg_name", ["C0", "C1", "C2", "C3", "C4"])
def test_small_shapes_one_compile(ctx, cfg_name):
    h = None
    for i, dims in enumerate(SMALL[cfg_name]):
        print(f"[parity] {cfg_name} dims={dims}", flush=True)
        h = check(ctx, cfg_name, dims, seed=100 + i, handle=h)
    assert h.ctx.pattern_info(h.id)["compile_events"] == 1
