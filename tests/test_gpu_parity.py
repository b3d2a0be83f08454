"""GPU library vs CPU oracle, element by element, through the C ABI.

Sizes here are what the oracle finishes in seconds while still spanning several
chunks and a ragged tail.  Copies, broadcasts and statuses are compared bit-exactly;
all-reduce results within |y - s| <= tol * sum_r |x_r| (tol 1e-6 fp32, 1e-2 bf16)
against the float64 sum, and bit-exactly against the ascending-order fp32 sum.
"""

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import workloads
from workloads import materialize

from helpers import compare_runs


@pytest.fixture(scope="module")
def gpu():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2407_08980_amd import binding, trace_runner

    binding.lib()  # fail loudly if the HIP library is not built
    return trace_runner


def _both(trace, gpu, host_pools):
    from oracle.run_trace import run_trace as run_oracle

    mat = lambda spec: materialize(spec, host_pools)
    grun = gpu.run_trace(trace, host_pools, mat)
    orun = run_oracle(trace, mat)
    return orun, grun


def test_config1_full(gpu, host_pools):
    t = workloads.config1()
    orun, grun = _both(t, gpu, host_pools)
    rep = compare_runs(t, orun, grun)
    assert rep["exact"] == 200 + 4 and rep["toleranced"] == 4
    assert grun.payload_bytes_done == orun.payload_bytes_done == 204 * 32768


@pytest.mark.parametrize("shape", [(3, 331, 1031), (1, 7, 13), (2, 2048, 129)])
def test_config2_ragged_shapes(gpu, host_pools, shape):
    t = workloads.config2(shape=shape, steps=6)
    orun, grun = _both(t, gpu, host_pools)
    rep = compare_runs(t, orun, grun)
    assert rep["exact"] == 6 * 8


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("lds", [0, 1])
def test_config3_full_shapes_few_iterations(gpu, host_pools, dtype, lds):
    from paper_2407_08980_amd import binding

    binding.mw_config_set("reduce_lds", lds)
    try:
        t = workloads.config3(iters=6, dtype=dtype)
        orun, grun = _both(t, gpu, host_pools)
    finally:
        binding.mw_config_set("reduce_lds", 0)
    rep = compare_runs(t, orun, grun)
    assert rep["toleranced"] == 6 * 4 * 4 * 2
    assert rep["worst_allreduce_ratio"] <= (3 * 2.0 ** -24 if dtype == "f32" else 2.0 ** -8)
    # bit-exact against the ascending-rank fp32 sum, and identical on all ranks
    import oracle

    checks = [i for i, op in enumerate(t.ops) if op.kind == "check"]
    first_iter = checks[: 4 * 4 * 2]
    # buffers were created world-major, rank, pool set, shape: rebuild inputs per (world, shape)
    n_ranks, pool_k, n_shapes = 4, 4, 2
    for w in range(4):
        for j in range(n_shapes):
            ids = [((w * n_ranks + r) * pool_k + 0) * n_shapes + j for r in range(n_ranks)]
            ins = [materialize(t.bufs[b], host_pools) for b in ids]
            count = t.bufs[ids[0]].nbytes // (4 if dtype == "f32" else 2)
            want = oracle.allreduce_sum_ordered(ins, count, dtype)
            for b in ids:
                ci = next(i for i in first_iter if t.ops[i].buf == b)
                assert np.array_equal(grun.snapshots[ci], want), (w, j, b)


def test_config3_ragged_shapes(gpu, host_pools):
    for dtype in ("f32", "bf16"):
        t = workloads.config3(shapes=((3, 1031), (7, 4099)), iters=5, dtype=dtype)
        orun, grun = _both(t, gpu, host_pools)
        compare_runs(t, orun, grun)


def test_config4_small_fault_isolation(gpu, host_pools):
    t = workloads.config4(shape=(2, 129, 517), steps=30, abort_step=10)
    orun, grun = _both(t, gpu, host_pools)
    rep = compare_runs(t, orun, grun)
    assert rep["exact"] == 30 * 16
    assert grun.world_state == orun.world_state
    assert [w for w, s in grun.world_state.items() if s == "broken"] == [7]
    # world 7's destination is untouched after the abort: its last checked content is the poison
    last7 = [i for i, op in enumerate(t.ops) if op.kind == "check"][-16 + 7]
    assert np.all(grun.snapshots[last7] == 0xA5)


def test_config5_small_mixed(gpu, host_pools):
    t = workloads.config5(n_ops=800, max_bytes=1 << 20, check_all=True)
    orun, grun = _both(t, gpu, host_pools)
    rep = compare_runs(t, orun, grun)
    assert rep["exact"] > 800 and rep["toleranced"] > 50
    assert grun.world_state == orun.world_state
    assert set(grun.status.values()) == {"done", "broken"}
