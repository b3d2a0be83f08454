"""The paper's two single-host experiments in shape, on the GPU, against the CPU oracle.

Online instantiation and recovery under load (Sec. 3.1 / Fig. 2, Sec. 4.2 / Fig. 5): worlds are created while
other worlds have operations in flight, a worker fails with a window in flight, a new worker takes its place
through new worlds -- every status and every byte of every world is compared.  The multi-sender experiment
(Sec. 4.3 / Fig. 7): 1-3 senders to one receiver with fp32 tensors of 1 000 ... 1 000 000 elements, through one
world per sender and through one shared world -- every received tensor is compared.
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

    binding.lib()
    return trace_runner


def _both(trace, gpu, host_pools, **kw):
    from oracle.run_trace import run_trace as run_oracle

    mat = lambda spec: materialize(spec, host_pools)
    grun = gpu.run_trace(trace, host_pools, mat, **kw)
    orun = run_oracle(trace, mat)
    return orun, grun


def test_online_instantiation_and_recovery_under_load(gpu, host_pools):
    from paper_2407_08980_amd import binding as mw

    t = workloads.online_recovery()  # 4 MB fp32 tensors, as in Sec. 4.2
    seen = {}

    def start_watchdog():  # the watchdog thread runs throughout, as it does in the paper's runs (Sec. 3.3)
        for k in range(t.n_workers):
            mw.mw_heartbeat(k)
        mw.mw_watchdog_start(60.0, 0.01)

    def stop_watchdog():
        seen["epochs"] = [mw.mw_heartbeat_epoch(k) for k in range(t.n_workers)]
        seen["failed"] = [mw.mw_worker_state(k) for k in range(t.n_workers)]
        mw.mw_watchdog_stop()

    orun, grun = _both(t, gpu, host_pools, on_init=start_watchdog, on_exit=stop_watchdog)
    rep = compare_runs(t, orun, grun)
    n_checks = sum(1 for op in t.ops if op.kind == "check")
    assert rep["exact"] == n_checks and rep["toleranced"] == 0
    assert grun.world_state == orun.world_state == {1: "alive", 3: "alive", 2: "broken", 4: "broken", 6: "alive", 7: "alive"}
    counts = {s: list(grun.status.values()).count(s) for s in ("done", "broken", "pending")}
    assert counts == {"done": 2 * 30 * 4, "broken": 2 + 2 * 2 * 4, "pending": 0}, counts
    assert grun.payload_bytes_done == orun.payload_bytes_done == 30 * 4 * 4_000_000
    assert seen["epochs"] == [1] * 5 and seen["failed"] == [mw.MW_ALIVE] * 5  # an explicit abort, no timeout


def test_world_creation_happens_with_operations_in_flight(gpu):
    """The scenario above relies on it: a world created right after a flush of large transfers comes into being
    while they are still running, and does not wait for them."""
    import time

    import torch

    from paper_2407_08980_amd import binding as mw

    mw.mw_init(0, 8)
    try:
        mw.mw_world_create(1, [0, 1])
        n = 1 << 30
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        hs = [mw.mw_send(1, 0, 1, src.data_ptr(), n // 4, mw.MW_F32, mw.STREAM_NONE),
              mw.mw_recv(1, 0, 1, dst.data_ptr(), n // 4, mw.MW_F32, mw.STREAM_NONE)]
        mw.mw_flush()
        t0 = time.perf_counter()
        mw.mw_world_create(2, [0, 2])
        took = time.perf_counter() - t0
        assert mw.mw_poll(hs[1]) == mw.MW_PENDING, "the 1 GiB transfer should still be running"
        assert took < 5e-3, f"mw_world_create took {took * 1e3:.2f} ms with a transfer in flight"
        ps = mw.PollSet(hs)
        t0 = time.time()
        while ps.poll():
            assert time.time() - t0 < 30
        assert bool((dst == 7).all())
    finally:
        mw.mw_shutdown()


@pytest.mark.parametrize("count", [1_000, 10_000, 100_000, 1_000_000])
@pytest.mark.parametrize("senders", [1, 2, 3])
def test_multi_sender_sweep_every_tensor(gpu, host_pools, senders, count):
    for multi_world in (True, False):
        t = workloads.multi_sender(senders, count, multi_world)
        orun, grun = _both(t, gpu, host_pools)
        rep = compare_runs(t, orun, grun)
        assert rep["exact"] == 2 * 8 * senders and rep["toleranced"] == 0
        assert set(grun.status.values()) == {"done"}
        assert grun.payload_bytes_done == orun.payload_bytes_done == 2 * 8 * senders * count * 4
