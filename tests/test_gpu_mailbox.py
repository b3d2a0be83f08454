"""The resident mailbox kernel ("mailbox" = 1) on the GPU: the same traces as everywhere else, every status and byte
against the CPU oracle, now served from the descriptor queue instead of by launches; and the kernel's life cycle --
it closes by itself when idle, when a large flush comes and at shutdown, and operations that arrive afterwards are
served by the next one.  Every wait in that kernel is bounded; nothing here can outlive its limits.
"""

import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
import workloads
from workloads import materialize

from helpers import compare_runs


@pytest.fixture(scope="module")
def torch():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    torch.cuda.set_device(0)
    return torch


@pytest.fixture
def mailbox(torch):
    from paper_2407_08980_amd import binding

    binding.lib()
    before = binding.mw_config_get("mailbox")
    binding.mw_config_set("mailbox", 1)
    yield binding
    binding.mw_config_set("mailbox", before)


def _both(trace, host_pools):
    from oracle.run_trace import run_trace as run_oracle
    from paper_2407_08980_amd import binding, trace_runner

    seen = {}
    mat = lambda spec: materialize(spec, host_pools)
    grun = trace_runner.run_trace(trace, host_pools, mat, on_exit=lambda: seen.update(state=binding.mw_debug_mailbox()),
                                  settle=True)
    orun = run_oracle(trace, mat)
    return orun, grun, seen["state"]


def test_config1_through_the_mailbox(mailbox, host_pools):
    t = workloads.config1()
    orun, grun, (epoch, _, tail) = _both(t, host_pools)
    rep = compare_runs(t, orun, grun)
    assert rep["exact"] == 200 + 4 and rep["toleranced"] == 4
    assert epoch >= 1 and tail == 200 + 2 + 2  # every operation went through the queue: one descriptor each


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_config3_through_the_mailbox(mailbox, host_pools, dtype):
    t = workloads.config3(iters=12, dtype=dtype)
    orun, grun, (epoch, _, tail) = _both(t, host_pools)
    rep = compare_runs(t, orun, grun)
    assert rep["toleranced"] == 12 * 32 and rep["worst_allreduce_ratio"] <= (3 * 2.0 ** -24 if dtype == "f32" else 2.0 ** -8)
    assert tail == 12 * 8


def test_config3_full_length_through_the_mailbox(mailbox, host_pools):
    """The tensor-parallel workload at its full length: 500 iterations of 8 all-reduces, every one a descriptor in the
    queue (4000, i.e. more than one resident kernel serves), data checked on 12 iterations."""
    checked = [0, 1, 2, 3, 4, 5, 250, 251, 496, 497, 498, 499]
    t = workloads.config3(iters=500, check_iters=checked)
    orun, grun, (epoch, _, tail) = _both(t, host_pools)
    rep = compare_runs(t, orun, grun)
    assert rep["toleranced"] == len(checked) * 32 and rep["worst_allreduce_ratio"] <= 3 * 2.0 ** -24
    assert all(v == "done" for v in grun.status.values()) and len(grun.status) == 500 * 32
    assert epoch >= 2 and 3000 <= tail <= 500 * 8  # (a few flushes are launched while one kernel hands over to the next)


def test_mixed_operations_aborts_and_sizes_through_the_mailbox(mailbox, host_pools):
    """All eight operations with worker aborts (windows small enough for the queue), then the mixed scale-out recipe
    at small sizes, then the fan-in with a fault: small flushes go through the queue, larger ones are launched while
    the resident kernel is asked to make room -- both in one run."""
    for t in (workloads.collectives_mix(), workloads.config5(n_ops=600, max_bytes=1 << 21, check_all=True),
              workloads.config4(shape=(2, 8, 20), steps=30, abort_step=10)):
        orun, grun, (epoch, _, tail) = _both(t, host_pools)
        rep = compare_runs(t, orun, grun)
        assert rep["exact"] + rep["toleranced"] > 0 and tail > 0
        assert grun.world_state == orun.world_state


@pytest.mark.parametrize("count", [1_000, 100_000])
def test_multi_sender_through_the_mailbox(mailbox, host_pools, count):
    for multi_world in (True, False):
        t = workloads.multi_sender(3, count, multi_world)
        orun, grun, _ = _both(t, host_pools)
        assert compare_runs(t, orun, grun)["exact"] == 2 * 8 * 3


def _wait(mw, hs, timeout=30.0):
    mw.mw_flush()
    ps = mw.PollSet(hs)
    t0 = time.time()
    while ps.poll():
        assert time.time() - t0 < timeout, "operations did not complete"
    return list(ps.states)


def test_the_resident_kernel_ends_by_itself_and_the_next_one_takes_over(mailbox, torch):
    mw = mailbox
    mw.mw_init(0, 4)
    try:
        mw.mw_world_create(0, [0, 1])
        n = 8192
        src = [np.random.default_rng(k).integers(0, 256, size=4 * n, dtype=np.uint8) for k in range(3)]
        sdev = [torch.from_numpy(s).cuda() for s in src]
        ddev = [torch.full((4 * n,), 0xA5, dtype=torch.uint8, device="cuda") for _ in range(3)]
        big_s = torch.full((1 << 30,), 3, dtype=torch.uint8, device="cuda")
        big_d = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()

        def message(k):
            hs = [mw.mw_send(0, 0, 1, sdev[k].data_ptr(), n, mw.MW_F32, mw.STREAM_NONE),
                  mw.mw_recv(0, 0, 1, ddev[k].data_ptr(), n, mw.MW_F32, mw.STREAM_NONE)]
            assert _wait(mw, hs) == [mw.MW_DONE] * 2
            assert np.array_equal(ddev[k].cpu().numpy(), oracle.copy_result(src[k]))  # read the moment it is DONE

        assert mw.mw_debug_mailbox() == (0, 0, 0)
        message(0)
        assert mw.mw_debug_mailbox()[0] == 1 and mw.mw_debug_mailbox()[2] == 1
        # idle: the kernel closes by itself after 300 us without work (the host asks for nothing)
        t0 = time.time()
        while mw.mw_debug_mailbox()[1]:
            assert time.time() - t0 < 5.0, "the resident kernel did not end when idle"
        assert time.time() - t0 < 0.5
        message(1)  # served by the next kernel
        assert mw.mw_debug_mailbox()[0] == 2
        # a large flush asks the open kernel to make room: it closes although it has been idle for less than 300 us
        hs = [mw.mw_send(0, 0, 1, big_s.data_ptr(), 1 << 28, mw.MW_F32, mw.STREAM_NONE),
              mw.mw_recv(0, 0, 1, big_d.data_ptr(), 1 << 28, mw.MW_F32, mw.STREAM_NONE)]
        mw.mw_flush()
        t0 = time.time()
        while mw.mw_debug_mailbox()[1]:
            assert time.time() - t0 < 5.0
        assert _wait(mw, hs) == [mw.MW_DONE] * 2 and bool((big_d == 3).all())
        assert mw.mw_debug_mailbox()[2] == 2  # the large one was launched, not queued
        message(2)
        assert mw.mw_debug_mailbox()[0] == 3 and mw.mw_debug_mailbox()[1] == 1
    finally:
        t0 = time.time()
        mw.mw_shutdown()  # with a kernel open: it is asked to stop and ends at once
        assert time.time() - t0 < 2.0


def test_the_idle_time_is_configurable(mailbox, torch):
    """"mailbox_idle_us": with 20 ms the kernel is still open 2 ms after its last message and closes by itself later."""
    mw = mailbox
    before = mw.mw_config_get("mailbox_idle_us")
    assert before == 300
    with pytest.raises(mw.MwError):
        mw.mw_config_set("mailbox_idle_us", 5)
    mw.mw_config_set("mailbox_idle_us", 20000)
    mw.mw_init(0, 2)
    try:
        mw.mw_world_create(0, [0, 1])
        src = torch.arange(1024, dtype=torch.int32, device="cuda")
        dst = torch.zeros(1024, dtype=torch.int32, device="cuda")
        torch.cuda.current_stream().synchronize()
        hs = [mw.mw_send(0, 0, 1, src.data_ptr(), 1024, mw.MW_F32, mw.STREAM_NONE),
              mw.mw_recv(0, 0, 1, dst.data_ptr(), 1024, mw.MW_F32, mw.STREAM_NONE)]
        assert _wait(mw, hs) == [mw.MW_DONE] * 2
        t_done = time.time()
        time.sleep(0.002)
        still_open = mw.mw_debug_mailbox()[1]
        late = time.time() - t_done > 0.015  # (a stalled host: the check would say nothing)
        assert still_open == 1 or late
        while mw.mw_debug_mailbox()[1]:
            assert time.time() - t_done < 5.0, "the resident kernel did not end when idle"
        assert time.time() - t_done >= 0.015
        assert bool(torch.equal(src, dst))
    finally:
        mw.mw_shutdown()
        mw.mw_config_set("mailbox_idle_us", before)


def test_more_workers_than_compute_units_are_not_used(mailbox, torch):
    """A worker that is not resident serves its chunks only when the others have left (hundreds of microseconds later):
    the library uses at most one workgroup per compute unit, whatever "mailbox_workers" asks for."""
    mw = mailbox
    before = mw.mw_config_get("mailbox_workers")
    mw.mw_config_set("mailbox_workers", 700)
    mw.mw_init(0, 2)
    try:
        mw.mw_world_create(0, [0, 1])
        n = 70001  # five chunks: five workers per message, a different five every time
        src = torch.randint(0, 2 ** 31 - 1, (n,), dtype=torch.int32, device="cuda")
        dst = torch.zeros(n, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        took = []
        for k in range(300):
            t0 = time.perf_counter()
            hs = [mw.mw_send(0, 0, 1, src.data_ptr(), n, mw.MW_F32, mw.STREAM_NONE),
                  mw.mw_recv(0, 0, 1, dst.data_ptr(), n, mw.MW_F32, mw.STREAM_NONE)]
            assert _wait(mw, hs) == [mw.MW_DONE] * 2
            took.append(time.perf_counter() - t0)
        took.sort()
        assert mw.mw_debug_mailbox()[2] == 300 and bool(torch.equal(src, dst))
        assert took[len(took) // 2] < 100e-6, took[len(took) // 2]  # (with workers left out of the chip: > 300 us)
    finally:
        mw.mw_shutdown()
        mw.mw_config_set("mailbox_workers", before)


def test_more_descriptors_than_one_kernel_serves(mailbox, torch):
    """A resident kernel serves at most half the queue (2048 descriptors); 6000 one-chunk messages in windows of 16
    go through several kernels, with some windows launched the ordinary way while one kernel ends and the next has
    not begun -- every message arrives."""
    mw = mailbox
    mw.mw_init(0, 4)
    try:
        mw.mw_world_create(0, [0, 1])
        n_msgs, count = 6000, 256
        src = torch.randint(0, 2 ** 31 - 1, (n_msgs, count), dtype=torch.int32, device="cuda")
        dst = torch.zeros(n_msgs, count, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        for lo in range(0, n_msgs, 16):
            posts = []
            for k in range(lo, min(lo + 16, n_msgs)):
                posts.append((mw.POST_SEND, 0, 0, 1, src[k].data_ptr(), count, mw.MW_F32, mw.STREAM_NONE))
                posts.append((mw.POST_RECV, 0, 0, 1, dst[k].data_ptr(), count, mw.MW_F32, mw.STREAM_NONE))
            hs, rc = mw.mw_post_many(posts)
            assert set(_wait(mw, hs)) == {mw.MW_DONE}
        epoch, _, tail = mw.mw_debug_mailbox()
        assert epoch >= 3 and 5000 <= tail <= n_msgs
        assert np.array_equal(dst.cpu().numpy(), oracle.copy_result(src.cpu().numpy().view(np.uint8).ravel()).view(np.int32).reshape(n_msgs, count))
    finally:
        mw.mw_shutdown()
