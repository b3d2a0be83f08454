"""The workloads at their full sizes on the GPU, in the launch configuration bench.py times.

The oracle cannot hold these runs in host memory, so: terminal statuses are compared for every
operation (the oracle runs the whole trace without data); on the steps that between them use every
source tensor of every world (and on the last steps) the WHOLE destination is brought to the host and
compared with what the oracle computes from the input recipe, 64 MiB at a time; on the other checked
steps received == sent is checked on the device and seeded byte windows against the oracle.
"""

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
import workloads
from oracle.run_trace import run_trace as run_oracle
from workloads import materialize
from workloads.data import ITEMSIZE, pool_slice

from helpers import compare_runs


@pytest.fixture(scope="module")
def gpu():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2407_08980_amd import binding, trace_runner

    binding.lib()
    return trace_runner


def window_of(spec, pools, lo, n):
    """Bytes [lo, lo+n) of a buffer's initial contents, from its recipe."""
    kind = spec.init[0]
    if kind == "fill":
        return np.full(n, spec.init[1], np.uint8)
    assert kind == "pool" and lo % ITEMSIZE[spec.init[1]] == 0
    return pool_slice(pools.get(spec.init[1]), spec.init[1], spec.init[2] + lo // ITEMSIZE[spec.init[1]], n)


def assert_whole_buffer(tensor, src_spec, pools, what, piece=64 << 20):
    """Every byte of a device buffer against the oracle's copy of its source's recipe bytes."""
    nbytes = src_spec.nbytes
    assert tensor.numel() == nbytes
    for lo in range(0, nbytes, piece):
        n = min(piece, nbytes - lo)
        want = oracle.copy_result(window_of(src_spec, pools, lo, n))
        got = tensor[lo:lo + n].cpu().numpy()
        if not np.array_equal(got, want):
            bad = np.flatnonzero(got != want)
            raise AssertionError(f"{what}: {bad.size} bytes differ from the oracle in [{lo}, {lo + n}), first at {lo + bad[0]}")


def windows(nbytes, rng, k=6, width=1 << 16):
    los = [0, max(0, nbytes - width)] + [int(x) & ~1 for x in rng.integers(0, max(1, nbytes - width), size=k)]
    return [(lo, min(width, nbytes - lo)) for lo in los]


def test_config2_full_size(gpu, host_pools):
    """8 worlds x 512 MiB bf16, 50 steps; data checked on steps 0-2, 24, 25, 47-49."""
    import torch

    steps = 50
    checked = [0, 1, 2, 24, 25, 47, 48, 49]
    t = workloads.config2(steps=steps, check_steps=checked)
    rng = np.random.default_rng(2)
    n_checked = [0]

    def check(idx, op, bufs):
        # which source fed this destination: step s of world i used src[i][s % 4], dst[i][s % 2]
        world, slot = divmod(op.buf - 8 * 4, 2)
        s = checked[n_checked[0] // 8]
        n_checked[0] += 1
        src_id = world * 4 + s % 4
        assert s % 2 == slot
        if s in (0, 1, 2, 47, 49):  # between them: all four source tensors of every world, and the last step
            assert_whole_buffer(bufs[op.buf], t.bufs[src_id], host_pools, f"world {world} step {s}")
            return
        assert torch.equal(bufs[op.buf], bufs[src_id]), f"world {world} step {s}: received != sent"
        for lo, n in windows(t.bufs[op.buf].nbytes, rng):
            want = oracle.copy_result(window_of(t.bufs[src_id], host_pools, lo, n))
            assert np.array_equal(bufs[op.buf][lo:lo + n].cpu().numpy(), want), (world, s, lo)

    grun = gpu.run_trace(t, host_pools, lambda sp: materialize(sp, host_pools), snapshots=False, check_fn=check)
    orun = run_oracle(t, None, data_bufs=set())
    compare_runs(t, orun, grun, require_checks=False)
    assert n_checked[0] == 8 * len(checked)
    assert all(v == "done" for v in grun.status.values()) and len(grun.status) == steps * 16
    assert grun.payload_bytes_done == steps * 8 * (512 << 20)


def test_config4_full_size_fault_isolation(gpu, host_pools):
    """16 worlds x 160 MiB bf16, 300 steps, worker 7 aborted before step 100."""
    import torch

    steps, abort_step = 300, 100
    checked = [0, 1, 98, 99, 100, 101, 102, 298, 299]
    t = workloads.config4(steps=steps, abort_step=abort_step, check_steps=checked)
    rng = np.random.default_rng(4)
    n_checked = [0]

    def check(idx, op, bufs):
        world, slot = divmod(op.buf - 16 * 4, 2)
        s = checked[n_checked[0] // 16]
        n_checked[0] += 1
        if world == 7 and s >= abort_step:
            assert bool((bufs[op.buf] == 0xA5).all()), f"step {s}: the broken world's destination was written"
            return
        src_id = world * 4 + s % 4
        if s in (0, 1, 98, 99, 299):  # all four source tensors of every world (98, 99 use the third and fourth), and the last step
            assert_whole_buffer(bufs[op.buf], t.bufs[src_id], host_pools, f"world {world} step {s}")
            return
        assert torch.equal(bufs[op.buf], bufs[src_id]), f"world {world} step {s}: received != sent"
        for lo, n in windows(t.bufs[op.buf].nbytes, rng, k=2):
            want = oracle.copy_result(window_of(t.bufs[src_id], host_pools, lo, n))
            assert np.array_equal(bufs[op.buf][lo:lo + n].cpu().numpy(), want), (world, s, lo)

    grun = gpu.run_trace(t, host_pools, lambda sp: materialize(sp, host_pools), snapshots=False, check_fn=check)
    orun = run_oracle(t, None, data_bufs=set())
    compare_runs(t, orun, grun, require_checks=False)
    assert n_checked[0] == 16 * len(checked)
    st = list(grun.status.values())
    assert st.count("done") == 2 * (15 * steps + abort_step) and st.count("broken") == 2 * (steps - abort_step)
    assert grun.world_state == orun.world_state and [w for w, s in grun.world_state.items() if s == "broken"] == [7]
    assert grun.payload_bytes_done == (15 * steps + abort_step) * (160 << 20)


def test_config3_full_length(gpu, host_pools):
    """4 worlds x 4 ranks, 500 iterations of two all-reduces; data checked on 12 iterations."""
    checked = [0, 1, 2, 3, 4, 5, 250, 251, 496, 497, 498, 499]
    t = workloads.config3(iters=500, check_iters=checked)
    mat = lambda sp: materialize(sp, host_pools)
    grun = gpu.run_trace(t, host_pools, mat)
    orun = run_oracle(t, mat)
    rep = compare_runs(t, orun, grun)
    assert rep["toleranced"] == len(checked) * 32 and rep["worst_allreduce_ratio"] <= 3 * 2.0 ** -24
    assert all(v == "done" for v in grun.status.values()) and len(grun.status) == 500 * 32


def test_config5_full_size(gpu, host_pools):
    """64 worlds, 10 000 mixed operations up to 64 MiB, three worker aborts: every status, and the
    data of every operation up to 1 MiB plus 5 % of the larger ones (about 250 of them, up to 64 MiB each)."""
    t = workloads.config5(check_small=1 << 20, check_fraction=0.05)
    mat = lambda sp: materialize(sp, host_pools)
    grun = gpu.run_trace(t, host_pools, mat)
    orun = run_oracle(t, mat)
    rep = compare_runs(t, orun, grun)
    assert len(grun.status) == len(orun.status) > 20000
    assert rep["exact"] > 7000 and rep["toleranced"] > 400
    assert grun.world_state == orun.world_state
    assert grun.payload_bytes_done == orun.payload_bytes_done


def test_headline_workload_in_the_benchmarks_own_loop(gpu, host_pools):
    """bench.py's launch configuration: its Workload object, its double-buffered posting loop, its streams.
    Every step's destinations are compared with the sources on the device, and byte windows of them with
    what the oracle computes from the input recipe (pool offsets are the benchmark's own seeded draw)."""
    import torch

    import bench
    from paper_2407_08980_amd import binding as mw
    from workloads.data import pool_slice

    dev = torch.device("cuda", 0)
    mw.mw_init(0, 2 * bench.N_WORLDS)
    try:
        wl = bench.Workload(torch, mw, bench.SHAPE, dev)
        for w in range(bench.N_WORLDS):
            mw.mw_world_create(w, [2 * w, 2 * w + 1])
        multi = (list(range(bench.N_WORLDS)), [(0, 1)] * bench.N_WORLDS)
        rng = np.random.default_rng(7)
        pool = host_pools.get("bf16")
        for first in (0, 3, 6):
            wl.run(3, *multi, first_step=first)  # steps first..first+2, two in flight at a time
            for s in (first + 1, first + 2):  # the two steps whose destinations are still intact
                for w in range(bench.N_WORLDS):
                    d, src = wl.dst[w][s % 2], wl.src[w][s % bench.POOL_K]
                    if s == 8:  # the last step: every byte of every world's destination against the oracle
                        for lo in range(0, wl.nbytes, 64 << 20):
                            n = min(64 << 20, wl.nbytes - lo)
                            want = oracle.copy_result(pool_slice(pool, "bf16", wl.offsets[w][s % bench.POOL_K] + lo // 2, n))
                            assert np.array_equal(d[lo:lo + n].cpu().numpy(), want), (w, s, lo)
                        continue
                    assert torch.equal(d, src), (w, s)
                    for lo, n in windows(wl.nbytes, rng, k=2):
                        want = oracle.copy_result(pool_slice(pool, "bf16", wl.offsets[w][s % bench.POOL_K] + lo // 2, n))
                        assert np.array_equal(d[lo:lo + n].cpu().numpy(), want), (w, s, lo)
            for w in range(bench.N_WORLDS):
                for d in wl.dst[w]:
                    d.fill_(0xA5)
            torch.cuda.synchronize()
    finally:
        mw.mw_shutdown()


def test_every_operation_at_the_large_payload_of_the_collectives_benchmark():
    """One world of 4 ranks, 64 MiB fp32 per rank (the payload `bench.py --workload collectives` times), all
    seven operations, every byte of every result against the oracle's per-operation functions."""
    import time

    import torch

    from paper_2407_08980_amd import binding as mw

    n, S = 4, 64 << 20
    count = S // 4
    mw.mw_init(0, n)
    try:
        mw.mw_world_create(0, list(range(n)))

        def wait(post):
            torch.cuda.synchronize()  # the posts below state (MW_STREAM_NONE) that their buffers are final
            hs = post()
            mw.mw_flush()
            ps = mw.PollSet(hs)
            t0 = time.time()
            while ps.poll():
                assert time.time() - t0 < 60
            assert list(ps.states) == [mw.MW_DONE] * len(hs)

        rng = np.random.default_rng(64)
        host = [rng.integers(-6, 7, size=count).astype(np.float32).view(np.uint8) for _ in range(n)]  # exact sums
        small = [torch.from_numpy(h).cuda() for h in host]
        big = [torch.full((n * S,), 0xA5, dtype=torch.uint8, device="cuda") for _ in range(n)]
        NONE = mw.STREAM_NONE

        # send / recv: 0 -> 1 into a fresh buffer
        dst = torch.zeros(S, dtype=torch.uint8, device="cuda")
        wait(lambda: [mw.mw_send(0, 0, 1, small[0].data_ptr(), count, mw.MW_F32, NONE),
              mw.mw_recv(0, 0, 1, dst.data_ptr(), count, mw.MW_F32, NONE)])
        assert np.array_equal(dst.cpu().numpy(), oracle.copy_result(host[0]))
        # all-gather
        wait(lambda: [mw.mw_all_gather(0, r, small[r].data_ptr(), big[r].data_ptr(), count, mw.MW_F32, NONE) for r in range(n)])
        want = oracle.all_gather_result(host)
        for r in range(n):
            assert np.array_equal(big[r].cpu().numpy(), want), r
        # gather to rank 2 (the other ranks' big buffers must stay as they are)
        for b in big:
            b.fill_(0x5A)
        wait(lambda: [mw.mw_gather(0, r, 2, small[r].data_ptr(), big[r].data_ptr() if r == 2 else None, count, mw.MW_F32, NONE)
              for r in range(n)])
        assert np.array_equal(big[2].cpu().numpy(), oracle.gather_result(host))
        assert all(bool((big[r] == 0x5A).all()) for r in range(n) if r != 2)
        # scatter from rank 1: its big buffer holds the gathered tensor of before
        big[1].copy_(big[2])
        outs = [torch.zeros(S, dtype=torch.uint8, device="cuda") for _ in range(n)]
        wait(lambda: [mw.mw_scatter(0, r, 1, big[1].data_ptr() if r == 1 else None, outs[r].data_ptr(), count, mw.MW_F32, NONE)
              for r in range(n)])
        src = oracle.gather_result(host)
        for r in range(n):
            assert np.array_equal(outs[r].cpu().numpy(), oracle.scatter_result(src, n, r)), r
        # broadcast from rank 3 into the scatter outputs
        outs[3].copy_(small[3])
        wait(lambda: [mw.mw_broadcast(0, r, 3, outs[r].data_ptr(), count, mw.MW_F32, NONE) for r in range(n)])
        want = oracle.broadcast_result([o.cpu().numpy() if r == 3 else None for r, o in enumerate(outs)], 3)
        for r in range(n):
            assert np.array_equal(outs[r].cpu().numpy(), want[r]), r
        # reduce to rank 1, then all-reduce (integer-valued inputs: the float64 sum is exactly representable)
        work = [s.clone() for s in small]
        wait(lambda: [mw.mw_reduce_sum(0, r, 1, work[r].data_ptr(), count, mw.MW_F32, NONE) for r in range(n)])
        s, sabs = oracle.reduce_result_f64(host, count, oracle.F32)
        got = work[1].cpu().numpy()
        assert oracle.allreduce_within_tolerance(got, s, sabs, count, oracle.F32)[0]
        assert np.array_equal(got.view(np.float32).astype(np.float64), s)
        for r in (0, 2, 3):
            assert np.array_equal(work[r].cpu().numpy(), host[r]), r
        work = [s_.clone() for s_ in small]
        wait(lambda: [mw.mw_allreduce_sum(0, r, work[r].data_ptr(), count, mw.MW_F32, NONE) for r in range(n)])
        s, sabs = oracle.allreduce_sum_f64(host, count, oracle.F32)
        ordered = oracle.allreduce_sum_ordered(host, count, oracle.F32)
        for r in range(n):
            got = work[r].cpu().numpy()
            assert oracle.allreduce_within_tolerance(got, s, sabs, count, oracle.F32)[0], r
            assert np.array_equal(got, ordered), r
    finally:
        mw.mw_shutdown()
