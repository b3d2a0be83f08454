"""reduce / all-gather / gather / scatter on the GPU against the CPU oracle (the communicator's other
four operations), alone and mixed with the first four in a seeded trace with worker aborts."""

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


@pytest.fixture(params=[1, 0], ids=["mailbox", "launched"])
def mw(torch, request):
    """Every test of this module runs twice: with small flushes served by the resident mailbox kernel (the library's
    default) and with every flush launched."""
    from paper_2407_08980_amd import binding

    binding.lib()
    before = binding.mw_config_get("mailbox")
    binding.mw_config_set("mailbox", request.param)
    binding.mw_init(0, 16)
    yield binding
    binding.mw_shutdown()
    binding.mw_config_set("mailbox", before)


def wait(mw, handles, timeout=60.0):
    mw.mw_flush()
    ps = mw.PollSet(handles)
    t0 = time.time()
    while ps.poll():
        assert time.time() - t0 < timeout, "operations did not complete"
    return list(ps.states)


def dev(torch, arr, offset=0):
    base = torch.full((offset + arr.size + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    view = base[offset:offset + arr.size]
    view.copy_(torch.from_numpy(arr))
    return base, view


def rand_bytes(n, seed):
    return np.random.default_rng(seed).integers(0, 256, size=n, dtype=np.uint8)


def test_mixed_trace_of_all_eight_operations(torch, host_pools):
    from oracle.run_trace import run_trace as run_oracle
    from paper_2407_08980_amd import trace_runner

    t = workloads.collectives_mix()
    mat = lambda spec: materialize(spec, host_pools)
    grun = trace_runner.run_trace(t, host_pools, mat)
    orun = run_oracle(t, mat)
    rep = compare_runs(t, orun, grun)
    assert rep["exact"] > 1000 and rep["toleranced"] > 100
    assert grun.world_state == orun.world_state and "broken" in grun.world_state.values()
    assert set(grun.status.values()) == {"done", "broken"}


@pytest.mark.parametrize("n", [2, 3, 5, 8])
def test_gather_scatter_allgather_every_root(torch, mw, n):
    mw.mw_world_create(0, list(range(n)))
    for count, dtype, off in [(1, "bf16", 0), (4099, "f32", 0), (70001, "bf16", 2), (300003, "f32", 4)]:
        isz = 4 if dtype == "f32" else 2
        S = count * isz
        dt = mw.DTYPES[dtype]
        send = [rand_bytes(S, 7000 + 100 * n + r) for r in range(n)]
        sdev = [dev(torch, send[r], off) for r in range(n)]
        # all-gather, rank n-1 contributing in place
        rdev = [dev(torch, np.full(n * S, 0xA5, np.uint8), off) for r in range(n)]
        rdev[n - 1][1][(n - 1) * S:n * S].copy_(sdev[n - 1][1])
        hs = []
        for r in reversed(range(n)):
            sp = sdev[r][1].data_ptr() if r != n - 1 else rdev[r][1].data_ptr() + r * S
            hs.append(mw.mw_all_gather(0, r, sp, rdev[r][1].data_ptr(), count, dt))
        assert wait(mw, hs) == [mw.MW_DONE] * n
        want = oracle.all_gather_result(send)
        for r in range(n):
            base = rdev[r][0].cpu().numpy()
            assert np.array_equal(base[off:off + n * S], want), (n, count, r)
            assert np.all(base[:off] == 0x5A) and np.all(base[off + n * S:] == 0x5A)
        for root in range(n):
            groot = dev(torch, np.full(n * S, 0xA5, np.uint8), off)
            hs = [mw.mw_gather(0, r, root, sdev[r][1].data_ptr(), groot[1].data_ptr() if r == root else None, count, dt)
                  for r in range(n)]
            assert wait(mw, hs) == [mw.MW_DONE] * n
            assert np.array_equal(groot[1].cpu().numpy(), oracle.gather_result(send)), (n, count, root)
            back = [dev(torch, np.full(S, 0xA5, np.uint8), off) for _ in range(n)]
            hs = [mw.mw_scatter(0, r, root, groot[1].data_ptr() if r == root else None, back[r][1].data_ptr(), count, dt)
                  for r in range(n)]
            assert wait(mw, hs) == [mw.MW_DONE] * n
            for r in range(n):
                got = back[r][0].cpu().numpy()
                assert np.array_equal(got[off:off + S], oracle.scatter_result(want, n, r)), (n, count, root, r)
                assert np.all(got[:off] == 0x5A) and np.all(got[off + S:] == 0x5A)
        for r in range(n):
            assert np.array_equal(sdev[r][1].cpu().numpy(), send[r])  # sources are only read


@pytest.mark.parametrize("lds", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 8])
def test_reduce_every_root(torch, mw, n, dtype, lds):
    mw.mw_config_set("reduce_lds", lds)
    try:
        mw.mw_world_create(0, list(range(n)))
        isz = 4 if dtype == "f32" else 2
        for count, off_elems in [(5, 0), (65536 + 3, 0), (100001, 1)]:
            for root in sorted({0, n // 2, n - 1}):
                rng = np.random.default_rng(n * 1000 + count + root)
                xs = [rng.uniform(-1, 1, count).astype(np.float32) for _ in range(n)]
                host = [x.view(np.uint8) if dtype == "f32" else oracle.f32_to_bf16_bits(x).view(np.uint8) for x in xs]
                d = [dev(torch, host[r], off_elems * isz) for r in range(n)]
                hs = [mw.mw_reduce_sum(0, r, root, d[r][1].data_ptr(), count, mw.DTYPES[dtype]) for r in range(n)]
                assert wait(mw, hs) == [mw.MW_DONE] * n
                s, sabs = oracle.reduce_result_f64(host, count, dtype)
                got = d[root][1].cpu().numpy()
                ok, worst = oracle.allreduce_within_tolerance(got, s, sabs, count, dtype)
                assert ok, (n, dtype, count, root, worst)
                assert np.array_equal(got, oracle.allreduce_sum_ordered(host, count, dtype))
                for r in range(n):
                    if r != root:
                        assert np.array_equal(d[r][1].cpu().numpy(), host[r]), "a non-root buffer was written"
    finally:
        mw.mw_config_set("reduce_lds", 0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_real_valued_sums_forwarded_through_further_operations(torch, mw, dtype):
    """A buffer that has been all-reduced is sent on, broadcast, reduced again and all-reduced again, with N(0,1)
    values.  The device accumulates in fp32 in ascending rank order, so on the oracle's side each step continues
    from the bytes of its ascending-order fp32 sum: every step is then compared bit for bit, and every sum also
    against the float64 sum of the bytes that went into it, within the summation tolerance."""
    count = 300007
    isz = 4 if dtype == "f32" else 2
    dt = mw.DTYPES[dtype]
    rng = np.random.default_rng(77 if dtype == "f32" else 78)

    def draw():
        x = rng.standard_normal(count).astype(np.float32)
        return x.view(np.uint8).copy() if dtype == "f32" else oracle.f32_to_bf16_bits(x).view(np.uint8).copy()

    def check_sum(got, inputs, what):
        s, sabs = oracle.allreduce_sum_f64(inputs, count, dtype)
        ok, worst = oracle.allreduce_within_tolerance(got, s, sabs, count, dtype)
        assert ok, (what, worst)
        want = oracle.allreduce_sum_ordered(inputs, count, dtype)
        assert np.array_equal(got, want), what
        return want

    mw.mw_world_create(0, [0, 1, 2, 3])   # the first sum
    mw.mw_world_create(1, [0, 4])         # forwards it
    mw.mw_world_create(2, [4, 5, 6])      # broadcasts it, then reduces it with fresh tensors
    mw.mw_world_create(3, [5, 6])         # sums the reduction's result once more
    x = [draw() for _ in range(4)]
    d = [dev(torch, h)[1] for h in x]
    assert wait(mw, [mw.mw_allreduce_sum(0, r, d[r].data_ptr(), count, dt) for r in range(4)]) == [mw.MW_DONE] * 4
    s1 = check_sum(d[0].cpu().numpy(), x, "first all-reduce")
    for r in range(1, 4):
        assert np.array_equal(d[r].cpu().numpy(), s1)
    # worker 0 sends its sum to worker 4
    fwd = dev(torch, np.full(count * isz, 0xA5, np.uint8))[1]
    hs = [mw.mw_send(1, 0, 1, d[0].data_ptr(), count, dt), mw.mw_recv(1, 0, 1, fwd.data_ptr(), count, dt)]
    assert wait(mw, hs) == [mw.MW_DONE] * 2
    assert np.array_equal(fwd.cpu().numpy(), oracle.copy_result(s1))
    # worker 4 broadcasts it in world 2
    others = [dev(torch, np.full(count * isz, 0xA5, np.uint8))[1] for _ in range(2)]
    bufs = [fwd] + others
    assert wait(mw, [mw.mw_broadcast(2, r, 0, bufs[r].data_ptr(), count, dt) for r in range(3)]) == [mw.MW_DONE] * 3
    want = oracle.broadcast_result([s1, None, None], 0)
    for r in range(3):
        assert np.array_equal(bufs[r].cpu().numpy(), want[r]), r
    # ranks 1 and 2 add fresh tensors of their own into the copy they received, reduced onto rank 2
    fresh = [draw(), draw()]
    others[0].copy_(torch.from_numpy(fresh[0]).cuda())
    torch.cuda.synchronize()
    inputs = [s1, fresh[0], s1]
    assert wait(mw, [mw.mw_reduce_sum(2, r, 2, bufs[r].data_ptr(), count, dt) for r in range(3)]) == [mw.MW_DONE] * 3
    s2 = check_sum(bufs[2].cpu().numpy(), inputs, "reduce of forwarded sums")
    assert np.array_equal(bufs[0].cpu().numpy(), s1) and np.array_equal(bufs[1].cpu().numpy(), fresh[0])  # only read
    # workers 5 and 6 all-reduce: a fresh tensor and the reduction's result
    last = [dev(torch, fresh[1])[1], bufs[2]]
    assert wait(mw, [mw.mw_allreduce_sum(3, r, last[r].data_ptr(), count, dt) for r in range(2)]) == [mw.MW_DONE] * 2
    s3 = check_sum(last[0].cpu().numpy(), [fresh[1], s2], "all-reduce of a reduction's result")
    assert np.array_equal(last[1].cpu().numpy(), s3)
