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


@pytest.fixture
def mw(torch):
    from paper_2407_08980_amd import binding

    binding.lib()
    binding.mw_init(0, 16)
    yield binding
    binding.mw_shutdown()


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
