"""Several host threads drive their own worlds through one library instance at the same time (each logical
worker's process in the paper is a thread here): every thread's results must equal the oracle's, and a world
aborted by one thread must not disturb the others."""

import threading
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle

N_THREADS = 6
ITERS = 150


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
    binding.mw_init(0, 4 * N_THREADS)
    yield binding
    binding.mw_shutdown()


def test_threads_stream_through_their_own_worlds(torch, mw):
    cap = 1 << 20
    host_src = [np.random.default_rng(300 + t).integers(0, 256, size=cap, dtype=np.uint8) for t in range(N_THREADS)]
    dev_src = [torch.from_numpy(h).cuda() for h in host_src]
    dev_dst = [torch.zeros(cap, dtype=torch.uint8, device="cuda") for _ in range(N_THREADS)]
    # thread t also all-reduces in a 3-rank world of its own
    red_host = [[np.random.default_rng(700 + 10 * t + r).integers(-8, 9, size=5000).astype(np.float32) for r in range(3)]
                for t in range(N_THREADS)]
    red_dev = [[torch.from_numpy(x).cuda() for x in red_host[t]] for t in range(N_THREADS)]
    torch.cuda.synchronize()
    for t in range(N_THREADS):
        mw.mw_world_create(t, [4 * t, 4 * t + 1])
        mw.mw_world_create(100 + t, [4 * t, 4 * t + 2, 4 * t + 3])
    errors, done = [], [0] * N_THREADS
    victim = N_THREADS - 1  # its copy world is aborted half-way by another thread

    def worker(t):
        try:
            rng = np.random.default_rng(t)
            for i in range(ITERS):
                n = int(rng.integers(1, cap // 2)) * 2
                off = int(rng.integers(0, cap - n + 1)) & ~1
                try:
                    hs = mw.mw_send(t, 0, 1, dev_src[t].data_ptr() + off, n // 2, mw.MW_BF16, mw.STREAM_NONE)
                    hr = mw.mw_recv(t, 0, 1, dev_dst[t].data_ptr() + off, n // 2, mw.MW_BF16, mw.STREAM_NONE)
                except mw.MwError as e:
                    assert t == victim and e.code == mw.MW_EBROKEN, (t, e.code)
                    break
                mw.mw_flush()
                t0 = time.time()
                while True:
                    st = mw.mw_poll(hr)
                    if st != mw.MW_PENDING:
                        break
                    assert time.time() - t0 < 30
                if st == mw.MW_BROKEN:
                    assert t == victim
                    break
                assert st == mw.MW_DONE and mw.mw_poll(hs) == mw.MW_DONE
                got = dev_dst[t][off:off + n].cpu().numpy()
                assert np.array_equal(got, oracle.copy_result(host_src[t][off:off + n])), (t, i)
                done[t] += 1
                if t == 0 and i == ITERS // 2:
                    mw.mw_world_abort(victim)
                if i % 10 == 0:  # integer-valued inputs: the sum is exact, so the check is bit for bit
                    hs3 = [mw.mw_allreduce_sum(100 + t, r, red_dev[t][r].data_ptr(), 5000, mw.MW_F32, mw.STREAM_NONE)
                           for r in range(3)]
                    mw.mw_flush()
                    while any(mw.mw_poll(h) == mw.MW_PENDING for h in hs3):
                        assert time.time() - t0 < 30
                    s, _ = oracle.allreduce_sum_f64([x.view(np.uint8) for x in red_host[t]], 5000, oracle.F32)
                    for r in range(3):
                        assert np.array_equal(red_dev[t][r].cpu().numpy().astype(np.float64), s), (t, i, r)
                    for r in range(3):  # next round starts from the same inputs
                        red_dev[t][r].copy_(torch.from_numpy(red_host[t][r]))
                    torch.cuda.synchronize()
        except BaseException as e:  # noqa: BLE001 - reported by the main thread
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(N_THREADS)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=120)
    assert not any(th.is_alive() for th in threads), "a thread is stuck"
    assert not errors, errors
    assert all(done[t] == ITERS for t in range(N_THREADS) if t != victim), done
    assert done[victim] < ITERS and mw.mw_world_state(victim) == mw.MW_BROKEN
    assert mw.mw_world_state(100 + victim) == mw.MW_ALIVE  # the victim's other world is untouched
