"""The asyncio face of polling (the paper's programming model, Sec. 3.2 / 3.3): a task waiting on a world whose
peer never shows up must not keep another task from streaming through its own world on the same event loop, and
a broken world must surface as an exception in the task that waits on it.  CPU only (byte-less device double)."""

import asyncio

import pytest

from paper_2407_08980_amd import aio
from paper_2407_08980_amd import binding as mw

from helpers import hostcheck_library


@pytest.fixture(scope="module")
def hostlib():
    lib = hostcheck_library()
    old = mw._lib
    mw.use_library(lib)
    yield lib
    mw._lib = old


def test_a_pending_world_does_not_hold_up_another_task(hostlib):
    mw.mw_init(0, 3)
    try:
        mw.mw_world_create(1, [0, 1])
        mw.mw_world_create(2, [0, 2])
        log = []

        async def stuck():
            h = mw.mw_recv(2, 1, 0, 0x2000, 4, mw.MW_F32)  # worker 2 never sends
            try:
                await aio.wait(h)
                log.append("stuck: done")
            except aio.BrokenWorldError:
                log.append("stuck: broken")

        async def streaming():
            for k in range(100):
                hs = mw.mw_send(1, 1, 0, 0x100, 4, mw.MW_F32)
                hr = mw.mw_recv(1, 1, 0, 0x200, 4, mw.MW_F32)
                mw.mw_flush()
                hostlib.mwt_complete(1, 0)  # the device double finishes the launched operation
                await aio.wait_all([hs, hr])
            log.append("streaming: 100 done")
            mw.mw_worker_abort(2)  # the silent peer is declared failed: only world 2 breaks

        async def mismatch():
            a = mw.mw_send(1, 0, 1, 0x100, 4, mw.MW_F32)
            b = mw.mw_recv(1, 0, 1, 0x200, 8, mw.MW_F32)
            with pytest.raises(aio.MismatchError):
                await aio.wait_all([a, b])
            log.append("mismatch: raised")

        async def main():
            await asyncio.wait_for(asyncio.gather(stuck(), streaming(), mismatch()), timeout=30)

        asyncio.run(main())
        assert sorted(log) == ["mismatch: raised", "streaming: 100 done", "stuck: broken"]
        assert log.index("streaming: 100 done") < log.index("stuck: broken")
        assert mw.mw_world_state(1) == mw.MW_ALIVE and mw.mw_world_state(2) == mw.MW_BROKEN
    finally:
        mw.mw_shutdown()
