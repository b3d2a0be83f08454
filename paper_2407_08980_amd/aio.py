"""asyncio face of the polling interface.

The paper's communicator issues its operations in a non-blocking fashion and waits for them by busy polling that
yields to the event loop whenever the operation is still pending, so that work on other worlds is scheduled at
once (Sec. 3.2, Sec. 3.3 "World Communicator"); a broken world surfaces as an exception the application can
handle (Sec. 3.3 "World Manager").  This module is that loop around mw_poll, nothing more: it moves no data and
keeps no state.
"""

from __future__ import annotations

import asyncio

from . import binding as mw


class BrokenWorldError(RuntimeError):
    """The operation's world broke before the operation had all its sides."""


class MismatchError(RuntimeError):
    """The sides of the operation disagreed (count, dtype, kind or root)."""


async def wait(handle):
    """Return when the operation is done; raise BrokenWorldError / MismatchError if it ended that way.
    Every poll that finds it pending gives the event loop a turn."""
    while True:
        st = mw.mw_poll(handle)
        if st == mw.MW_DONE:
            return
        if st == mw.MW_BROKEN:
            raise BrokenWorldError(f"handle {handle:#x}")
        if st == mw.MW_EMISMATCH:
            raise MismatchError(f"handle {handle:#x}")
        if st != mw.MW_PENDING:
            raise mw.MwError(st, "mw_poll")
        await asyncio.sleep(0)


async def wait_all(handles):
    """Wait for several operations; the first failure is raised after all of them have ended."""
    results = await asyncio.gather(*(wait(h) for h in handles), return_exceptions=True)
    for r in results:
        if isinstance(r, BaseException):
            raise r
