"""Watchdog (Sec. 3.3): heartbeats, timeout, automatic clean-up of exactly the failed worker's worlds.

The oracle is pinned by the closed form (a watched worker is declared failed at the first
inspection whose time exceeds its latest heartbeat by more than the timeout) and by the paper's
numbers (periodic reports, a timeout of about 3 seconds); the host runtime is then compared with
the oracle on seeded schedules with an explicit clock, and once with its own thread and the real
clock.  CPU only: the runtime is linked against the byte-less device double.
"""

import ctypes as C
import os
import time

import numpy as np
import pytest

from oracle import ALIVE, BROKEN, DONE, F32, PENDING, WorldOracle
from oracle.mw_oracle import OracleError
from paper_2407_08980_amd import binding as mw
from paper_2407_08980_amd import build as mwbuild

from helpers import hostcheck_library


@pytest.fixture(scope="module")
def hostlib():
    lib = hostcheck_library()
    old = mw._lib
    mw.use_library(lib)
    yield lib
    mw._lib = old


def test_oracle_watchdog_paper_numbers():
    """Workers report every second, the timeout is 3 s; one worker stops after t = 10."""
    o = WorldOracle(4)
    o.create(1, (0, 1))
    o.create(2, (0, 2))
    o.create(3, (1, 3))  # worker 3 never reports: it is not watched
    pend = {w: o.post_recv(w, 1, 0, np.zeros(4, np.uint8), 1, F32) for w in (1, 2, 3)}
    declared_at = None
    for t in range(0, 31):
        for k in (0, 1):
            o.heartbeat(k, float(t))
        if t <= 10:
            o.heartbeat(2, float(t))
        newly = o.watchdog_check(t + 0.5, 3.0)
        if newly:
            assert newly == [2] and declared_at is None
            declared_at = t + 0.5
    assert declared_at == 13.5  # first inspection later than 10 + 3
    assert o.world_state(2) == BROKEN and o.status(pend[2]) == BROKEN
    assert o.world_state(1) == ALIVE and o.world_state(3) == ALIVE
    assert o.status(pend[1]) == PENDING and o.status(pend[3]) == PENDING
    with pytest.raises(OracleError) as e:
        o.heartbeat(2, 40.0)  # a failed worker does not come back
    assert e.value.code == "EBROKEN"
    with pytest.raises(OracleError) as e:
        o.create(9, (0, 2))
    assert e.value.code == "EBROKEN"
    o.create(9, (0, 3))  # recovery: a new world with another worker
    # the boundary (a reading: reports count as missing once the latest one is OLDER than the timeout):
    # a report exactly 3 s old is not yet a miss, anything older is
    o = WorldOracle(2)
    o.create(1, (0, 1))
    o.heartbeat(1, 10.0)
    assert o.watchdog_check(13.0, 3.0) == [] and o.world_state(1) == ALIVE
    assert o.watchdog_check(13.0 + 2 ** -20, 3.0) == [1] and o.world_state(1) == BROKEN


def _schedule(seed, n_workers=8, n_events=300):
    rng = np.random.default_rng(seed)
    t = 0.0
    quiet_from = {int(k): float(rng.uniform(5, 40)) for k in rng.choice(n_workers, size=3, replace=False)}
    never = int(rng.integers(0, n_workers))
    ev = []
    for _ in range(n_events):
        t += float(rng.exponential(0.2))
        if rng.random() < 0.2:
            ev.append(("check", t))
        else:
            k = int(rng.integers(0, n_workers))
            if k != never and t < quiet_from.get(k, 1e9):
                ev.append(("beat", t, k))
    ev.append(("check", t + 100.0))
    return ev, quiet_from, never


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_oracle_watchdog_closed_form(seed):
    ev, quiet_from, never = _schedule(seed)
    timeout = 2.5
    o = WorldOracle(8)
    last, dead_at = {}, {}
    for e in ev:
        if e[0] == "beat":
            if e[2] in dead_at:  # random gaps can exceed the timeout: such a worker stays failed
                with pytest.raises(OracleError):
                    o.heartbeat(e[2], e[1])
                continue
            o.heartbeat(e[2], e[1])
            last[e[2]] = e[1]
        else:
            newly = o.watchdog_check(e[1], timeout)
            want = sorted(k for k, tb in last.items() if k not in dead_at and e[1] - tb > timeout)
            assert newly == want
            for k in want:
                dead_at[k] = e[1]
    assert never not in dead_at and set(quiet_from) <= set(dead_at)


@pytest.mark.parametrize("seed", [11, 12])
def test_runtime_matches_oracle_with_explicit_clock(hostlib, seed):
    ev, _, _ = _schedule(seed)
    timeout = 2.5
    rng = np.random.default_rng(seed)
    worlds = {w: tuple(int(x) for x in rng.choice(8, size=int(rng.integers(2, 4)), replace=False)) for w in range(10)}
    o = WorldOracle(8)
    mw.mw_init(0, 8)
    try:
        oh, gh = {}, {}
        for w, m in worlds.items():
            o.create(w, m)
            mw.mw_world_create(w, list(m))
            oh[w] = o.post_recv(w, 1, 0, None, 4, F32)
            gh[w] = mw.mw_recv(w, 1, 0, 0x1000, 4, mw.MW_F32)
        for e in ev:
            if e[0] == "beat":
                try:
                    o.heartbeat(e[2], e[1])
                    oerr = None
                except OracleError as x:
                    oerr = x.code
                try:
                    mw.mw_heartbeat_at(e[2], e[1])
                    gerr = None
                except mw.MwError as x:
                    gerr = x.code
                assert (oerr, gerr) in ((None, None), ("EBROKEN", mw.MW_EBROKEN))
            else:
                assert mw.mw_watchdog_check_at(e[1], timeout) == len(o.watchdog_check(e[1], timeout))
                for w in worlds:
                    assert (mw.mw_world_state(w) == mw.MW_BROKEN) == (o.world_state(w) == BROKEN)
                    assert (mw.mw_poll(gh[w]) == mw.MW_BROKEN) == (o.status(oh[w]) == BROKEN)
        assert {k for k in range(8) if mw.mw_worker_state(k) == mw.MW_BROKEN} == o.dead and o.dead
        dead = next(iter(o.dead))
        with pytest.raises(mw.MwError) as e:
            mw.mw_world_create(99, [dead, (dead + 1) % 8])
        assert e.value.code == mw.MW_EBROKEN
        alive = next(k for k in range(8) if k not in o.dead)  # the boundary: exactly as old as the timeout is no miss
        mw.mw_heartbeat_at(alive, 1000.0)
        mw.mw_watchdog_check_at(1000.0 + timeout, timeout)
        assert mw.mw_worker_state(alive) == mw.MW_ALIVE
        mw.mw_watchdog_check_at(1000.0 + timeout + 2 ** -20, timeout)
        assert mw.mw_worker_state(alive) == mw.MW_BROKEN
    finally:
        mw.mw_shutdown()


def test_watchdog_thread_breaks_only_the_silent_workers_worlds(hostlib):
    """The Fig. 4 setting with silent failure: the leader (worker 0) is in W1 and W2; W2's peer sends
    ten tensors and then stops reporting.  The watchdog thread cleans up W2, W1 keeps working."""
    mw.mw_init(0, 3)
    try:
        mw.mw_world_create(1, [0, 1])
        mw.mw_world_create(2, [0, 2])
        mw.mw_watchdog_start(0.25, 0.02)
        with pytest.raises(mw.MwError):
            mw.mw_watchdog_start(0.25, 0.02)
        got = {1: 0, 2: 0}
        for k in range(10):
            for w in (1, 2):
                mw.mw_heartbeat(w)
                hs = mw.mw_send(w, 1, 0, 0x100, 4, mw.MW_F32)
                hr = mw.mw_recv(w, 1, 0, 0x200, 4, mw.MW_F32)
                mw.mw_flush()
                hostlib.mwt_complete(1, 0)
                got[w] += mw.mw_poll(hr) == mw.MW_DONE
            mw.mw_heartbeat(0)
        waiting = mw.mw_recv(2, 1, 0, 0x200, 4, mw.MW_F32)  # the leader already waits for the 11th tensor
        t0 = time.time()
        while mw.mw_world_state(2) == mw.MW_ALIVE and time.time() - t0 < 5:
            mw.mw_heartbeat(0)
            mw.mw_heartbeat(1)
            hs = mw.mw_send(1, 1, 0, 0x100, 4, mw.MW_F32)
            hr = mw.mw_recv(1, 1, 0, 0x200, 4, mw.MW_F32)
            mw.mw_flush()
            hostlib.mwt_complete(1, 0)
            got[1] += mw.mw_poll(hr) == mw.MW_DONE
            time.sleep(0.01)
        dt = time.time() - t0
        assert mw.mw_world_state(2) == mw.MW_BROKEN and 0.2 < dt < 2.0
        assert mw.mw_poll(waiting) == mw.MW_BROKEN and got[2] == 10 and got[1] > 10
        assert mw.mw_worker_state(2) == mw.MW_BROKEN and mw.mw_worker_state(1) == mw.MW_ALIVE
        assert mw.mw_world_state(1) == mw.MW_ALIVE and mw.mw_heartbeat_epoch(2) == 10
        mw.mw_watchdog_stop()
        mw.mw_watchdog_stop()
    finally:
        mw.mw_shutdown()
