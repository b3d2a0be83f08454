"""Random, deliberately messy sequences of posts and aborts through the host runtime (on the byte-less
device double) and through the oracle: sides that never meet, counts / dtypes / roots / kinds that disagree,
ranks running ahead in their collective sequence, aborts in the middle.  After every step the state of
every handle must agree."""

import ctypes as C
import os

import numpy as np
import pytest

from oracle import BF16, BROKEN, DONE, F32, MISMATCH, PENDING, WorldOracle
from oracle.mw_oracle import OracleError
from paper_2407_08980_amd import binding as mw
from paper_2407_08980_amd import build as mwbuild

from helpers import hostcheck_library

STATE = {mw.MW_DONE: DONE, mw.MW_PENDING: PENDING, mw.MW_BROKEN: BROKEN, mw.MW_EMISMATCH: MISMATCH}


@pytest.fixture(scope="module")
def hostlib():
    lib = hostcheck_library()
    old = mw._lib
    mw.use_library(lib)
    yield lib
    mw._lib = old


@pytest.mark.parametrize("seed", range(6))
def test_random_post_sequences_agree_with_the_oracle(hostlib, seed):
    rng = np.random.default_rng(1000 + seed)
    n_workers = 8
    o = WorldOracle(n_workers)
    mw.mw_init(0, n_workers)
    try:
        worlds = {}
        pairs = []  # (oracle handle, library handle)
        next_world = 0

        def both(ofn, gfn):
            """Run the same call on both sides; argument errors must coincide."""
            try:
                oh, oerr = ofn(), None
            except OracleError as e:
                oh, oerr = None, e.code
            try:
                gh, gerr = gfn(), None
            except mw.MwError as e:
                gh, gerr = None, e.code
            if oerr == "EINVAL":
                assert gerr == mw.MW_EINVAL
            elif oerr is None and gerr == mw.MW_EBROKEN:
                assert o.status(oh) == BROKEN  # the oracle issues a handle that is broken from the start
            else:
                assert oerr is None and gerr is None, (oerr, gerr)
                pairs.append((oh, gh))

        for step in range(2000):
            r = rng.random()
            if r < 0.04 or not worlds:
                size = int(rng.integers(1, 4))
                members = tuple(int(x) for x in rng.choice(n_workers, size=size, replace=False))
                o.create(next_world, members)
                mw.mw_world_create(next_world, list(members))
                worlds[next_world] = members
                next_world += 1
            elif r < 0.05:
                w = int(rng.choice(list(worlds)))
                o.abort_world(w)
                mw.mw_world_abort(w)
            elif r < 0.053:
                k = int(rng.integers(0, n_workers))
                o.abort_worker(k)
                mw.mw_worker_abort(k)
            else:
                w = int(rng.choice(list(worlds)))
                n = len(worlds[w])
                a, b = int(rng.integers(0, n)), int(rng.integers(0, n))
                if rng.random() < 0.03:
                    a = int(rng.choice([-1, n]))  # out of range: refused by both sides
                count = int(rng.choice([0, 4, 4, 4, 4, 4, 4, 8]))
                dt, gdt = (F32, mw.MW_F32) if rng.random() < 0.9 else (BF16, mw.MW_BF16)
                kind = int(rng.integers(0, 8))
                buf, buf2 = 0x1000 + 64 * int(rng.integers(0, 64)), 0x9000 + 64 * int(rng.integers(0, 64))
                if kind == 0:
                    both(lambda: o.post_send(w, a, b, None, count, dt), lambda: mw.mw_send(w, a, b, buf, count, gdt))
                elif kind == 1:
                    both(lambda: o.post_recv(w, a, b, None, count, dt), lambda: mw.mw_recv(w, a, b, buf, count, gdt))
                elif kind == 2:
                    both(lambda: o.post_broadcast(w, a, b, None, count, dt), lambda: mw.mw_broadcast(w, a, b, buf, count, gdt))
                elif kind == 3:
                    both(lambda: o.post_allreduce(w, a, None, count, dt), lambda: mw.mw_allreduce_sum(w, a, buf, count, gdt))
                elif kind == 4:
                    both(lambda: o.post_reduce(w, a, b, None, count, dt), lambda: mw.mw_reduce_sum(w, a, b, buf, count, gdt))
                elif kind == 5:
                    both(lambda: o.post_all_gather(w, a, None, None, count, dt),
                         lambda: mw.mw_all_gather(w, a, buf, buf2, count, gdt))
                elif kind == 6:
                    both(lambda: o.post_gather(w, a, b, None, None, count, dt),
                         lambda: mw.mw_gather(w, a, b, buf, buf2, count, gdt))
                else:
                    both(lambda: o.post_scatter(w, a, b, None, None, count, dt),
                         lambda: mw.mw_scatter(w, a, b, buf, buf2, count, gdt))
            # let everything that can run, run; then every handle must be in the oracle's state
            mw.mw_flush()
            hostlib.mwt_complete(10 ** 6, int(rng.integers(0, 2)))
            if step % 10 == 0 or step > 1980:
                for oh, gh in pairs:
                    assert STATE[mw.mw_poll(gh)] == o.status(oh), (step, oh)
                for w in worlds:
                    assert (mw.mw_world_state(w) == mw.MW_BROKEN) == (o.world_state(w) == BROKEN)
        assert mw.mw_pending_ops() == 0
        seen = {o.status(oh) for oh, _ in pairs}
        assert {DONE, PENDING, BROKEN, MISMATCH} <= seen, seen
    finally:
        mw.mw_shutdown()
