"""Host runtime on the CPU: matching, handles, ring slots, abort, deferred ring release.

These tests link the host runtime against a device test double that records
launches and moves no bytes (libmw_hostcheck.so); the test decides when launched
operations "complete".  The product library is also loaded to check that it exports
every symbol the header declares (no compute calls: there is no GPU here).
"""

import ctypes as C
import os
import re

import pytest

from paper_2407_08980_amd import binding as mw
from paper_2407_08980_amd import build as mwbuild

from helpers import ROOT, hostcheck_library


@pytest.fixture(scope="module")
def hostlib():
    lib = hostcheck_library()
    lib.mwt_log_entry.argtypes = [C.c_int, C.POINTER(C.c_uint64)]
    old = mw._lib
    mw.use_library(lib)
    yield lib
    mw._lib = old


@pytest.fixture
def ctx(hostlib):
    mw.mw_init(0, 8)
    yield hostlib
    mw.mw_shutdown()


def log_entry(lib, i):
    out = (C.c_uint64 * 26)()
    assert lib.mwt_log_entry(i, out) == 0
    return dict(buf=list(out[:8]), nbytes=out[8], kind=out[9], dtype=out[10], nbuf=out[11], slot=out[12],
                gen=out[13], world=out[14], epoch=out[15], launch=out[16], root=out[17], buf_hi=list(out[18:26]))


def _id_in_child(path):
    import multiprocessing as mp

    with mp.get_context("spawn").Pool(1) as pool:  # a library mapped here would not be reloaded after a rebuild
        return pool.apply(mwbuild.library_id, (path,))


def test_header_symbols_are_exported_by_the_product_library():
    if not os.path.exists(mw.LIB_PATH) or _id_in_child(mw.LIB_PATH) != mwbuild.source_id():
        mwbuild.build_product()  # missing, or compiled from other sources than the ones in the tree
    text = open(os.path.join(ROOT, "include", "mw.h")).read()
    declared = set(re.findall(r"^\s*(?:int|long|const char\*)\s+(mw_\w+)\s*\(", text, flags=re.M))
    assert {"mw_world_create", "mw_send", "mw_recv", "mw_broadcast", "mw_allreduce_sum", "mw_poll",
            "mw_world_abort"} <= declared
    lib = C.CDLL(mw.LIB_PATH)
    missing = [s for s in sorted(declared) if not hasattr(lib, s)]
    assert not missing, missing
    assert declared == set(mw.SYMBOLS), declared ^ set(mw.SYMBOLS)
    lib.mw_build_id.restype = C.c_char_p
    assert lib.mw_build_id().decode() == mwbuild.source_id()
    # without a GPU the library must refuse loudly, not fall back
    import torch

    if not torch.cuda.is_available():
        lib.mw_init.argtypes = [C.c_int, C.c_int]
        assert lib.mw_init(0, 2) == mw.MW_EHIP
        assert lib.mw_poll(C.c_uint64(1 << 32)) == mw.MW_ENOTINIT


def test_calls_before_init_are_refused(hostlib):
    assert hostlib.mw_flush() == mw.MW_ENOTINIT
    assert hostlib.mw_poll(C.c_uint64(1 << 32)) == mw.MW_ENOTINIT
    with pytest.raises(mw.MwError) as e:
        mw.mw_world_create(0, [0, 1])
    assert e.value.code == mw.MW_ENOTINIT


def test_rendezvous_matching_and_batched_launch(ctx):
    mw.mw_world_create(5, [0, 1])
    mw.mw_world_create(6, [0, 2])
    hs = mw.mw_send(5, 1, 0, 0x1000, 100, mw.MW_F32)
    assert mw.mw_poll(hs) == mw.MW_PENDING and ctx.mwt_launch_count() == 0  # no receiver yet: nothing launched
    hr = mw.mw_recv(5, 1, 0, 0x2000, 100, mw.MW_F32)
    h2r = mw.mw_recv(6, 1, 0, 0x4000, 7, mw.MW_BF16)
    h2s = mw.mw_send(6, 1, 0, 0x3000, 7, mw.MW_BF16)
    assert mw.mw_pending_ops() == 2 and ctx.mwt_launch_count() == 0
    mw.mw_flush()
    assert ctx.mwt_launch_count() == 1 and ctx.mwt_launch_size(0) == 2  # one launch covers both worlds
    a, b = log_entry(ctx, 0), log_entry(ctx, 1)
    assert (a["buf"][:2], a["nbytes"], a["kind"], a["world"]) == ([0x1000, 0x2000], 400, 0, 5)
    assert (b["buf"][:2], b["nbytes"], b["kind"], b["world"]) == ([0x3000, 0x4000], 14, 0, 6)
    assert a["slot"] // 128 != b["slot"] // 128  # each world has its own ring
    assert [mw.mw_poll(h) for h in (hs, hr, h2s, h2r)] == [mw.MW_PENDING] * 4
    ctx.mwt_complete(1, 0)
    assert [mw.mw_poll(h) for h in (hs, hr, h2s, h2r)] == [mw.MW_DONE, mw.MW_DONE, mw.MW_PENDING, mw.MW_PENDING]
    ctx.mwt_complete(1, 0)
    assert mw.mw_poll(h2r) == mw.MW_DONE and mw.mw_poll(h2s) == mw.MW_DONE and mw.mw_pending_ops() == 0
    assert mw.mw_poll(hs) == mw.MW_DONE  # sticky


def test_poll_launches_on_demand(ctx):
    mw.mw_world_create(0, [0, 1])
    hs = mw.mw_send(0, 0, 1, 0x10, 4, mw.MW_F32)
    hr = mw.mw_recv(0, 0, 1, 0x20, 4, mw.MW_F32)
    assert ctx.mwt_launch_count() == 0
    assert mw.mw_poll(hr) == mw.MW_PENDING and ctx.mwt_launch_count() == 1
    ctx.mwt_complete(1, 0)
    assert mw.mw_poll(hs) == mw.MW_DONE


def test_fifo_per_pair_and_no_crosstalk(ctx):
    mw.mw_world_create(0, [0, 1, 2])
    sends = [mw.mw_send(0, 1, 0, 0x1000 + 16 * k, 1, mw.MW_F32) for k in range(5)]
    other = mw.mw_send(0, 2, 0, 0x9000, 1, mw.MW_F32)
    recvs = [mw.mw_recv(0, 1, 0, 0x2000 + 16 * k, 1, mw.MW_F32) for k in range(5)]
    mw.mw_flush()
    assert ctx.mwt_log_size() == 5
    for k in range(5):
        assert log_entry(ctx, k)["buf"][:2] == [0x1000 + 16 * k, 0x2000 + 16 * k]
    assert mw.mw_poll(other) == mw.MW_PENDING


def test_mismatch_and_zero_count(ctx):
    mw.mw_world_create(0, [0, 1])
    hs = mw.mw_send(0, 0, 1, 0x10, 8, mw.MW_F32)
    hr = mw.mw_recv(0, 0, 1, 0x20, 4, mw.MW_F32)
    assert mw.mw_poll(hs) == mw.MW_EMISMATCH and mw.mw_poll(hr) == mw.MW_EMISMATCH
    hs = mw.mw_send(0, 0, 1, 0x10, 8, mw.MW_BF16)
    hr = mw.mw_recv(0, 0, 1, 0x20, 8, mw.MW_F32)
    assert mw.mw_poll(hs) == mw.MW_EMISMATCH and mw.mw_poll(hr) == mw.MW_EMISMATCH
    hs = mw.mw_send(0, 0, 1, 0, 0, mw.MW_F32)
    hr = mw.mw_recv(0, 0, 1, 0, 0, mw.MW_F32)
    assert mw.mw_poll(hs) == mw.MW_DONE and mw.mw_poll(hr) == mw.MW_DONE
    assert ctx.mwt_launch_count() == 0


def test_argument_errors(ctx):
    mw.mw_world_create(0, [0, 1])
    for args, code in [((0, 0, 0, 0x10, 1), mw.MW_EINVAL), ((0, 0, 2, 0x10, 1), mw.MW_EINVAL),
                       ((0, -1, 1, 0x10, 1), mw.MW_EINVAL), ((9, 0, 1, 0x10, 1), mw.MW_ENOWORLD),
                       ((0, 0, 1, 0, 1), mw.MW_EINVAL)]:
        with pytest.raises(mw.MwError) as e:
            mw.mw_send(*args, mw.MW_F32)
        assert e.value.code == code
    for members, code in [([0, 0], mw.MW_EINVAL), ([0, 8], mw.MW_EINVAL), ([], mw.MW_EINVAL)]:
        with pytest.raises(mw.MwError) as e:
            mw.mw_world_create(3, members)
        assert e.value.code == code
    with pytest.raises(mw.MwError) as e:
        mw.mw_world_create(0, [2, 3])
    assert e.value.code == mw.MW_EEXIST
    with pytest.raises(mw.MwError) as e:
        mw.mw_allreduce_sum(0, 0, 0x11, 4, mw.MW_F32)  # not aligned to the element size
    assert e.value.code == mw.MW_EINVAL
    assert mw.mw_poll(12345) == mw.MW_EBADHANDLE and mw.mw_poll((77 << 32) | 3) == mw.MW_EBADHANDLE
    with pytest.raises(mw.MwError) as e:
        mw.mw_world_state(42)
    assert e.value.code == mw.MW_ENOWORLD


def test_collectives_sequence_and_descriptor_order(ctx):
    mw.mw_world_create(0, [0, 1, 2])
    # rank 2 runs ahead by two collectives
    h = [mw.mw_allreduce_sum(0, 2, 0x300, 16, mw.MW_F32), mw.mw_broadcast(0, 2, 1, 0x310, 8, mw.MW_BF16)]
    h += [mw.mw_allreduce_sum(0, 0, 0x100, 16, mw.MW_F32), mw.mw_allreduce_sum(0, 1, 0x200, 16, mw.MW_F32)]
    mw.mw_flush()
    assert ctx.mwt_log_size() == 1
    e = log_entry(ctx, 0)
    assert (e["kind"], e["nbuf"], e["buf"][:3], e["nbytes"]) == (2, 3, [0x100, 0x200, 0x300], 64)
    h += [mw.mw_broadcast(0, 0, 1, 0x110, 8, mw.MW_BF16), mw.mw_broadcast(0, 1, 1, 0x210, 8, mw.MW_BF16)]
    mw.mw_flush()
    e = log_entry(ctx, 1)
    assert (e["kind"], e["nbuf"], e["buf"][:3], e["nbytes"]) == (1, 3, [0x210, 0x110, 0x310], 16)  # root first
    ctx.mwt_complete(2, 0)
    assert [mw.mw_poll(x) for x in h] == [mw.MW_DONE] * 6
    # disagreement on the root
    a = mw.mw_broadcast(0, 0, 0, 0x110, 8, mw.MW_BF16)
    b = mw.mw_broadcast(0, 1, 1, 0x210, 8, mw.MW_BF16)
    c = mw.mw_broadcast(0, 2, 0, 0x310, 8, mw.MW_BF16)
    assert [mw.mw_poll(x) for x in (a, b, c)] == [mw.MW_EMISMATCH] * 3


def test_abort_breaks_unmatched_delivers_matched_and_refuses_later_posts(ctx):
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [0, 2])
    matched_s = mw.mw_send(0, 1, 0, 0x10, 4, mw.MW_F32)
    matched_r = mw.mw_recv(0, 1, 0, 0x20, 4, mw.MW_F32)  # all sides present, not launched yet
    lonely = mw.mw_recv(0, 1, 0, 0x30, 4, mw.MW_F32)
    coll = mw.mw_allreduce_sum(0, 0, 0x40, 4, mw.MW_F32)
    other = mw.mw_recv(1, 1, 0, 0x50, 4, mw.MW_F32)
    marks = ctx.mwt_marks()
    mw.mw_world_abort(0)
    mw.mw_world_abort(0)  # idempotent
    assert ctx.mwt_marks() == marks + 1  # one header write: broken + bumped epoch
    assert mw.mw_world_state(0) == mw.MW_BROKEN and mw.mw_world_state(1) == mw.MW_ALIVE
    assert mw.mw_poll(lonely) == mw.MW_BROKEN and mw.mw_poll(coll) == mw.MW_BROKEN
    assert mw.mw_poll(other) == mw.MW_PENDING
    assert ctx.mwt_launch_count() == 1  # the matched pair was launched by the abort so that it retires
    assert mw.mw_poll(matched_r) == mw.MW_PENDING
    ctx.mwt_complete(1, 0)
    assert mw.mw_poll(matched_s) == mw.MW_DONE and mw.mw_poll(matched_r) == mw.MW_DONE
    for f in (lambda: mw.mw_send(0, 1, 0, 0x10, 4, mw.MW_F32), lambda: mw.mw_allreduce_sum(0, 1, 0x40, 4, mw.MW_F32)):
        with pytest.raises(mw.MwError) as e:
            f()
        assert e.value.code == mw.MW_EBROKEN
    hs = mw.mw_send(1, 1, 0, 0x60, 4, mw.MW_F32)
    mw.mw_flush()
    ctx.mwt_complete(1, 0)
    assert mw.mw_poll(hs) == mw.MW_DONE and mw.mw_poll(other) == mw.MW_DONE


def test_worker_abort_breaks_exactly_the_worlds_containing_it(ctx):
    worlds = {10: [0, 1], 11: [0, 2], 12: [1, 3], 13: [2, 3], 14: [4, 5, 6]}
    for w, m in worlds.items():
        mw.mw_world_create(w, m)
    mw.mw_worker_abort(2)
    assert {w for w in worlds if mw.mw_world_state(w) == mw.MW_BROKEN} == {11, 13}
    mw.mw_worker_abort(7)  # member of nothing
    assert {w for w in worlds if mw.mw_world_state(w) == mw.MW_BROKEN} == {11, 13}


def test_ring_slots_recycle_and_full_ring_defers(hostlib):
    mw.mw_config_set("ring_depth", 4)
    try:
        mw.mw_init(0, 4)
        mw.mw_world_create(0, [0, 1])
        mw.mw_world_create(1, [2, 3])
        hs = []
        for k in range(6):
            mw.mw_send(0, 0, 1, 0x1000 + k, 1, mw.MW_F32)
            hs.append(mw.mw_recv(0, 0, 1, 0x2000 + k, 1, mw.MW_F32))
        mw.mw_flush()
        assert hostlib.mwt_launch_size(0) == 4 and mw.mw_pending_ops() == 6  # two wait for a slot
        slots = {log_entry(hostlib, i)["slot"] for i in range(4)}
        assert len(slots) == 4
        # the other world is not held up by the full ring
        mw.mw_send(1, 0, 1, 0x3000, 1, mw.MW_F32)
        ho = mw.mw_recv(1, 0, 1, 0x4000, 1, mw.MW_F32)
        mw.mw_flush()
        assert hostlib.mwt_launch_size(1) == 1 and log_entry(hostlib, 4)["world"] == 1
        hostlib.mwt_complete(2, 0)
        assert mw.mw_poll(hs[5]) == mw.MW_PENDING  # polling a deferred op retires finished ones and launches it
        assert hostlib.mwt_launch_count() == 3 and hostlib.mwt_launch_size(2) == 2
        reused = [log_entry(hostlib, i) for i in (5, 6)]
        assert {e["slot"] for e in reused} <= slots and all(e["gen"] == 2 for e in reused)
        hostlib.mwt_complete(10, 0)
        assert [mw.mw_poll(h) for h in hs] == [mw.MW_DONE] * 6 and mw.mw_poll(ho) == mw.MW_DONE
    finally:
        mw.mw_shutdown()
        mw.mw_config_set("ring_depth", 128)


def test_ring_of_a_broken_world_is_reused_only_after_its_operations_retired(hostlib):
    mw.mw_config_set("max_rings", 2)
    try:
        mw.mw_init(0, 6)
        mw.mw_world_create(0, [0, 1])
        mw.mw_world_create(1, [2, 3])
        mw.mw_send(0, 0, 1, 0x10, 1, mw.MW_F32)
        h = mw.mw_recv(0, 0, 1, 0x20, 1, mw.MW_F32)
        mw.mw_flush()
        ring0 = log_entry(hostlib, 0)["slot"] // 128
        mw.mw_world_abort(0)
        with pytest.raises(mw.MwError) as e:
            mw.mw_world_create(2, [4, 5])  # world 0's operation is still in flight: its ring is not free
        assert e.value.code == mw.MW_ENOMEM
        hostlib.mwt_complete(1, 0)
        mw.mw_world_create(2, [4, 5])  # retires world 0's operation, takes over its ring
        assert mw.mw_poll(h) == mw.MW_DONE
        mw.mw_send(2, 0, 1, 0x30, 1, mw.MW_F32)
        mw.mw_recv(2, 0, 1, 0x40, 1, mw.MW_F32)
        mw.mw_flush()
        e2 = log_entry(hostlib, 1)
        assert e2["slot"] // 128 == ring0 and e2["gen"] >= 1 and e2["world"] == 2
        with pytest.raises(mw.MwError) as e:
            mw.mw_world_create(0, [0, 1])  # ids are never reused
        assert e.value.code == mw.MW_EEXIST
    finally:
        mw.mw_shutdown()
        mw.mw_config_set("max_rings", 1024)


def test_handles_are_recycled_only_when_terminal(hostlib):
    mw.mw_config_set("handle_capacity", 16)
    try:
        mw.mw_init(0, 2)
        mw.mw_world_create(0, [0, 1])
        stuck = mw.mw_recv(0, 1, 0, 0x10, 1, mw.MW_F32)  # never matched: must survive any number of posts
        first = None
        for k in range(100):
            hs = mw.mw_send(0, 0, 1, 0x20, 0, mw.MW_F32)
            hr = mw.mw_recv(0, 0, 1, 0x30, 0, mw.MW_F32)
            first = first or hs
            assert mw.mw_poll(hs) == mw.MW_DONE and mw.mw_poll(hr) == mw.MW_DONE
        assert mw.mw_poll(stuck) == mw.MW_PENDING
        assert mw.mw_poll(first) == mw.MW_EBADHANDLE  # its slot has a newer generation now
        pend = [mw.mw_recv(0, 1, 0, 0x10, 1, mw.MW_F32) for _ in range(15)]
        with pytest.raises(mw.MwError) as e:
            mw.mw_recv(0, 1, 0, 0x10, 1, mw.MW_F32)
        assert e.value.code == mw.MW_ENOMEM  # every slot holds a live operation
        assert all(mw.mw_poll(h) == mw.MW_PENDING for h in pend)
    finally:
        mw.mw_shutdown()
        mw.mw_config_set("handle_capacity", 1 << 20)


def test_launch_failure_is_reported_and_nothing_is_lost(ctx):
    mw.mw_world_create(0, [0, 1])
    mw.mw_send(0, 0, 1, 0x10, 1, mw.MW_F32)
    h = mw.mw_recv(0, 0, 1, 0x20, 1, mw.MW_F32)
    ctx.mwt_fail_next_launch()
    with pytest.raises(mw.MwError) as e:
        mw.mw_flush()
    assert e.value.code == mw.MW_EHIP and mw.mw_pending_ops() == 1
    mw.mw_flush()
    ctx.mwt_complete(1, 0)
    assert mw.mw_poll(h) == mw.MW_DONE


def test_polls_and_flushes_look_after_work_left_without_a_kernel(ctx):
    """When the backend says that queued work has no kernel to serve it (its resident kernel closed as the work came
    in), the next poll of a pending operation -- also the lock-free kind -- and the next flush must have it looked after."""
    mw.mw_world_create(0, [0, 1])
    mw.mw_send(0, 0, 1, 0x10, 1, mw.MW_F32)
    h = mw.mw_recv(0, 0, 1, 0x20, 1, mw.MW_F32)
    mw.mw_flush()  # in flight, not complete
    assert mw.mw_poll(h) == mw.MW_PENDING and ctx.mwt_attends() == 0
    ctx.mwt_want_attention()
    assert mw.mw_poll(h) == mw.MW_PENDING and ctx.mwt_attends() == 1
    assert mw.mw_poll(h) == mw.MW_PENDING and ctx.mwt_attends() == 1  # once is enough
    ctx.mwt_want_attention()
    ps = mw.PollSet([h])
    assert ps.poll() == 1 and ctx.mwt_attends() == 2  # mw_poll_many too
    ctx.mwt_want_attention()
    mw.mw_flush()
    assert ctx.mwt_attends() == 3
    ctx.mwt_complete(1, 0)
    assert mw.mw_poll(h) == mw.MW_DONE


def test_streams_are_deduplicated_and_none_is_skipped(ctx):
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [2, 3])
    mw.mw_send(0, 0, 1, 0x10, 1, mw.MW_F32, stream=0x111)
    mw.mw_recv(0, 0, 1, 0x20, 1, mw.MW_F32, stream=0x111)
    mw.mw_send(1, 0, 1, 0x30, 1, mw.MW_F32, stream=0x222)
    mw.mw_recv(1, 0, 1, 0x40, 1, mw.MW_F32, stream=mw.STREAM_NONE)
    mw.mw_flush()
    assert ctx.mwt_launch_streams(0) == 2
    ctx.mwt_complete(2, 0)


def test_many_worlds_lookup_is_by_key(ctx):
    # world ids are arbitrary integers; state is found by key, never by scanning or swapping
    ids = [7, -3, 1 << 30, 123456, 0]
    for i, w in enumerate(ids):
        mw.mw_world_create(w, [i, (i + 1) % 8])
    hs = []
    for w in ids:
        mw.mw_send(w, 0, 1, 0x100, 2, mw.MW_F32)
        hs.append(mw.mw_recv(w, 0, 1, 0x200, 2, mw.MW_F32))
    mw.mw_flush()
    assert ctx.mwt_launch_size(0) == 5 and sorted(log_entry(ctx, i)["world"] for i in range(5)) == sorted(
        w & 0xFFFFFFFF for w in ids)
    ctx.mwt_complete(5, 1)  # completion order is irrelevant
    assert [mw.mw_poll(h) for h in hs] == [mw.MW_DONE] * 5


def test_rooted_and_gathering_collectives_descriptors(ctx):
    mw.mw_world_create(0, [0, 1, 2])
    n, S = 3, 40
    # reduce: all ranks' buffers in rank order, root recorded
    h = [mw.mw_reduce_sum(0, r, 2, 0x100 * (r + 1), 10, mw.MW_F32) for r in (1, 2, 0)]
    # all-gather: sources in 0..n-1, destinations in 8..8+n-1
    h += [mw.mw_all_gather(0, r, 0x1000 + r, 0x2000 + 0x100 * r, 20, mw.MW_BF16) for r in range(n)]
    # gather to root 1 / scatter from root 0: NULL where the buffer is unused
    h += [mw.mw_gather(0, r, 1, 0x3000 + r, 0x4000 if r == 1 else None, 10, mw.MW_F32) for r in range(n)]
    h += [mw.mw_scatter(0, r, 0, 0x5000 if r == 0 else None, 0x6000 + 0x100 * r, 10, mw.MW_F32) for r in range(n)]
    mw.mw_flush()
    assert ctx.mwt_log_size() == 4 and ctx.mwt_launch_size(0) == 4
    red, ag, ga, sc = (log_entry(ctx, i) for i in range(4))
    assert (red["kind"], red["nbuf"], red["root"], red["buf"][:3], red["nbytes"]) == (3, 3, 2, [0x100, 0x200, 0x300], S)
    assert (ag["kind"], ag["buf"][:3], ag["buf_hi"][:3]) == (4, [0x1000, 0x1001, 0x1002], [0x2000, 0x2100, 0x2200])
    assert (ga["kind"], ga["root"], ga["buf"][:3], ga["buf_hi"][0], ga["nbytes"]) == (5, 1, [0x3000, 0x3001, 0x3002], 0x4000, S)
    assert (sc["kind"], sc["root"], sc["buf"][0], sc["buf_hi"][:3]) == (6, 0, 0x5000, [0x6000, 0x6100, 0x6200])
    ctx.mwt_complete(4, 0)
    assert [mw.mw_poll(x) for x in h] == [mw.MW_DONE] * 12
    # argument checks: the root needs its receive / send buffer; roots and kinds must agree
    with pytest.raises(mw.MwError) as e:
        mw.mw_gather(0, 1, 1, 0x3000, None, 10, mw.MW_F32)
    assert e.value.code == mw.MW_EINVAL
    with pytest.raises(mw.MwError) as e:
        mw.mw_scatter(0, 0, 0, None, 0x6000, 10, mw.MW_F32)
    assert e.value.code == mw.MW_EINVAL
    with pytest.raises(mw.MwError) as e:
        mw.mw_reduce_sum(0, 0, 3, 0x100, 10, mw.MW_F32)
    assert e.value.code == mw.MW_EINVAL
    a = mw.mw_reduce_sum(0, 0, 1, 0x100, 10, mw.MW_F32)
    b = mw.mw_reduce_sum(0, 1, 2, 0x200, 10, mw.MW_F32)
    c = mw.mw_allreduce_sum(0, 2, 0x300, 10, mw.MW_F32)
    assert [mw.mw_poll(x) for x in (a, b, c)] == [mw.MW_EMISMATCH] * 3
    # a one-rank world: gathering into place is nothing to do, otherwise it is a copy
    mw.mw_world_create(1, [5])
    assert mw.mw_poll(mw.mw_all_gather(1, 0, 0x7000, 0x7000, 4, mw.MW_F32)) == mw.MW_DONE
    hcopy = mw.mw_gather(1, 0, 0, 0x7000, 0x8000, 4, mw.MW_F32)
    assert mw.mw_poll(hcopy) == mw.MW_PENDING and log_entry(ctx, 4)["kind"] == 5
    ctx.mwt_complete(1, 0)
    assert mw.mw_poll(hcopy) == mw.MW_DONE


def test_post_many_mixed_batch(ctx):
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [2, 3])
    mw.mw_world_abort(1)
    handles, results = mw.mw_post_many([
        (mw.POST_SEND, 0, 0, 1, 0x10, 4, mw.MW_F32, mw.STREAM_NONE),
        (mw.POST_RECV, 0, 0, 1, 0x20, 4, mw.MW_F32, mw.STREAM_NONE),
        (mw.POST_SEND, 1, 0, 1, 0x10, 4, mw.MW_F32, mw.STREAM_NONE),          # broken world: refused
        (mw.POST_ALL_GATHER, 0, 0, 0, 0x30, 4, mw.MW_F32, mw.STREAM_NONE, 0x40),
        (mw.POST_ALL_GATHER, 0, 1, 0, 0x50, 4, mw.MW_F32, mw.STREAM_NONE, 0x60),
        (99, 0, 0, 1, 0x10, 4, mw.MW_F32, mw.STREAM_NONE),                      # unknown kind
    ])
    assert results == [0, 0, mw.MW_EBROKEN, 0, 0, mw.MW_EINVAL]
    assert handles[2] == 0 and handles[5] == 0 and all(handles[i] for i in (0, 1, 3, 4))
    mw.mw_flush()
    assert ctx.mwt_launch_size(0) == 2
    ctx.mwt_complete(2, 0)
    assert [mw.mw_poll(handles[i]) for i in (0, 1, 3, 4)] == [mw.MW_DONE] * 4


def test_per_operation_host_cost_does_not_grow_with_the_number_of_worlds(hostlib):
    """Per-world state is looked up by key, never swapped in and out (Sec. 3.2 "State management for multiple
    worlds"): the host cost of post + match + launch + completion + poll per message must stay flat from
    4 worlds to 1000 worlds."""
    import time

    def cost(n_worlds, msgs=20000):
        mw.mw_init(0, 2 * n_worlds)
        try:
            for w in range(n_worlds):
                mw.mw_world_create(w, [2 * w, 2 * w + 1])
            batch = 50
            pbs = []
            for lo in range(0, min(n_worlds * 4, 400), batch):  # messages spread round-robin over the worlds
                posts = []
                for k in range(lo, lo + batch):
                    w = k % n_worlds
                    posts.append((mw.POST_SEND, w, 0, 1, 0x1000, 8, mw.MW_F32, mw.STREAM_NONE))
                    posts.append((mw.POST_RECV, w, 0, 1, 0x2000, 8, mw.MW_F32, mw.STREAM_NONE))
                pbs.append(mw.PostBatch(posts))
            best = 1e9
            for rep in range(3):
                t0 = time.perf_counter()
                done = 0
                while done < msgs:
                    for pb in pbs:
                        pb.post()
                        mw.mw_flush()
                        hostlib.mwt_complete(batch, 0)
                        ps = mw.PollSet(list(pb.handles))
                        assert ps.poll() == 0
                        done += batch
                best = min(best, (time.perf_counter() - t0) / done)
            return best
        finally:
            mw.mw_shutdown()

    few, many = cost(4), cost(1000)
    assert many < 1.6 * few, f"{few * 1e9:.0f} ns per message with 4 worlds, {many * 1e9:.0f} ns with 1000"


def test_worlds_a_worker_has_left_cost_nothing_later(hostlib):
    """Elastic recovery (Sec. 3.1): a worker rejoins through new worlds again and again.  Aborting the worker
    after 20 000 such generations must cost what it costs after 20."""
    import time

    mw.mw_config_set("max_rings", 8)
    mw.mw_init(0, 4)
    try:
        def generation(first_id, n):
            t0 = time.perf_counter()
            for i in range(n):
                mw.mw_world_create(first_id + i, [0, 1])
                h = mw.mw_recv(first_id + i, 0, 1, 0x1000, 8, mw.MW_F32, mw.STREAM_NONE)
                mw.mw_worker_abort(1)
                assert mw.mw_poll(h) == mw.MW_BROKEN
                assert mw.mw_world_state(first_id + i) == mw.MW_BROKEN
            return (time.perf_counter() - t0) / n

        early = min(generation(200 * k, 200) for k in range(3))  # best of three: robust on a busy host
        generation(1000, 20000)
        late = min(generation(100000 + 200 * k, 200) for k in range(3))
        assert late < 3 * early, f"{early * 1e6:.1f} us per generation at first, {late * 1e6:.1f} us after 20 000"
    finally:
        mw.mw_shutdown()
        mw.mw_config_set("max_rings", 1024)
