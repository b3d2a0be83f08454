"""Host side of the entry point that allocates nothing, on the CPU with the device test double: the matching of
whole operations inside one array follows the same rules as the posting calls, and what it hands to the device is
what the posting calls would have handed over."""

import ctypes as C

import pytest

from paper_2407_08980_amd import binding as mw

from helpers import hostcheck_library


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
    mw.mw_init(0, 12)
    yield hostlib
    mw.mw_shutdown()


def entries(lib, first=0):
    out = []
    for i in range(first, lib.mwt_log_size()):
        e = (C.c_uint64 * 26)()
        assert lib.mwt_log_entry(i, e) == 0
        out.append(dict(buf=list(e[:8]), nbytes=e[8], kind=e[9], dtype=e[10], nbuf=e[11], slot=e[12], gen=e[13],
                        world=e[14], launch=e[16], root=e[17], buf_hi=list(e[18:26])))
    return out


def strip(e):
    return {k: v for k, v in e.items() if k not in ("slot", "gen", "launch")}


def test_whole_operations_are_matched_like_posted_ones(ctx):
    """The same array through mw_post_many (+ flush) and through the variant: the operations handed to the
    device are the same (buffers, sizes, kinds, roots), in both cases."""
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [2, 3, 4])
    F, B = mw.MW_F32, mw.MW_BF16
    posts = [
        (mw.POST_RECV, 0, 0, 1, 0x1000, 10, F, 0), (mw.POST_RECV, 0, 0, 1, 0x2000, 20, F, 0),
        (mw.POST_SEND, 0, 0, 1, 0x3000, 10, F, 0), (mw.POST_SEND, 0, 1, 0, 0x4000, 5, B, 0),
        (mw.POST_SEND, 0, 0, 1, 0x5000, 20, F, 0), (mw.POST_RECV, 0, 1, 0, 0x6000, 5, B, 0),
        (mw.POST_BROADCAST, 1, 2, 1, 0x7000, 8, F, 0), (mw.POST_ALLREDUCE_SUM, 1, 0, 0, 0x8000, 6, B, 0),
        (mw.POST_BROADCAST, 1, 0, 1, 0x9000, 8, F, 0), (mw.POST_BROADCAST, 1, 1, 1, 0xA000, 8, F, 0),
        (mw.POST_ALLREDUCE_SUM, 1, 2, 0, 0xB000, 6, B, 0), (mw.POST_ALLREDUCE_SUM, 1, 1, 0, 0xC000, 6, B, 0),
        (mw.POST_GATHER, 1, 0, 2, 0xD000, 4, F, 0, None), (mw.POST_GATHER, 1, 1, 2, 0xD100, 4, F, 0, None),
        (mw.POST_GATHER, 1, 2, 2, 0xD200, 4, F, 0, 0xE000),
    ]
    # rank 0 of world 1 posts all-reduce before broadcast, the others the other way round: a disagreement in
    # the first collective for the posting calls -- use an array every rank agrees on instead
    posts[7], posts[8] = posts[8], posts[7]
    assert mw.mw_post_many_noalloc(posts, 0x77) == mw.MW_OK
    static = entries(ctx)
    assert ctx.mwt_launch_count() == 1 and [e["slot"] for e in static] == list(range(6))
    assert len({e["gen"] for e in static}) == 1 and static[0]["gen"] != 0
    assert mw.mw_pending_ops() == 0  # nothing of the context's queues was touched
    handles, results = mw.mw_post_many(posts)
    assert all(r == 0 for r in results)
    mw.mw_flush()
    posted = entries(ctx, len(static))
    key = lambda e: (e["world"], e["kind"], e["buf"][0])
    assert sorted(map(strip, static), key=key) == sorted(map(strip, posted), key=key)
    # first in, first out per pair: 0x3000 -> 0x1000 and 0x5000 -> 0x2000
    copies = sorted((e["buf"][0], e["buf"][1], e["nbytes"]) for e in static if e["kind"] == 0)
    assert copies == [(0x3000, 0x1000, 40), (0x4000, 0x6000, 10), (0x5000, 0x2000, 80)]
    ctx.mwt_complete(10, 0)
    # a second call gets a new generation and starts at slot 0 again
    assert mw.mw_post_many_noalloc(posts[:6], 0x77) == mw.MW_OK
    again = entries(ctx, len(static) + len(posted))
    assert [e["slot"] for e in again] == [0, 1, 2] and again[0]["gen"] == static[0]["gen"] + 1


def test_refusals_enqueue_nothing(ctx):
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [2, 3, 4])
    F = mw.MW_F32
    n0 = ctx.mwt_log_size()
    bad = [
        ([(mw.POST_SEND, 0, 0, 1, 0x10, 4, F, 0)], mw.MW_EINVAL),  # no peer
        ([(mw.POST_SEND, 0, 0, 1, 0x10, 4, F, 0), (mw.POST_RECV, 0, 0, 1, 0x20, 5, F, 0)], mw.MW_EMISMATCH),
        ([(mw.POST_SEND, 0, 0, 0, 0x10, 4, F, 0), (mw.POST_RECV, 0, 0, 0, 0x20, 4, F, 0)], mw.MW_EINVAL),  # src == dst
        ([(mw.POST_SEND, 0, 0, 2, 0x10, 4, F, 0), (mw.POST_RECV, 0, 0, 2, 0x20, 4, F, 0)], mw.MW_EINVAL),  # rank out of range
        ([(mw.POST_SEND, 5, 0, 1, 0x10, 4, F, 0)], mw.MW_ENOWORLD),
        ([(mw.POST_BROADCAST, 1, 0, 0, 0x10, 4, F, 0), (mw.POST_BROADCAST, 1, 1, 0, 0x20, 4, F, 0)], mw.MW_EINVAL),  # rank 2 missing
        ([(mw.POST_BROADCAST, 1, r, r % 2, 0x10 * (r + 1), 4, F, 0) for r in range(3)], mw.MW_EMISMATCH),  # roots differ
        ([(mw.POST_ALLREDUCE_SUM, 1, r, 0, 0x10 * (r + 1) + 2, 4, F, 0) for r in range(3)], mw.MW_EINVAL),  # misaligned elements
        ([(mw.POST_SEND, 0, 0, 1, 0, 4, F, 0), (mw.POST_RECV, 0, 0, 1, 0x20, 4, F, 0)], mw.MW_EINVAL),  # NULL buffer
    ]
    for posts, want in bad:
        assert mw.mw_post_many_noalloc(posts, 0) == want, posts
    assert mw.mw_post_many_noalloc([(mw.POST_SEND, 0, 0, 1, 0x10, 4, F, 0), (mw.POST_RECV, 0, 0, 1, 0x20, 4, F, 0)],
                                   mw.STREAM_NONE) == mw.MW_EINVAL
    assert ctx.mwt_log_size() == n0 and ctx.mwt_launch_count() == 0
    # empty operations are complete without a launch entry; 64 operations fit, 65 do not
    zero = [(mw.POST_SEND, 0, 0, 1, 0, 0, F, 0), (mw.POST_RECV, 0, 0, 1, 0, 0, F, 0)]
    assert mw.mw_post_many_noalloc(zero, 0) == mw.MW_OK and ctx.mwt_log_size() == n0
    pair = [(mw.POST_SEND, 0, 0, 1, 0x10, 4, F, 0), (mw.POST_RECV, 0, 0, 1, 0x20, 4, F, 0)]
    assert mw.mw_post_many_noalloc(pair * 64, 0) == mw.MW_OK and ctx.mwt_log_size() == n0 + 64
    assert mw.mw_post_many_noalloc(pair * 65, 0) == mw.MW_EINVAL
    mw.mw_world_abort(0)
    assert mw.mw_post_many_noalloc(pair, 0) == mw.MW_EBROKEN
