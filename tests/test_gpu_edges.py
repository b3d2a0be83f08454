"""Edge cases of the GPU path, through the C ABI, against the CPU oracle's per-operation
functions: alignment, empty and huge messages, world sizes up to the collective limit,
non-finite values, early completion, stream ordering, non-blocking polls, ring isolation.
"""

import struct
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle


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


def dev_bytes(torch, arr, offset=0, pad=64):
    """Upload bytes to a fresh device buffer at `offset` bytes past a 256-byte aligned base."""
    base = torch.full((offset + arr.size + pad,), 0x5A, dtype=torch.uint8, device="cuda")
    view = base[offset:offset + arr.size]
    view.copy_(torch.from_numpy(arr))
    return base, view


def served_as_configured(mw):
    """With the mailbox on, flushes of this test went through the queue; with it off, none did."""
    epoch, _, tail = mw.mw_debug_mailbox()
    if mw.mw_config_get("mailbox"):
        assert epoch >= 1 and tail >= 1
    else:
        assert (epoch, tail) == (0, 0)


def rand_bytes(n, seed):
    return np.random.default_rng(seed).integers(0, 256, size=n, dtype=np.uint8)


@pytest.mark.parametrize("soff,doff", [(0, 0), (1, 3), (2, 6), (4, 12), (8, 8), (16, 1), (3, 3)])
def test_copy_any_alignment_and_ragged_sizes(torch, mw, soff, doff):
    mw.mw_world_create(0, [0, 1])
    for i, nbytes in enumerate([2, 30, 4094, 65538, 300002, 1048578 + 14]):
        src = rand_bytes(nbytes, 100 + i)
        sbase, sview = dev_bytes(torch, src, soff)
        dbase, dview = dev_bytes(torch, np.full(nbytes, 0xA5, np.uint8), doff)
        hs = mw.mw_send(0, 0, 1, sview.data_ptr(), nbytes // 2, mw.MW_BF16)
        hr = mw.mw_recv(0, 0, 1, dview.data_ptr(), nbytes // 2, mw.MW_BF16)
        assert wait(mw, [hs, hr]) == [mw.MW_DONE] * 2
        got = dbase.cpu().numpy()
        assert np.array_equal(got[doff:doff + nbytes], oracle.copy_result(src))
        assert np.all(got[:doff] == 0x5A) and np.all(got[doff + nbytes:] == 0x5A)  # nothing outside is touched
        assert np.array_equal(sview.cpu().numpy(), src)
    served_as_configured(mw)


@pytest.mark.parametrize("n", [2, 3, 5, 8])
def test_broadcast_every_root_up_to_eight_ranks(torch, mw, n):
    mw.mw_world_create(n, list(range(n)))
    count = 70001
    for root in range(n):
        host = [rand_bytes(count * 4, 1000 * n + 10 * root + r) for r in range(n)]
        dev = [dev_bytes(torch, host[r], offset=(r % 3) * 4) for r in range(n)]
        order = list(range(n))[::-1]
        hs = [mw.mw_broadcast(n, r, root, dev[r][1].data_ptr(), count, mw.MW_F32) for r in order]
        assert wait(mw, hs) == [mw.MW_DONE] * n
        want = oracle.broadcast_result(host, root)
        for r in range(n):
            assert np.array_equal(dev[r][1].cpu().numpy(), want[r]), (root, r)
    served_as_configured(mw)


@pytest.mark.parametrize("lds", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [2, 3, 4, 7, 8])
def test_allreduce_world_sizes_alignment_and_tails(torch, mw, n, dtype, lds):
    mw.mw_config_set("reduce_lds", lds)
    try:
        mw.mw_world_create(0, list(range(n)))
        isz = 4 if dtype == "f32" else 2
        for count, off_elems in [(1, 0), (7, 0), (4099, 0), (65536 + 5, 1), (300000, 3)]:
            rng = np.random.default_rng(n * 100 + count)
            xs = [rng.uniform(-1, 1, count).astype(np.float32) for _ in range(n)]
            host = [x.view(np.uint8) if dtype == "f32" else oracle.f32_to_bf16_bits(x).view(np.uint8) for x in xs]
            dev = [dev_bytes(torch, host[r], offset=off_elems * isz) for r in range(n)]
            hs = [mw.mw_allreduce_sum(0, r, dev[r][1].data_ptr(), count, mw.DTYPES[dtype]) for r in range(n)]
            assert wait(mw, hs) == [mw.MW_DONE] * n
            s, sabs = oracle.allreduce_sum_f64(host, count, dtype)
            ordered = oracle.allreduce_sum_ordered(host, count, dtype)
            for r in range(n):
                got = dev[r][1].cpu().numpy()
                ok, worst = oracle.allreduce_within_tolerance(got, s, sabs, count, dtype)
                assert ok, (n, dtype, count, r, worst)
                assert np.array_equal(got, ordered), (n, dtype, count, r)  # fixed order: bit-exact, same on all ranks
                base = dev[r][0].cpu().numpy()
                assert np.all(base[: off_elems * isz] == 0x5A) and np.all(base[off_elems * isz + count * isz:] == 0x5A)
        served_as_configured(mw)
    finally:
        mw.mw_config_set("reduce_lds", 0)


def test_allreduce_exact_cases(torch, mw):
    mw.mw_world_create(0, [0, 1, 2, 3])
    mw.mw_world_create(1, [0, 1])
    rng = np.random.default_rng(5)
    # integer-valued inputs: the sum is exact in every precision
    for dtype in ("f32", "bf16"):
        ints = [rng.integers(-16, 17, size=10007) for _ in range(4)]
        host = [(v.astype(np.float32).view(np.uint8) if dtype == "f32" else
                 oracle.f32_to_bf16_bits(v.astype(np.float32)).view(np.uint8)) for v in ints]
        dev = [dev_bytes(torch, h) for h in host]
        hs = [mw.mw_allreduce_sum(0, r, dev[r][1].data_ptr(), 10007, mw.DTYPES[dtype]) for r in range(4)]
        assert wait(mw, hs) == [mw.MW_DONE] * 4
        got = dev[2][1].cpu().numpy()
        vals = got.view(np.float32) if dtype == "f32" else oracle.bf16_bits_to_f32(got.view(np.uint16))
        assert np.array_equal(vals.astype(np.int64), sum(ints))
    # x + (-x) = +0, bit pattern zero
    x = rng.standard_normal(5000).astype(np.float32)
    dev = [dev_bytes(torch, x.view(np.uint8)), dev_bytes(torch, (-x).view(np.uint8))]
    hs = [mw.mw_allreduce_sum(1, r, dev[r][1].data_ptr(), 5000, mw.MW_F32) for r in range(2)]
    assert wait(mw, hs) == [mw.MW_DONE] * 2
    assert not dev[0][1].cpu().numpy().any() and not dev[1][1].cpu().numpy().any()
    # two fp32 ranks: the correctly rounded sum
    a = (rng.standard_normal(9000) * 10.0 ** rng.integers(-3, 4, 9000)).astype(np.float32)
    b = (rng.standard_normal(9000) * 10.0 ** rng.integers(-3, 4, 9000)).astype(np.float32)
    dev = [dev_bytes(torch, a.view(np.uint8)), dev_bytes(torch, b.view(np.uint8))]
    hs = [mw.mw_allreduce_sum(1, r, dev[r][1].data_ptr(), 9000, mw.MW_F32) for r in range(2)]
    assert wait(mw, hs) == [mw.MW_DONE] * 2
    assert np.array_equal(dev[0][1].cpu().numpy().view(np.float32), a + b)


def test_allreduce_non_finite_values(torch, mw):
    mw.mw_world_create(0, [0, 1, 2])
    for dtype in ("f32", "bf16"):
        x = [np.array([1.0, np.inf, -np.inf, np.nan, np.inf, 2.0, -0.0, 1e-40], np.float32),
             np.array([2.0, 1.0, -1.0, 1.0, -np.inf, np.nan, -0.0, 1e-40], np.float32),
             np.array([3.0, 1.0, -1.0, 1.0, 1.0, 1.0, -0.0, 1e-40], np.float32)]
        host = [v.view(np.uint8) if dtype == "f32" else oracle.f32_to_bf16_bits(v).view(np.uint8) for v in x]
        dev = [dev_bytes(torch, h) for h in host]
        hs = [mw.mw_allreduce_sum(0, r, dev[r][1].data_ptr(), 8, mw.DTYPES[dtype]) for r in range(3)]
        assert wait(mw, hs) == [mw.MW_DONE] * 3
        with np.errstate(invalid="ignore"):
            s, _ = oracle.allreduce_sum_f64(host, 8, dtype)
        got = dev[1][1].cpu().numpy()
        y = got.view(np.float32) if dtype == "f32" else oracle.bf16_bits_to_f32(got.view(np.uint16))
        assert np.array_equal(np.isnan(y), np.isnan(s)) and list(np.isnan(s)) == [False, False, False, True, True, True, False, False]
        assert y[0] == 6.0 and y[1] == np.inf and y[2] == -np.inf
        assert y[6] == 0.0 and np.signbit(y[6])  # (-0) + (-0) + (-0) = -0
        # everything that is not NaN (whose sign and payload IEEE leaves open) is bit-exact, denormals included
        with np.errstate(invalid="ignore"):
            want = oracle.allreduce_sum_ordered(host, 8, dtype)
        isz = 4 if dtype == "f32" else 2
        keep = np.repeat(~np.isnan(s), isz)
        assert np.array_equal(got[keep], want[keep])


def test_empty_and_single_rank_operations(torch, mw):
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [3])
    buf = torch.full((64,), 7, dtype=torch.uint8, device="cuda")
    hs = [mw.mw_send(0, 0, 1, 0, 0, mw.MW_F32), mw.mw_recv(0, 0, 1, 0, 0, mw.MW_F32)]
    hs += [mw.mw_allreduce_sum(0, r, buf.data_ptr(), 0, mw.MW_BF16) for r in range(2)]
    hs += [mw.mw_allreduce_sum(1, 0, buf.data_ptr(), 16, mw.MW_F32), mw.mw_broadcast(1, 0, 0, buf.data_ptr(), 16, mw.MW_F32)]
    assert [mw.mw_poll(h) for h in hs] == [mw.MW_DONE] * 6
    assert mw.mw_pending_ops() == 0 and bool((buf == 7).all())
    hs = [mw.mw_send(0, 0, 1, buf.data_ptr(), 4, mw.MW_F32), mw.mw_recv(0, 0, 1, buf.data_ptr(), 5, mw.MW_F32)]
    assert [mw.mw_poll(h) for h in hs] == [mw.MW_EMISMATCH] * 2


def test_message_larger_than_4GiB(torch, mw):
    """64-bit offsets: one 4.5 GiB message; the whole destination is compared on the device and
    windows around the start, the 4 GiB boundary and the ragged end against the oracle."""
    mw.mw_world_create(0, [0, 1])
    nbytes = (9 << 29) + 6
    g = torch.Generator(device="cuda")
    g.manual_seed(1234)
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
    dst = torch.full((nbytes + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    hs = [mw.mw_send(0, 0, 1, src.data_ptr(), nbytes // 2, mw.MW_BF16), mw.mw_recv(0, 0, 1, dst.data_ptr(), nbytes // 2, mw.MW_BF16)]
    assert wait(mw, hs, timeout=120) == [mw.MW_DONE] * 2
    assert torch.equal(dst[:nbytes], src) and bool((dst[nbytes:] == 0xA5).all())
    for lo in (0, (1 << 32) - 4096, (1 << 32), nbytes - 70001):
        hi = min(lo + 70001, nbytes)
        assert np.array_equal(dst[lo:hi].cpu().numpy(), oracle.copy_result(src[lo:hi].cpu().numpy()))


def test_many_operations_in_one_flush(torch, mw):
    """More operations than one launch's argument block holds: the flush splits into several launches."""
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [1, 2, 3])
    n = 60
    src = [rand_bytes(4000 + 2 * i, i) for i in range(n)]
    sdev = [dev_bytes(torch, s) for s in src]
    ddev = [dev_bytes(torch, np.full(s.size, 0xA5, np.uint8)) for s in src]
    hs = []
    for i in range(n):
        hs.append(mw.mw_send(0, 0, 1, sdev[i][1].data_ptr(), src[i].size // 2, mw.MW_BF16))
        hs.append(mw.mw_recv(0, 0, 1, ddev[i][1].data_ptr(), src[i].size // 2, mw.MW_BF16))
    xs = [[np.random.default_rng(1000 + 3 * i + r).uniform(-1, 1, 999).astype(np.float32) for r in range(3)] for i in range(n)]
    xdev = [[dev_bytes(torch, x.view(np.uint8)) for x in row] for row in xs]
    for i in range(n):
        for r in range(3):
            hs.append(mw.mw_allreduce_sum(1, r, xdev[i][r][1].data_ptr(), 999, mw.MW_F32))
    assert mw.mw_pending_ops() == 2 * n
    assert wait(mw, hs) == [mw.MW_DONE] * len(hs)
    for i in range(n):
        assert np.array_equal(ddev[i][1].cpu().numpy(), src[i])
        want = oracle.allreduce_sum_ordered([x.view(np.uint8) for x in xs[i]], 999, "f32")
        assert np.array_equal(xdev[i][0][1].cpu().numpy(), want)


def test_more_outstanding_operations_than_ring_slots(torch, mw):
    """One world's ring has 128 slots; 300 messages are posted before the first poll.  The ones that find no slot
    wait on the host until earlier ones retire; all of them arrive, in order, byte for byte."""
    mw.mw_world_create(0, [0, 1])
    n, size = 300, 2048
    src = np.stack([rand_bytes(size, 5000 + k) for k in range(n)])
    src[:, 0] = np.arange(n) % 251  # a stamp: the k-th receive must hold the k-th send
    sdev = torch.from_numpy(src).cuda()
    ddev = torch.full((n, size), 0xA5, dtype=torch.uint8, device="cuda")
    hs = []
    for k in range(n):  # all sends first, then all receives: matching is FIFO per (world, src, dst)
        hs.append(mw.mw_send(0, 0, 1, sdev[k].data_ptr(), size // 4, mw.MW_F32))
    for k in range(n):
        hs.append(mw.mw_recv(0, 0, 1, ddev[k].data_ptr(), size // 4, mw.MW_F32))
    assert mw.mw_pending_ops() == n
    mw.mw_flush()
    assert mw.mw_pending_ops() == n  # 128 in flight, the rest queued: nothing is complete before a poll sees it
    assert wait(mw, hs) == [mw.MW_DONE] * len(hs)
    got = ddev.cpu().numpy()
    for k in range(n):
        assert np.array_equal(got[k], oracle.copy_result(src[k])), k
    assert mw.mw_pending_ops() == 0


def test_early_completion_is_visible(torch, mw):
    """A small message batched with large ones is reported complete while the launch is still
    running; its bytes must be readable (here: by a DMA copy to the host) at that moment."""
    for w in range(8):
        mw.mw_world_create(w, [2 * w, 2 * w + 1])
    big = 256 << 20
    bsrc = [torch.full((big,), w + 1, dtype=torch.uint8, device="cuda") for w in range(1, 8)]
    bdst = [torch.zeros(big, dtype=torch.uint8, device="cuda") for _ in range(1, 8)]
    early = 0
    for it, small in enumerate([4096, 65536, 1 << 20, 4 << 20, 32 << 20, 65536, 1 << 20, 4 << 20]):
        src = rand_bytes(small, 500 + it)
        sbase, sview = dev_bytes(torch, src)
        dbase, dview = dev_bytes(torch, np.full(small, 0xA5, np.uint8))
        torch.cuda.synchronize()
        hsmall = [mw.mw_send(0, 0, 1, sview.data_ptr(), small // 4, mw.MW_F32), mw.mw_recv(0, 0, 1, dview.data_ptr(), small // 4, mw.MW_F32)]
        hbig = []
        for w in range(1, 8):
            hbig.append(mw.mw_send(w, 0, 1, bsrc[w - 1].data_ptr(), big // 4, mw.MW_F32))
            hbig.append(mw.mw_recv(w, 0, 1, bdst[w - 1].data_ptr(), big // 4, mw.MW_F32))
        mw.mw_flush()
        t0 = time.time()
        while mw.mw_poll(hsmall[1]) != mw.MW_DONE:
            assert time.time() - t0 < 30
        got = dview.cpu().numpy()  # right away
        early += any(mw.mw_poll(h) == mw.MW_PENDING for h in hbig)
        assert np.array_equal(got, oracle.copy_result(src)), f"stale bytes in a {small}-byte message"
        assert wait(mw, hbig) == [mw.MW_DONE] * 14
        for w in range(1, 8):
            assert bool((bdst[w - 1] == w + 1).all())
            bdst[w - 1].zero_()
    assert early >= 1, "the small message never completed ahead of the large ones"


@pytest.mark.parametrize("soff,doff", [(1, 1), (2, 6), (4, 12), (8, 8), (3, 0)])
def test_early_completion_is_visible_for_every_store_width(torch, mw, soff, doff):
    """The same for buffers that are not 16-byte aligned: their chunks are moved with 8-, 16-, 32- or 64-bit
    accesses, whose stores must be as visible at completion as the 128-bit ones."""
    for w in range(8):
        mw.mw_world_create(w, [2 * w, 2 * w + 1])
    big = 256 << 20
    bsrc = [torch.full((big,), w + 1, dtype=torch.uint8, device="cuda") for w in range(1, 8)]
    bdst = [torch.zeros(big, dtype=torch.uint8, device="cuda") for _ in range(1, 8)]
    early = 0
    for it, small in enumerate([4096 + 2, 65536 + 6, (1 << 20) + 10, 300002]):
        src = rand_bytes(small, 700 + it)
        sbase, sview = dev_bytes(torch, src, soff)
        dbase, dview = dev_bytes(torch, np.full(small, 0xA5, np.uint8), doff)
        torch.cuda.synchronize()
        hsmall = [mw.mw_send(0, 0, 1, sview.data_ptr(), small // 2, mw.MW_BF16), mw.mw_recv(0, 0, 1, dview.data_ptr(), small // 2, mw.MW_BF16)]
        hbig = []
        for w in range(1, 8):
            hbig.append(mw.mw_send(w, 0, 1, bsrc[w - 1].data_ptr(), big // 4, mw.MW_F32))
            hbig.append(mw.mw_recv(w, 0, 1, bdst[w - 1].data_ptr(), big // 4, mw.MW_F32))
        mw.mw_flush()
        t0 = time.time()
        while mw.mw_poll(hsmall[1]) != mw.MW_DONE:
            assert time.time() - t0 < 30
        got = dbase.cpu().numpy()  # right away
        early += any(mw.mw_poll(h) == mw.MW_PENDING for h in hbig)
        assert np.array_equal(got[doff:doff + small], oracle.copy_result(src)), f"stale bytes in a {small}-byte message"
        assert np.all(got[:doff] == 0x5A) and np.all(got[doff + small:] == 0x5A)
        assert wait(mw, hbig) == [mw.MW_DONE] * 14
    assert early >= 1, "the small message never completed ahead of the large ones"


@pytest.mark.parametrize("n", [2, 4])
def test_early_completion_is_visible_after_a_broadcast(torch, mw, n):
    """A small broadcast batched with seven large ones in the same fan-out launch."""
    for w in range(8):
        mw.mw_world_create(w, list(range(n)))
    big = 128 << 20
    bbuf = [[torch.full((big,), (w + 1) * (r == 0), dtype=torch.uint8, device="cuda") for r in range(n)] for w in range(1, 8)]
    early = 0
    for it, (small, off) in enumerate([(4096, 0), (65536 + 4, 4), (1 << 20, 0), (4 << 20, 2), (300001 * 4, 1)]):
        root = it % n
        host = [rand_bytes(small, 800 + 10 * it + r) for r in range(n)]
        dev = [dev_bytes(torch, host[r], off) for r in range(n)]
        torch.cuda.synchronize()
        hsmall = [mw.mw_broadcast(0, r, root, dev[r][1].data_ptr(), small // 4, mw.MW_F32) for r in range(n)]
        hbig = [mw.mw_broadcast(w, r, 0, bbuf[w - 1][r].data_ptr(), big // 4, mw.MW_F32) for w in range(1, 8) for r in range(n)]
        mw.mw_flush()
        t0 = time.time()
        while mw.mw_poll(hsmall[0]) != mw.MW_DONE:
            assert time.time() - t0 < 30
        got = [dev[r][0].cpu().numpy() for r in range(n)]  # right away
        early += any(mw.mw_poll(h) == mw.MW_PENDING for h in hbig)
        want = oracle.broadcast_result(host, root)
        for r in range(n):
            assert np.array_equal(got[r][off:off + small], want[r]), f"stale bytes on rank {r} of a {small}-byte broadcast"
        assert wait(mw, hbig) == [mw.MW_DONE] * (7 * n)
        for w in range(1, 8):
            for r in range(1, n):
                assert bool((bbuf[w - 1][r] == w + 1).all())
                bbuf[w - 1][r].zero_()
    assert early >= 1, "the small broadcast never completed ahead of the large ones"


@pytest.mark.parametrize("lds", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_early_completion_is_visible_after_an_allreduce(torch, mw, dtype, lds):
    """A small in-place all-reduce batched with seven large ones in the same launch, register and LDS-staged
    kernels: every rank's sum must be readable the moment the operation is reported complete."""
    mw.mw_config_set("reduce_lds", lds)
    try:
        n = 3
        for w in range(8):
            mw.mw_world_create(w, list(range(n)))
        isz = 4 if dtype == "f32" else 2
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        big = (96 << 20) // isz
        bbuf = [[torch.full((big,), float(r + 1), dtype=tdt, device="cuda") for r in range(n)] for _ in range(1, 8)]
        early = 0
        for it, (count, off_elems) in enumerate([(1024, 0), (16384 + 3, 1), (262144, 0), (1 << 20, 3), (300001, 2)]):
            rng = np.random.default_rng(900 + it)
            xs = [rng.uniform(-1, 1, count).astype(np.float32) for _ in range(n)]
            host = [x.view(np.uint8) if dtype == "f32" else oracle.f32_to_bf16_bits(x).view(np.uint8) for x in xs]
            dev = [dev_bytes(torch, host[r], offset=off_elems * isz) for r in range(n)]
            torch.cuda.synchronize()
            hsmall = [mw.mw_allreduce_sum(0, r, dev[r][1].data_ptr(), count, mw.DTYPES[dtype]) for r in range(n)]
            hbig = [mw.mw_allreduce_sum(w, r, bbuf[w - 1][r].data_ptr(), big, mw.DTYPES[dtype]) for w in range(1, 8) for r in range(n)]
            mw.mw_flush()
            t0 = time.time()
            while mw.mw_poll(hsmall[0]) != mw.MW_DONE:
                assert time.time() - t0 < 30
            got = [dev[r][1].cpu().numpy() for r in range(n)]  # right away
            early += any(mw.mw_poll(h) == mw.MW_PENDING for h in hbig)
            s, sabs = oracle.allreduce_sum_f64(host, count, dtype)
            ordered = oracle.allreduce_sum_ordered(host, count, dtype)
            for r in range(n):
                ok, worst = oracle.allreduce_within_tolerance(got[r], s, sabs, count, dtype)
                assert ok, (dtype, lds, count, r, worst)
                assert np.array_equal(got[r], ordered), f"stale bytes on rank {r} of a {count}-element all-reduce"
            assert wait(mw, hbig) == [mw.MW_DONE] * (7 * n)
            for w in range(1, 8):
                for r in range(n):
                    assert bool((bbuf[w - 1][r] == 6.0).all())  # 1 + 2 + 3, exact in both types
                    bbuf[w - 1][r].fill_(float(r + 1))
        assert early >= 1, "the small all-reduce never completed ahead of the large ones"
    finally:
        mw.mw_config_set("reduce_lds", 0)


def test_a_busy_or_stuck_producer_stream_holds_up_only_its_own_operations(torch, mw):
    """World A's send is ordered after a long queue of producer kernels on A's stream; world B posts buffers that
    are final, in the same flush.  B must complete while A is still waiting for its producer (Sec. 3.2: a pending
    operation in one world must not hold up another), and later flushes of B must not queue behind A either."""
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [2, 3])
    n = 1 << 30
    a_src = torch.zeros(n, dtype=torch.uint8, device="cuda")
    a_dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    nb = 1 << 20
    b_host = [rand_bytes(nb, 40 + k) for k in range(3)]
    b_src = [dev_bytes(torch, h) for h in b_host]
    b_dst = [dev_bytes(torch, np.full(nb, 0xA5, np.uint8)) for _ in range(3)]
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        for k in range(1, 121):  # ~0.3 ms each: the producer is busy for tens of milliseconds
            a_src.fill_(k % 251)
    ha = [mw.mw_send(0, 0, 1, a_src.data_ptr(), n // 4, mw.MW_F32, s.cuda_stream),
          mw.mw_recv(0, 0, 1, a_dst.data_ptr(), n // 4, mw.MW_F32, mw.STREAM_NONE)]
    a_pending_seen = 0
    for k in range(3):  # the first shares A's flush, the others come in flushes of their own
        hb = [mw.mw_send(1, 0, 1, b_src[k][1].data_ptr(), nb // 4, mw.MW_F32, mw.STREAM_NONE),
              mw.mw_recv(1, 0, 1, b_dst[k][1].data_ptr(), nb // 4, mw.MW_F32, mw.STREAM_NONE)]
        mw.mw_flush()
        t0 = time.time()
        while mw.mw_poll(hb[1]) != mw.MW_DONE:
            assert time.time() - t0 < 30
        a_pending_seen += mw.mw_poll(ha[1]) == mw.MW_PENDING
        assert np.array_equal(b_dst[k][1].cpu().numpy(), oracle.copy_result(b_host[k]))
    assert a_pending_seen == 3, "world B's transfers should all have completed while world A waited for its producer"
    assert wait(mw, ha) == [mw.MW_DONE] * 2
    assert bool((a_dst == 120 % 251).all())  # ordered after the LAST producer kernel


def test_post_is_ordered_after_the_callers_stream(torch, mw):
    mw.mw_world_create(0, [0, 1])
    n = 64 << 20
    s = torch.cuda.Stream()
    src = torch.zeros(n, dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        for k in range(1, 41):  # a queue of producer kernels; the last one writes the final value
            src.fill_(k)
        hs = [mw.mw_send(0, 0, 1, src.data_ptr(), n // 4, mw.MW_F32, s.cuda_stream),
              mw.mw_recv(0, 0, 1, dst.data_ptr(), n // 4, mw.MW_F32, mw.STREAM_NONE)]
    assert wait(mw, hs) == [mw.MW_DONE] * 2
    assert bool((dst == 40).all())


def test_pending_operation_never_blocks_other_worlds_or_polls(torch, mw):
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [0, 2])
    lonely_buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    stuck = mw.mw_recv(0, 1, 0, lonely_buf.data_ptr(), 1024, mw.MW_F32)  # its sender never shows up
    src = torch.arange(0, 8192, dtype=torch.int32, device="cuda")
    dst = torch.zeros(8192, dtype=torch.int32, device="cuda")
    worst = 0.0
    for k in range(1000):
        hs = [mw.mw_recv(1, 1, 0, dst.data_ptr(), 8192, mw.MW_F32), mw.mw_send(1, 1, 0, src.data_ptr(), 8192, mw.MW_F32)]
        assert wait(mw, hs) == [mw.MW_DONE] * 2
        t0 = time.perf_counter()
        assert mw.mw_poll(stuck) == mw.MW_PENDING
        worst = max(worst, time.perf_counter() - t0)
    assert torch.equal(src, dst)
    assert worst < 5e-3, f"a poll took {worst * 1e3:.2f} ms: polls must not wait for the device"
    mw.mw_world_abort(0)
    assert mw.mw_poll(stuck) == mw.MW_BROKEN and mw.mw_world_state(1) == mw.MW_ALIVE


def _slot_fields(raw, i):
    """Decode ring slot i of a ring image: journal half and sync half."""
    base = 256 + 256 * i
    bufs = struct.unpack_from("<8Q", raw, base)
    nbytes, = struct.unpack_from("<Q", raw, base + 64)
    kind, dtype, nbuf, world, epoch, gen, nchunks, chunk = struct.unpack_from("<8I", raw, base + 72)
    arrived, done_gen = struct.unpack_from("<2I", raw, base + 128)
    return dict(bufs=bufs, nbytes=nbytes, kind=kind, dtype=dtype, nbuf=nbuf, world=world, epoch=epoch, gen=gen,
                nchunks=nchunks, chunk=chunk, arrived=arrived, done_gen=done_gen)


def test_ring_journal_header_and_isolation_across_abort(torch, mw):
    mw.mw_world_create(40, [0, 1])
    mw.mw_world_create(41, [0, 2])
    mw.mw_world_create(42, [3, 4, 5])
    n = 3 << 20
    bufs = {w: (torch.full((n,), w, dtype=torch.uint8, device="cuda"), torch.zeros(n, dtype=torch.uint8, device="cuda")) for w in (40, 41)}
    hs = []
    for w in (40, 41):
        hs += [mw.mw_send(w, 1, 0, bufs[w][0].data_ptr(), n // 2, mw.MW_BF16), mw.mw_recv(w, 1, 0, bufs[w][1].data_ptr(), n // 2, mw.MW_BF16)]
    xs = [torch.ones(1000, dtype=torch.float32, device="cuda") for _ in range(3)]
    hs += [mw.mw_allreduce_sum(42, r, xs[r].data_ptr(), 1000, mw.MW_F32) for r in range(3)]
    assert wait(mw, hs) == [mw.MW_DONE] * 7
    raw = mw.mw_debug_ring_read(40)
    wid, state, epoch, depth, first_slot, n_ranks = struct.unpack_from("<6I", raw, 0)
    assert (wid, state, epoch, depth, n_ranks) == (40, 0, 0, 128, 2)
    used = [s for s in (_slot_fields(raw, i) for i in range(depth)) if s["gen"]]
    assert len(used) == 1
    s = used[0]
    assert s["bufs"][:2] == (bufs[40][0].data_ptr(), bufs[40][1].data_ptr()) and s["nbytes"] == n
    assert (s["kind"], s["nbuf"], s["world"], s["epoch"], s["dtype"]) == (0, 2, 40, 0, mw.MW_BF16)
    assert s["nchunks"] * s["chunk"] >= n > (s["nchunks"] - 1) * s["chunk"]
    assert s["nchunks"] > 1 and s["arrived"] == s["nchunks"] and s["done_gen"] == s["gen"]  # every chunk counted in, completion published
    r42 = mw.mw_debug_ring_read(42)
    s42 = [x for x in (_slot_fields(r42, i) for i in range(128)) if x["gen"]][0]
    assert (s42["kind"], s42["nbuf"], s42["nbytes"], s42["world"]) == (2, 3, 4000, 42)
    assert s42["nchunks"] == 1 and s42["arrived"] == 0 and s42["done_gen"] == s42["gen"]  # one chunk: no counting
    # abort world 40 while one of its operations waits for a peer: nothing else changes
    before = mw.mw_debug_arena_hash(40)
    snap41, snap42 = mw.mw_debug_ring_read(41), mw.mw_debug_ring_read(42)
    keep = {w: bufs[w][1].clone() for w in (40, 41)}
    lonely = mw.mw_recv(40, 1, 0, bufs[40][1].data_ptr(), n // 2, mw.MW_BF16)
    mw.mw_world_abort(40)
    assert mw.mw_poll(lonely) == mw.MW_BROKEN
    assert mw.mw_debug_arena_hash(40) == before
    assert mw.mw_debug_ring_read(41) == snap41 and mw.mw_debug_ring_read(42) == snap42
    raw = mw.mw_debug_ring_read(40)
    wid, state, epoch = struct.unpack_from("<3I", raw, 0)
    assert (wid, state, epoch) == (40, mw.MW_BROKEN, 1)
    assert torch.equal(bufs[41][1], keep[41]) and torch.equal(bufs[40][1], keep[40])
    # the healthy worlds go on
    hs = [mw.mw_send(41, 1, 0, bufs[41][0].data_ptr(), n // 2, mw.MW_BF16), mw.mw_recv(41, 1, 0, bufs[41][1].data_ptr(), n // 2, mw.MW_BF16)]
    assert wait(mw, hs) == [mw.MW_DONE] * 2
    with pytest.raises(mw.MwError) as e:
        mw.mw_send(40, 1, 0, bufs[40][0].data_ptr(), n // 2, mw.MW_BF16)
    assert e.value.code == mw.MW_EBROKEN


@pytest.mark.parametrize("n", [2, 3, 4, 5, 6, 8])
def test_large_reductions_in_every_chunk_size_the_library_chooses(torch, mw, n):
    """The chunk of a reduce entry depends on the number of ranks and on who is written (all-reduce 32 ... 8 KiB,
    reduce to a root 48 ... 12 KiB, sizes that are not powers of two among them; two vectors per thread for 2
    ranks).  Payloads here are large enough for the largest choice, with a ragged tail; the journal in the world's
    ring tells which was taken."""
    mw.mw_world_create(0, list(range(n)))
    count = (17 << 20) // 4 + 1237  # 17 MiB and a tail per rank: several hundred chunks of any size
    rng = np.random.default_rng(900 + n)
    seen = set()
    for dtype, root in (("f32", None), ("bf16", None), ("f32", n - 1)):
        c = count if dtype == "f32" else 2 * count + 3
        xs = [rng.uniform(-1, 1, c).astype(np.float32) for _ in range(n)]
        host = [x.view(np.uint8) if dtype == "f32" else oracle.f32_to_bf16_bits(x).view(np.uint8) for x in xs]
        dev = [dev_bytes(torch, host[r]) for r in range(n)]
        if root is None:
            hs = [mw.mw_allreduce_sum(0, r, dev[r][1].data_ptr(), c, mw.DTYPES[dtype]) for r in range(n)]
        else:
            hs = [mw.mw_reduce_sum(0, r, root, dev[r][1].data_ptr(), c, mw.DTYPES[dtype]) for r in range(n)]
        assert wait(mw, hs) == [mw.MW_DONE] * n
        s, sabs = oracle.allreduce_sum_f64(host, c, dtype)
        ordered = oracle.allreduce_sum_ordered(host, c, dtype)
        for r in range(n):
            got = dev[r][1].cpu().numpy()
            if root is None or r == root:
                ok, worst = oracle.allreduce_within_tolerance(got, s, sabs, c, dtype)
                assert ok, (n, dtype, root, r, worst)
                assert np.array_equal(got, ordered), (n, dtype, root, r)
            else:
                assert np.array_equal(got, host[r]), "a non-root buffer was written"
            base = dev[r][0].cpu().numpy()
            assert np.all(base[host[r].size:] == 0x5A)  # nothing past the end
        raw = mw.mw_debug_ring_read(0)
        mine = [f for f in (_slot_fields(raw, i) for i in range(128))
                if f["gen"] and f["bufs"][0] == dev[0][1].data_ptr() and f["nbytes"] == host[0].size
                and f["kind"] == (2 if root is None else 3) and f["dtype"] == mw.DTYPES[dtype]]
        last = max(mine, key=lambda f: f["gen"])
        assert last["nchunks"] * last["chunk"] >= host[0].size > (last["nchunks"] - 1) * last["chunk"]
        seen.add((root is None, last["chunk"]))
    want_all = {2: 32, 3: 16, 4: 12}.get(n, 8) << 10
    want_root = {2: 48, 3: 32, 4: 24, 5: 24, 6: 16, 8: 12}[n] << 10
    assert seen == {(True, want_all), (False, want_root)}, seen


def test_watchdog_cleans_up_a_silent_worker_while_others_stream(torch, mw):
    """Silent failure on the GPU path: worker 2 stops reporting; the watchdog thread breaks its world only,
    the transfer it had already been matched for is delivered, the other world keeps moving data."""
    mw.mw_world_create(1, [0, 1])
    mw.mw_world_create(2, [0, 2])
    n = 8 << 20
    src = {w: torch.full((n,), w, dtype=torch.uint8, device="cuda") for w in (1, 2)}
    dst = {w: torch.zeros(n, dtype=torch.uint8, device="cuda") for w in (1, 2)}
    mw.mw_watchdog_start(0.3, 0.02)
    try:
        for k in (0, 1, 2):
            mw.mw_heartbeat(k)
        last2 = [mw.mw_send(2, 1, 0, src[2].data_ptr(), n // 4, mw.MW_F32), mw.mw_recv(2, 1, 0, dst[2].data_ptr(), n // 4, mw.MW_F32)]
        lonely = mw.mw_recv(2, 1, 0, dst[2].data_ptr(), n // 4, mw.MW_F32)  # waits for a tensor that never comes
        moved = 0
        t0 = time.time()
        while mw.mw_world_state(2) == mw.MW_ALIVE:
            assert time.time() - t0 < 10
            mw.mw_heartbeat(0)
            mw.mw_heartbeat(1)
            dst[1].zero_()
            hs = [mw.mw_send(1, 1, 0, src[1].data_ptr(), n // 4, mw.MW_F32), mw.mw_recv(1, 1, 0, dst[1].data_ptr(), n // 4, mw.MW_F32)]
            assert wait(mw, hs) == [mw.MW_DONE] * 2 and bool((dst[1] == 1).all())
            moved += 1
        assert 0.25 < time.time() - t0 < 3.0 and moved > 3
        assert wait(mw, last2) == [mw.MW_DONE] * 2 and bool((dst[2] == 2).all())  # matched before the failure: delivered
        assert mw.mw_poll(lonely) == mw.MW_BROKEN
        assert mw.mw_world_state(1) == mw.MW_ALIVE and mw.mw_worker_state(2) == mw.MW_BROKEN
        hs = [mw.mw_send(1, 1, 0, src[1].data_ptr(), n // 4, mw.MW_F32), mw.mw_recv(1, 1, 0, dst[1].data_ptr(), n // 4, mw.MW_F32)]
        assert wait(mw, hs) == [mw.MW_DONE] * 2
    finally:
        mw.mw_watchdog_stop()
