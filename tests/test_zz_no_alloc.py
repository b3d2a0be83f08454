"""The entry point that allocates nothing (mw_post_many_noalloc) against the one it is a variant of
(mw_post_many + mw_flush + mw_poll), through the C ABI: the same whole operations on identical inputs must leave
identical bytes, on two calls in a row, the second with a smaller input.  The copies and fan-outs are also held to
the CPU oracle's bytes and the sums to its ascending-order fp32 sum, as everywhere else.
"""

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


@pytest.fixture
def mw(torch):
    from paper_2407_08980_amd import binding

    binding.lib()
    binding.mw_init(0, 16)
    yield binding
    binding.mw_shutdown()


def _workload(torch, mw, scale, seed):
    """Whole operations over four worlds: ragged copies (one unaligned), a broadcast, fp32 and bf16 all-reduces, a
    reduce, a gather, a scatter and an all-gather.  Returns (host inputs, make(bufs) -> posts, expectations)."""
    rng = np.random.default_rng(seed)
    host = {}

    def raw(name, nbytes):
        host[name] = rng.integers(0, 256, size=nbytes, dtype=np.uint8)

    def vals(name, count, dtype):
        x = rng.uniform(-1, 1, count).astype(np.float32)
        host[name] = x.view(np.uint8).copy() if dtype == "f32" else oracle.f32_to_bf16_bits(x).view(np.uint8).copy()

    def poison(name, nbytes):
        host[name] = np.full(nbytes, 0xA5, np.uint8)

    c1, c2, c3 = 70001 * scale, 33333 * scale + 1, 9001 * scale + 3
    raw("p0s", c1 * 4), poison("p0d", c1 * 4)
    raw("p1s", c2 * 2), poison("p1d", c2 * 2)
    raw("p2s", c3 * 2), poison("p2d", c3 * 2)
    for r in range(3):
        (raw if r == 1 else poison)(f"b{r}", c2 * 4)
    for r in range(4):
        vals(f"a{r}", c1, "f32")
        vals(f"h{r}", c2, "bf16")
        vals(f"r{r}", c3, "f32")
    for r in range(3):
        raw(f"gs{r}", c3 * 4)
        poison(f"sd{r}", c3 * 4)
        raw(f"ags{r}", c3 * 2)
        poison(f"agd{r}", 3 * c3 * 2)
    poison("gd", 3 * c3 * 4)
    raw("ss", 3 * c3 * 4)
    offsets = {"p2s": 2, "p2d": 6}  # one copy that is not 16-byte aligned

    def make(ptr):
        F, B = mw.MW_F32, mw.MW_BF16
        P = []
        # world 0 = (0, 1): two messages of the same pair, receives first, then one the other way round
        P.append((mw.POST_RECV, 0, 0, 1, ptr["p0d"], c1, F, 0))
        P.append((mw.POST_RECV, 0, 0, 1, ptr["p1d"], c2, B, 0))
        P.append((mw.POST_SEND, 0, 0, 1, ptr["p0s"], c1, F, 0))
        P.append((mw.POST_SEND, 0, 0, 1, ptr["p1s"], c2, B, 0))
        P.append((mw.POST_SEND, 0, 1, 0, ptr["p2s"], c3, B, 0))
        P.append((mw.POST_RECV, 0, 1, 0, ptr["p2d"], c3, B, 0))
        # world 1 = (2, 3, 4): broadcast from rank 1, then a gather, a scatter, an all-gather (in this order per rank)
        for r in (2, 0, 1):
            P.append((mw.POST_BROADCAST, 1, r, 1, ptr[f"b{r}"], c2, F, 0))
        for r in (0, 1, 2):
            P.append((mw.POST_GATHER, 1, r, 2, ptr[f"gs{r}"], c3, F, 0, ptr["gd"] if r == 2 else None))
        for r in (1, 2, 0):
            P.append((mw.POST_SCATTER, 1, r, 0, ptr["ss"] if r == 0 else None, c3, F, 0, ptr[f"sd{r}"]))
        for r in (0, 1, 2):
            P.append((mw.POST_ALL_GATHER, 1, r, 0, ptr[f"ags{r}"], c3, B, 0, ptr[f"agd{r}"]))
        # world 2 = (5, 6, 7, 8): fp32 all-reduce, bf16 all-reduce, reduce to rank 3, interleaved over the ranks
        for r in (3, 1, 0, 2):
            P.append((mw.POST_ALLREDUCE_SUM, 2, r, 0, ptr[f"a{r}"], c1, F, 0))
            P.append((mw.POST_ALLREDUCE_SUM, 2, r, 0, ptr[f"h{r}"], c2, B, 0))
        for r in range(4):
            P.append((mw.POST_REDUCE_SUM, 2, r, 3, ptr[f"r{r}"], c3, F, 0))
        return P

    want = {"p0d": oracle.copy_result(host["p0s"]), "p1d": oracle.copy_result(host["p1s"]), "p2d": oracle.copy_result(host["p2s"]),
            "gd": oracle.gather_result([host[f"gs{r}"] for r in range(3)])}
    for r, b in enumerate(oracle.broadcast_result([host[f"b{r}"] for r in range(3)], 1)):
        want[f"b{r}"] = b
    for r in range(3):
        want[f"sd{r}"] = oracle.scatter_result(host["ss"], 3, r)
        want[f"agd{r}"] = oracle.all_gather_result([host[f"ags{q}"] for q in range(3)])
    ar = oracle.allreduce_sum_ordered([host[f"a{r}"] for r in range(4)], c1, "f32")
    hr = oracle.allreduce_sum_ordered([host[f"h{r}"] for r in range(4)], c2, "bf16")
    rr = oracle.allreduce_sum_ordered([host[f"r{r}"] for r in range(4)], c3, "f32")
    for r in range(4):
        want[f"a{r}"], want[f"h{r}"] = ar, hr
        want[f"r{r}"] = rr if r == 3 else host[f"r{r}"]
    return host, offsets, make, want


def _upload(torch, host, offsets):
    base, view = {}, {}
    for name, arr in host.items():
        off = offsets.get(name, 0)
        b = torch.full((off + arr.size + 64,), 0x5A, dtype=torch.uint8, device="cuda")
        b[off:off + arr.size].copy_(torch.from_numpy(arr))
        base[name], view[name] = b, b[off:off + arr.size]
    return base, view


def _run_pair(torch, mw, scale, seed, stream):
    host, offsets, make, want = _workload(torch, mw, scale, seed)
    base_a, view_a = _upload(torch, host, offsets)
    base_b, view_b = _upload(torch, host, offsets)
    torch.cuda.synchronize()
    # the existing entry point
    handles, results = mw.mw_post_many(make({k: v.data_ptr() for k, v in view_a.items()}))
    assert all(r == 0 for r in results)
    mw.mw_flush()
    ps = mw.PollSet(handles)
    t0 = time.time()
    while ps.poll():
        assert time.time() - t0 < 60
    assert set(ps.states) == {mw.MW_DONE}
    # the one that allocates nothing: device memory in use must not move across the call
    pb = mw.PostBatch(make({k: v.data_ptr() for k, v in view_b.items()}))
    free_before = torch.cuda.mem_get_info()[0]
    rc = mw.mw_post_many_noalloc(pb, stream.cuda_stream)
    assert rc == 0, mw.mw_strerror(rc)
    stream.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before
    for name in host:
        a, b = base_a[name].cpu().numpy(), base_b[name].cpu().numpy()
        assert np.array_equal(a, b), f"{name}: the two entry points disagree"
        off = offsets.get(name, 0)
        got = b[off:off + host[name].size]
        assert np.array_equal(got, want.get(name, host[name])), f"{name}: differs from the oracle"
        assert np.all(b[:off] == 0x5A) and np.all(b[off + host[name].size:] == 0x5A), f"{name}: written outside"
    return len(pb.descs)


def _used_stream(torch):
    """A caller's stream that has run something already.  The runtime sets a stream's hardware queue up at the stream's
    first launch (2 MiB of device memory on this machine): that belongs to the stream, not to what is launched on it,
    and the free-memory check below must not see it."""
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        torch.zeros(16, device="cuda").add_(1)
    s.synchronize()
    return s


def test_noalloc_entry_point_matches_post_many_on_two_calls_in_a_row(torch, mw):
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [2, 3, 4])
    mw.mw_world_create(2, [5, 6, 7, 8])
    s = _used_stream(torch)
    assert _run_pair(torch, mw, scale=40, seed=1, stream=s) == 6 + 3 + 9 + 8 + 4  # several hundred chunks per kind
    _run_pair(torch, mw, scale=1, seed=2, stream=s)  # the second call is smaller: stale counters would show here
    _run_pair(torch, mw, scale=7, seed=3, stream=s)


def test_noalloc_entry_point_refuses_what_it_cannot_run(torch, mw):
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [2, 3])
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    keep = buf.clone()
    p, F = buf.data_ptr(), mw.MW_F32
    s = torch.cuda.Stream()
    half = [(mw.POST_SEND, 0, 0, 1, p, 16, F, 0)]
    assert mw.mw_post_many_noalloc(half, s.cuda_stream) == mw.MW_EINVAL  # a side without its peer
    pair = [(mw.POST_SEND, 0, 0, 1, p, 16, F, 0), (mw.POST_RECV, 0, 0, 1, p + 2048, 8, F, 0)]
    assert mw.mw_post_many_noalloc(pair, s.cuda_stream) == mw.MW_EMISMATCH
    assert mw.mw_post_many_noalloc([(mw.POST_SEND, 9, 0, 1, p, 16, F, 0)], s.cuda_stream) == mw.MW_ENOWORLD
    too_many = [(mw.POST_SEND, 0, 0, 1, p, 4, F, 0), (mw.POST_RECV, 0, 0, 1, p + 2048, 4, F, 0)] * 65
    assert mw.mw_post_many_noalloc(too_many, s.cuda_stream) == mw.MW_EINVAL  # more than MW_NOALLOC_MAX_POSTS
    assert mw.mw_post_many_noalloc(pair[:1] + [(mw.POST_RECV, 0, 0, 1, p + 2048, 16, F, 0)], mw.STREAM_NONE) == mw.MW_EINVAL
    mw.mw_world_abort(1)
    broken = [(mw.POST_SEND, 1, 0, 1, p, 16, F, 0), (mw.POST_RECV, 1, 0, 1, p + 2048, 16, F, 0)]
    assert mw.mw_post_many_noalloc(broken, s.cuda_stream) == mw.MW_EBROKEN
    assert mw.mw_post_many_noalloc([], s.cuda_stream) == mw.MW_OK
    s.synchronize()
    assert torch.equal(buf, keep)  # nothing was enqueued by any of the refused calls
    # sides posted through the other calls are neither consumed nor disturbed
    h = mw.mw_recv(0, 0, 1, p + 1024, 16, F)
    ok = [(mw.POST_SEND, 0, 0, 1, p, 16, F, 0), (mw.POST_RECV, 0, 0, 1, p + 2048, 16, F, 0)]
    buf[:64] = 7
    torch.cuda.synchronize()
    assert mw.mw_post_many_noalloc(ok, s.cuda_stream) == mw.MW_OK
    s.synchronize()
    assert mw.mw_poll(h) == mw.MW_PENDING and bool((buf[2048:2112] == 7).all()) and bool((buf[1024:1088] == 0).all())


def test_noalloc_entry_point_recorded_into_a_graph_and_replayed(torch, mw):
    """One of the callers the entry point is for: code under HIP graph capture.  The call is recorded into a graph
    once (nothing may allocate or clear memory with a memset node there) and the graph replayed four times, with eager
    work -- new inputs, cleared outputs, a synchronisation -- between the replays; every replay against the oracle."""
    mw.mw_world_create(0, [0, 1])
    mw.mw_world_create(1, [2, 3, 4, 5])
    n, m = 70001, 4099
    rng = np.random.default_rng(77)
    src = torch.zeros(n, dtype=torch.int32, device="cuda")
    dst = torch.zeros(n, dtype=torch.int32, device="cuda")
    xs = [torch.zeros(m, dtype=torch.float32, device="cuda") for _ in range(4)]
    posts = [(mw.POST_SEND, 0, 0, 1, src.data_ptr(), n, mw.MW_F32, 0), (mw.POST_RECV, 0, 0, 1, dst.data_ptr(), n, mw.MW_F32, 0)]
    posts += [(mw.POST_ALLREDUCE_SUM, 1, r, 0, xs[r].data_ptr(), m, mw.MW_F32, 0) for r in range(4)]
    pb = mw.PostBatch(posts)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        assert mw.mw_post_many_noalloc(pb, stream=s.cuda_stream) == 0
    for k in range(4):
        hsrc = rng.integers(-2 ** 31, 2 ** 31 - 1, size=n, dtype=np.int64).astype(np.int32)
        hx = [rng.uniform(-1, 1, m).astype(np.float32) for _ in range(4)]
        src.copy_(torch.from_numpy(hsrc))
        dst.fill_(0x5A5A5A5A)
        for x, h in zip(xs, hx):
            x.copy_(torch.from_numpy(h))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(dst.cpu().numpy().view(np.uint8), oracle.copy_result(hsrc.view(np.uint8))), k
        want = oracle.allreduce_sum_ordered([h.view(np.uint8) for h in hx], m, "f32")
        for r in range(4):
            assert np.array_equal(xs[r].cpu().numpy().view(np.uint8), want), (k, r)
