"""ctypes binding of libmw.so: the same names as include/mw.h, argument marshalling only.

Buffers are passed as integer device addresses (e.g. torch.Tensor.data_ptr()), streams as
integer hipStream_t values (e.g. torch.cuda.Stream.cuda_stream; 0 = the null stream,
STREAM_NONE = no ordering needed).  Calls that return a status raise MwError on a negative
code, except mw_poll, whose negative codes are states of the operation and are returned.
There is no fallback: if the library is missing or fails to load, the first call raises.
"""

from __future__ import annotations

import ctypes as C
import threading
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmw.so")

# mw_poll / mw_world_state results and error codes (mirrors include/mw.h)
MW_DONE, MW_PENDING, MW_BROKEN, MW_ALIVE = 0, 1, 2, 0
MW_OK, MW_EINVAL, MW_ENOWORLD, MW_EBROKEN, MW_EEXIST = 0, -1, -2, -3, -4
MW_EMISMATCH, MW_ENOMEM, MW_EBADHANDLE, MW_EHIP, MW_ENOTINIT = -5, -6, -7, -8, -9
MW_F32, MW_BF16 = 0, 1
DTYPES = {"f32": MW_F32, "bf16": MW_BF16}
STREAM_NONE = -1
KIND_COPY, KIND_BCAST, KIND_REDUCE = 0, 1, 2

SYMBOLS = [
    "mw_init", "mw_shutdown", "mw_world_create", "mw_world_abort", "mw_worker_abort", "mw_world_state",
    "mw_send", "mw_recv", "mw_broadcast", "mw_allreduce_sum", "mw_reduce_sum", "mw_all_gather", "mw_gather",
    "mw_scatter", "mw_poll", "mw_flush", "mw_pending_ops", "mw_poll_many", "mw_post_many",
    "mw_config_set", "mw_config_get", "mw_handle_capacity", "mw_last_hip_error", "mw_strerror",
    "mw_profile_enable", "mw_profile_read", "mw_debug_ring_read", "mw_debug_arena_hash", "mw_heartbeat",
    "mw_heartbeat_at", "mw_watchdog_start", "mw_watchdog_stop", "mw_watchdog_check_at", "mw_worker_state",
    "mw_heartbeat_epoch", "mw_build_id", "mw_post_many_noalloc", "mw_debug_mailbox",
]


POST_SEND, POST_RECV, POST_BROADCAST, POST_ALLREDUCE_SUM = 0, 1, 2, 3
POST_REDUCE_SUM, POST_ALL_GATHER, POST_GATHER, POST_SCATTER = 4, 5, 6, 7


class PostDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("world_id", C.c_int32), ("a", C.c_int32), ("b", C.c_int32),
                ("buf", C.c_void_p), ("count", C.c_uint64), ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("hip_stream", C.c_void_p), ("buf2", C.c_void_p)]


class MwError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def declare(lib):
    """Set argument and result types on a loaded library (also used for the host-check build)."""
    vp, i, sz, u64p = C.c_void_p, C.c_int, C.c_size_t, C.POINTER(C.c_uint64)
    lib.mw_init.argtypes = [i, i]
    lib.mw_shutdown.argtypes = []
    lib.mw_world_create.argtypes = [i, C.POINTER(C.c_int), i]
    lib.mw_world_abort.argtypes = [i]
    lib.mw_worker_abort.argtypes = [i]
    lib.mw_world_state.argtypes = [i]
    for f in (lib.mw_send, lib.mw_recv):
        f.argtypes = [i, i, i, vp, sz, i, vp, u64p]
    lib.mw_broadcast.argtypes = [i, i, i, vp, sz, i, vp, u64p]
    lib.mw_allreduce_sum.argtypes = [i, i, vp, sz, i, vp, u64p]
    lib.mw_reduce_sum.argtypes = [i, i, i, vp, sz, i, vp, u64p]
    lib.mw_all_gather.argtypes = [i, i, vp, vp, sz, i, vp, u64p]
    lib.mw_gather.argtypes = [i, i, i, vp, vp, sz, i, vp, u64p]
    lib.mw_scatter.argtypes = [i, i, i, vp, vp, sz, i, vp, u64p]
    lib.mw_poll.argtypes = [C.c_uint64]
    lib.mw_flush.argtypes = []
    lib.mw_pending_ops.argtypes = []
    lib.mw_poll_many.argtypes = [u64p, i, C.POINTER(C.c_int)]
    lib.mw_post_many.argtypes = [C.POINTER(PostDesc), i, u64p, C.POINTER(C.c_int)]
    lib.mw_post_many_noalloc.argtypes = [C.POINTER(PostDesc), i, vp]
    lib.mw_config_set.argtypes = [C.c_char_p, C.c_long]
    lib.mw_config_get.argtypes = [C.c_char_p]
    lib.mw_config_get.restype = C.c_long
    lib.mw_handle_capacity.argtypes = []
    lib.mw_last_hip_error.argtypes = []
    lib.mw_strerror.argtypes = [i]
    lib.mw_strerror.restype = C.c_char_p
    lib.mw_build_id.argtypes = []
    lib.mw_build_id.restype = C.c_char_p
    lib.mw_profile_enable.argtypes = [i]
    lib.mw_profile_read.argtypes = [i, u64p, C.POINTER(C.c_double), u64p]
    lib.mw_debug_ring_read.argtypes = [i, vp, sz]
    lib.mw_debug_ring_read.restype = C.c_long
    lib.mw_debug_arena_hash.argtypes = [i, u64p]
    u32p = C.POINTER(C.c_uint32)
    lib.mw_debug_mailbox.argtypes = [u32p, u32p, u32p]
    lib.mw_heartbeat.argtypes = [i]
    lib.mw_heartbeat_at.argtypes = [i, C.c_double]
    lib.mw_watchdog_start.argtypes = [C.c_double, C.c_double]
    lib.mw_watchdog_stop.argtypes = []
    lib.mw_watchdog_check_at.argtypes = [C.c_double, C.c_double]
    lib.mw_worker_state.argtypes = [i]
    lib.mw_heartbeat_epoch.argtypes = [i]
    lib.mw_heartbeat_epoch.restype = C.c_long
    return lib


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2407_08980_amd.build` "
                               "(there is no fallback path)")
        try:  # one HIP runtime per process: when torch is there, its copy must be the one already loaded
            import torch  # noqa: F401
        except ImportError:
            pass
        _lib = declare(C.CDLL(LIB_PATH))
        check_build(_lib, LIB_PATH)
    return _lib


def check_build(handle, path):
    """A library compiled from other sources than the ones beside it must not be measured or tested."""
    from . import build

    have, want = handle.mw_build_id().decode(), build.source_id()
    if have != want:
        raise RuntimeError(f"{path} was built from other sources (library {have}, sources {want}): run "
                           "`python -m paper_2407_08980_amd.build`")


def use_library(handle):
    """Route the binding through an already loaded library (the CPU tests pass the host-check build)."""
    global _lib
    _lib = declare(handle)


def strerror(code):
    return lib().mw_strerror(code).decode()


def _ck(rc, where):
    if rc < 0:
        raise MwError(rc, where)
    return rc


_NO_STREAM = C.c_void_p(-1).value  # MW_STREAM_NONE as the integer a c_void_p argument takes


def _stream(s):
    return s if s != STREAM_NONE else _NO_STREAM


_tls = threading.local()


def _out():
    """This thread's handle out-parameter and a reference to it (made once: they are on every post's path)."""
    h = getattr(_tls, "h", None)
    if h is None:
        h = _tls.h = C.c_uint64(0)
        _tls.ref = C.byref(h)
    return h, _tls.ref


def mw_init(hip_device, n_workers):
    return _ck(lib().mw_init(hip_device, n_workers), "mw_init")


def mw_shutdown():
    return _ck(lib().mw_shutdown(), "mw_shutdown")


def mw_world_create(world_id, worker_ids):
    arr = (C.c_int * len(worker_ids))(*worker_ids)
    return _ck(lib().mw_world_create(world_id, arr, len(worker_ids)), "mw_world_create")


def mw_world_abort(world_id):
    return _ck(lib().mw_world_abort(world_id), "mw_world_abort")


def mw_worker_abort(worker_id):
    return _ck(lib().mw_worker_abort(worker_id), "mw_worker_abort")


def mw_world_state(world_id):
    return _ck(lib().mw_world_state(world_id), "mw_world_state")


def mw_send(world, src_rank, dst_rank, buf, count, dtype, stream=0):
    h, ref = _out()
    rc = lib().mw_send(world, src_rank, dst_rank, buf, count, dtype, _stream(stream), ref)
    if rc < 0:
        raise MwError(rc, "mw_send")
    return h.value


def mw_recv(world, src_rank, dst_rank, buf, count, dtype, stream=0):
    h, ref = _out()
    rc = lib().mw_recv(world, src_rank, dst_rank, buf, count, dtype, _stream(stream), ref)
    if rc < 0:
        raise MwError(rc, "mw_recv")
    return h.value


def mw_broadcast(world, rank, root_rank, buf, count, dtype, stream=0):
    h, ref = _out()
    rc = lib().mw_broadcast(world, rank, root_rank, buf, count, dtype, _stream(stream), ref)
    if rc < 0:
        raise MwError(rc, "mw_broadcast")
    return h.value


def mw_allreduce_sum(world, rank, buf, count, dtype, stream=0):
    h, ref = _out()
    rc = lib().mw_allreduce_sum(world, rank, buf, count, dtype, _stream(stream), ref)
    if rc < 0:
        raise MwError(rc, "mw_allreduce_sum")
    return h.value


def mw_reduce_sum(world, rank, root_rank, buf, count, dtype, stream=0):
    h, ref = _out()
    rc = lib().mw_reduce_sum(world, rank, root_rank, buf, count, dtype, _stream(stream), ref)
    if rc < 0:
        raise MwError(rc, "mw_reduce_sum")
    return h.value


def mw_all_gather(world, rank, sendbuf, recvbuf, count, dtype, stream=0):
    h, ref = _out()
    rc = lib().mw_all_gather(world, rank, sendbuf, recvbuf, count, dtype, _stream(stream), ref)
    if rc < 0:
        raise MwError(rc, "mw_all_gather")
    return h.value


def mw_gather(world, rank, root_rank, sendbuf, recvbuf, count, dtype, stream=0):
    """recvbuf: None on every rank but the root."""
    h, ref = _out()
    rc = lib().mw_gather(world, rank, root_rank, sendbuf, recvbuf, count, dtype, _stream(stream), ref)
    if rc < 0:
        raise MwError(rc, "mw_gather")
    return h.value


def mw_scatter(world, rank, root_rank, sendbuf, recvbuf, count, dtype, stream=0):
    """sendbuf: None on every rank but the root."""
    h, ref = _out()
    rc = lib().mw_scatter(world, rank, root_rank, sendbuf, recvbuf, count, dtype, _stream(stream), ref)
    if rc < 0:
        raise MwError(rc, "mw_scatter")
    return h.value


def mw_poll(handle):
    return lib().mw_poll(handle)


def mw_flush():
    return _ck(lib().mw_flush(), "mw_flush")


def mw_pending_ops():
    return _ck(lib().mw_pending_ops(), "mw_pending_ops")


class PollSet:
    """Reusable arrays for mw_poll_many over a fixed list of handles."""

    def __init__(self, handles):
        self.n = len(handles)
        self.handles = (C.c_uint64 * self.n)(*handles)
        self.states = (C.c_int * self.n)()
        self._bind()

    def _bind(self):
        # pointers made once: converting an array argument on every call costs more than the library's own work
        self._hp = C.cast(self.handles, C.POINTER(C.c_uint64))
        self._sp = C.cast(self.states, C.POINTER(C.c_int))
        self._call = lib().mw_poll_many

    def poll(self):
        """Number of handles still pending; self.states holds every state."""
        rc = self._call(self._hp, self.n, self._sp)
        if rc < 0:
            raise MwError(rc, "mw_poll_many")
        return rc


class PostBatch:
    """A reusable array of posts for mw_post_many: (kind, world, a, b, buf, count, dtype, stream[, buf2]) tuples."""

    def __init__(self, posts):
        self.n = len(posts)
        self.descs = (PostDesc * self.n)()
        for d, p in zip(self.descs, posts):
            kind, world, a, b, buf, count, dtype, stream = p[:8]
            d.kind, d.world_id, d.a, d.b, d.buf, d.count, d.dtype = kind, world, a, b, buf, count, dtype
            d.buf2 = p[8] if len(p) > 8 else None
            d.hip_stream = stream if stream != STREAM_NONE else C.c_void_p(-1).value
        self.handles = (C.c_uint64 * self.n)()
        self.results = (C.c_int * self.n)()
        self._dp = C.cast(self.descs, C.POINTER(PostDesc))  # pointers made once (see PollSet._bind)
        self._hp = C.cast(self.handles, C.POINTER(C.c_uint64))
        self._rp = C.cast(self.results, C.POINTER(C.c_int))
        self._call = lib().mw_post_many

    def post(self, check=True):
        rc = self._call(self._dp, self.n, self._hp, self._rp)
        if check and rc < 0:
            raise MwError(rc, "mw_post_many")
        return rc

    def pollset(self):
        """A PollSet over this batch's own handle array (no copy): it always polls the handles of the latest post().
        Refused posts have handle 0, which polls as MW_EBADHANDLE, i.e. not pending."""
        ps = self.__dict__.get("_pollset")
        if ps is None:
            ps = PollSet.__new__(PollSet)
            ps.n, ps.handles, ps.states = self.n, self.handles, (C.c_int * self.n)()
            ps._bind()
            self._pollset = ps
        return ps


def mw_post_many(posts):
    """Post a list of (kind, world, a, b, buf, count, dtype, stream); returns (handles, results)."""
    pb = PostBatch(posts)
    pb.post(check=False)
    return list(pb.handles), list(pb.results)


def mw_post_many_noalloc(posts, stream=0):
    """Enqueue whole operations on `stream` without allocating; `posts` is a PostBatch or a list of post tuples.
    Returns the library's code (negative = refused, nothing enqueued)."""
    pb = posts if isinstance(posts, PostBatch) else PostBatch(posts)
    return lib().mw_post_many_noalloc(pb.descs, pb.n, _stream(stream))


def mw_poll_many(handles):
    ps = PollSet(handles)
    ps.poll()
    return list(ps.states)


def mw_config_set(key, value):
    return _ck(lib().mw_config_set(key.encode(), value), f"mw_config_set({key})")


def mw_config_get(key):
    return lib().mw_config_get(key.encode())


def mw_handle_capacity():
    return lib().mw_handle_capacity()


def mw_last_hip_error():
    return lib().mw_last_hip_error()


def mw_strerror(code):
    return strerror(code)


def mw_heartbeat(worker_id):
    return _ck(lib().mw_heartbeat(worker_id), "mw_heartbeat")


def mw_heartbeat_at(worker_id, t):
    return _ck(lib().mw_heartbeat_at(worker_id, t), "mw_heartbeat_at")


def mw_watchdog_start(timeout_s, period_s):
    return _ck(lib().mw_watchdog_start(timeout_s, period_s), "mw_watchdog_start")


def mw_watchdog_stop():
    return _ck(lib().mw_watchdog_stop(), "mw_watchdog_stop")


def mw_watchdog_check_at(t, timeout_s):
    """Number of workers newly declared failed by this inspection."""
    return _ck(lib().mw_watchdog_check_at(t, timeout_s), "mw_watchdog_check_at")


def mw_worker_state(worker_id):
    return _ck(lib().mw_worker_state(worker_id), "mw_worker_state")


def mw_heartbeat_epoch(worker_id):
    return _ck(lib().mw_heartbeat_epoch(worker_id), "mw_heartbeat_epoch")


def mw_profile_enable(on):
    return _ck(lib().mw_profile_enable(1 if on else 0), "mw_profile_enable")


def mw_profile_read(kind):
    """(launches, total_ms, op_bytes) of the finished launches of one kernel kind since the last read."""
    n, ms, b = C.c_uint64(0), C.c_double(0), C.c_uint64(0)
    _ck(lib().mw_profile_read(kind, C.byref(n), C.byref(ms), C.byref(b)), "mw_profile_read")
    return n.value, ms.value, b.value


def mw_debug_ring_read(world_id):
    """Bytes of a world's ring header and slots as they are in HBM."""
    cap = 256 + 256 * 256
    buf = (C.c_ubyte * cap)()
    n = lib().mw_debug_ring_read(world_id, buf, cap)
    _ck(n, "mw_debug_ring_read")
    return bytes(buf[:n])


def mw_debug_arena_hash(except_world=-1):
    h, ref = _out()
    rc = lib().mw_debug_arena_hash(except_world, ref)
    if rc < 0:
        raise MwError(rc, "mw_debug_arena_hash")
    return h.value


def mw_debug_mailbox():
    """(epoch, open, tail) of the resident mailbox kernel."""
    e, o, t = C.c_uint32(0), C.c_uint32(0), C.c_uint32(0)
    _ck(lib().mw_debug_mailbox(C.byref(e), C.byref(o), C.byref(t)), "mw_debug_mailbox")
    return e.value, o.value, t.value
