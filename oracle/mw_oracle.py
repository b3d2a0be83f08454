"""Plain CPU statement of what MultiWorld's worlds compute (numpy only).

TEST INFRASTRUCTURE ONLY -- see the package docstring.  Every function cites
the passage of the paper (arXiv 2407.08980) it restates.

The paper's data plane has exact definitions, so the oracle is the definition
written out, processed strictly in program (trace) order with no concurrency:

* a *world* is a fixed set of workers forming one fault domain; a worker may
  be in many worlds; a worker's failure breaks exactly the worlds that contain
  it (Sec. 3.1 "Overview", Fig. 2).
* collective operations are addressed by world (Sec. 1, contributions) and
  are non-blocking: an operation whose peers have not arrived stays pending
  and must not hold up any other world (Sec. 3.2 "Non-blocking CCL
  operations").
* all eight operations of the communicator are covered: send, recv,
  broadcast, all-reduce, reduce, all-gather, gather, scatter (Sec. 3.3
  "World Communicator").  The paper only names them; their meaning is the
  usual one of collective communication: reduce leaves the sum on the root
  only, all-gather concatenates every rank's tensor in rank order on every
  rank, gather does so on the root only, scatter hands slice r of the
  root's tensor to rank r.
* when a world is broken the manager fences it off, aborts its pending
  operations and raises to the application; later access is refused
  (Sec. 3.3 "World Manager"); everything that completed before the failure
  stays delivered (Sec. 4.1, Fig. 4: the ten tensors sent before the kill all
  arrive).

Where the paper is silent the readings are:

* matching of point-to-point operations: per (world, src, dst) first-in
  first-out, no tags -- the k-th send pairs with the k-th recv;
* a send completes only when its recv has been posted (rendezvous);
* collectives: the k-th collective a rank posts in a world belongs to that
  world's k-th collective, which executes when every rank has posted it;
* all-reduce is in place and leaves the same tensor on every rank;
* sides that disagree on count, dtype, kind or root yield MISMATCH and move
  no data.

Pinned by tests/test_oracle_pins.py (identity, brute force, exact-arithmetic
special cases, the paper's Fig. 2 and Fig. 4 scenarios).  Throughput figures
of the paper are for other hardware and are not part of the oracle.
"""

from __future__ import annotations

from collections import deque

import numpy as np

# dtypes ---------------------------------------------------------------------
F32 = "f32"
BF16 = "bf16"
_ITEMSIZE = {F32: 4, BF16: 2}

# per-handle results and per-world states --------------------------------------
DONE = "done"
PENDING = "pending"
BROKEN = "broken"
MISMATCH = "mismatch"
ALIVE = "alive"


class OracleError(Exception):
    """Argument errors; .code is one of EINVAL, ENOWORLD, EEXIST, EBROKEN."""

    def __init__(self, code, msg=""):
        super().__init__(f"{code}: {msg}")
        self.code = code


# ---------------------------------------------------------------------------
# bf16 <-> f32 (bf16 = the upper 16 bits of an IEEE-754 binary32)
# ---------------------------------------------------------------------------
def bf16_bits_to_f32(bits):
    """Widen bf16 bit patterns (uint16) to float32: exact, low 16 bits zero."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16_bits(x):
    """Round float32 to bf16, nearest with ties to even; NaN stays a quiet NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, ((u >> np.uint64(16)) | np.uint64(0x0040)).astype(np.uint16), r)
    return r


def _as_bytes(buf):
    a = np.asarray(buf)
    if a.dtype != np.uint8 or a.ndim != 1:
        raise OracleError("EINVAL", "buffers are 1-D uint8 views")
    return a


def _values_f64(raw, count, dtype):
    """Read `count` elements of `dtype` from a byte buffer as float64."""
    n = count * _ITEMSIZE[dtype]
    with np.errstate(invalid="ignore"):  # widening a signalling NaN raises the flag; the value is still a NaN
        if dtype == F32:
            return raw[:n].view(np.float32).astype(np.float64)
        return bf16_bits_to_f32(raw[:n].view(np.uint16)).astype(np.float64)


# ---------------------------------------------------------------------------
# what each operation computes (Sec. 3.3, "World Communicator")
# ---------------------------------------------------------------------------
def copy_result(src_bytes):
    """send/recv: the receiver's tensor is the sender's tensor, byte for byte."""
    return np.array(_as_bytes(src_bytes), copy=True)


def broadcast_result(bufs, root):
    """broadcast: every rank ends with the root's tensor; the root's is unchanged."""
    rootb = _as_bytes(bufs[root])
    return [np.array(rootb, copy=True) for _ in bufs]


def allreduce_sum_f64(bufs, count, dtype):
    """all-reduce (sum): element-wise sum over the ranks, taken in float64.

    Returns (s, sabs): s[i] = sum_r x_r[i] and sabs[i] = sum_r |x_r[i]|, the
    scale of the forward error bound of any summation order.
    """
    s = np.zeros(count, dtype=np.float64)
    sabs = np.zeros(count, dtype=np.float64)
    for b in bufs:
        v = _values_f64(_as_bytes(b), count, dtype)
        s += v
        sabs += np.abs(v)
    return s, sabs


def allreduce_sum_ordered(bufs, count, dtype):
    """all-reduce (sum) in float32, ranks added in ascending order
    ((x0 + x1) + x2) + ..., bf16 results rounded once, to nearest even.

    This is the arithmetic a float32 machine performs when it fixes the order;
    it is the bit-exact companion of the float64 definition above.  Returns the
    result as bytes of `dtype`.
    """
    acc = None
    for b in bufs:
        raw = _as_bytes(b)[: count * _ITEMSIZE[dtype]]
        v = raw.view(np.float32) if dtype == F32 else bf16_bits_to_f32(raw.view(np.uint16))
        acc = v.astype(np.float32) if acc is None else (acc + v).astype(np.float32)
    if dtype == F32:
        return acc.view(np.uint8).copy()
    return f32_to_bf16_bits(acc).view(np.uint8).copy()


def reduce_result_f64(bufs, count, dtype):
    """reduce (sum): what the ROOT ends with -- the same sum as all-reduce; every
    other rank's tensor is left as it was."""
    return allreduce_sum_f64(bufs, count, dtype)


def all_gather_result(send_bufs):
    """all-gather: every rank receives the ranks' tensors concatenated in rank order."""
    return np.concatenate([_as_bytes(b) for b in send_bufs])


def gather_result(send_bufs):
    """gather: the root receives the ranks' tensors concatenated in rank order."""
    return np.concatenate([_as_bytes(b) for b in send_bufs])


def scatter_result(root_send, n, rank):
    """scatter: rank r receives the r-th of n equal slices of the root's tensor."""
    raw = _as_bytes(root_send)
    if raw.size % n:
        raise OracleError("EINVAL", "scatter source is n equal slices")
    k = raw.size // n
    return np.array(raw[rank * k : (rank + 1) * k], copy=True)


def allreduce_within_tolerance(y_bytes, s, sabs, count, dtype, tol=None):
    """Check a device result y against the float64 sum s.

    Bar: |y - s| <= tol * max(sum_r |x_r|, 2**-126) per element with
    tol = 1e-6 for float32 and 1e-2 for bf16.  Returns (ok, worst) where
    worst = max |y - s| / max(sabs, 2**-126).
    """
    if tol is None:
        tol = 1e-6 if dtype == F32 else 1e-2
    y = _values_f64(_as_bytes(y_bytes), count, dtype)
    if count == 0:
        return True, 0.0
    if not np.all(np.isfinite(y)):
        return False, float("inf")
    ratio = np.abs(y - s) / np.maximum(sabs, 2.0 ** -126)
    worst = float(ratio.max())
    return worst <= tol, worst


def broken_worlds_of_worker(worlds, worker):
    """Fault domain rule (Sec. 3.1): a failed worker breaks the worlds that
    contain it and no other.  `worlds` maps world id -> iterable of workers."""
    return {w for w, members in worlds.items() if worker in members}


# ---------------------------------------------------------------------------
# the state machine
# ---------------------------------------------------------------------------
class _World:
    __slots__ = ("members", "state", "sends", "recvs", "coll", "coll_next", "coll_base")

    def __init__(self, members):
        self.members = tuple(members)
        self.state = ALIVE
        self.sends = {}  # (src, dst) -> deque of unmatched sends
        self.recvs = {}  # (src, dst) -> deque of unmatched recvs
        self.coll = deque()  # partially posted collectives, oldest first
        self.coll_base = 0  # sequence number of self.coll[0]
        self.coll_next = [0] * len(self.members)  # per rank: next collective seq


class WorldOracle:
    """Processes a trace of world operations in program order."""

    def __init__(self, n_workers):
        if n_workers <= 0:
            raise OracleError("EINVAL", "n_workers")
        self.n_workers = n_workers
        self.worlds = {}
        self.result = []  # handle -> DONE / PENDING / BROKEN / MISMATCH
        self.reduce_ref = {}  # handle -> (s, sabs) of a DONE all-reduce
        self.last_beat = {}  # worker -> time of its latest heartbeat (workers that ever sent one)
        self.dead = set()  # workers the watchdog has declared failed

    # -- world manager (Sec. 3.3 "World Manager": initialize_world) ---------
    def create(self, world, members):
        members = tuple(int(m) for m in members)
        if world in self.worlds:
            raise OracleError("EEXIST", f"world {world}")
        if len(members) < 1 or len(set(members)) != len(members):
            raise OracleError("EINVAL", "members must be distinct")
        if any(m < 0 or m >= self.n_workers for m in members):
            raise OracleError("EINVAL", "worker id out of range")
        if any(m in self.dead for m in members):
            raise OracleError("EBROKEN", "a member has been declared failed")
        self.worlds[world] = _World(members)

    def world_state(self, world):
        return self._world(world).state

    def status(self, h):
        return self.result[h]

    # -- helpers ----------------------------------------------------------------
    def _world(self, world):
        w = self.worlds.get(world)
        if w is None:
            raise OracleError("ENOWORLD", f"world {world}")
        return w

    def _new(self, st):
        self.result.append(st)
        return len(self.result) - 1

    @staticmethod
    def _check_buf(buf, count, dtype):
        if dtype not in _ITEMSIZE or count < 0:
            raise OracleError("EINVAL", "count/dtype")
        if buf is not None and _as_bytes(buf).size < count * _ITEMSIZE[dtype]:
            raise OracleError("EINVAL", "buffer shorter than count elements")

    # -- send / recv (Sec. 3.3; arrival order is arbitrary, Sec. 3.2) -------
    def _post_p2p(self, is_send, world, src, dst, buf, count, dtype):
        w = self._world(world)
        n = len(w.members)
        if not (0 <= src < n and 0 <= dst < n) or src == dst:
            raise OracleError("EINVAL", "ranks")
        self._check_buf(buf, count, dtype)
        if w.state == BROKEN:  # access to a broken world is refused
            return self._new(BROKEN)
        h = self._new(PENDING)
        mine, theirs = (w.sends, w.recvs) if is_send else (w.recvs, w.sends)
        q = theirs.get((src, dst))
        if q:
            oh, obuf, ocount, odtype = q.popleft()
            sbuf, rbuf = (buf, obuf) if is_send else (obuf, buf)
            if (ocount, odtype) != (count, dtype):
                self.result[h] = self.result[oh] = MISMATCH
            else:
                if sbuf is not None and rbuf is not None:
                    nb = count * _ITEMSIZE[dtype]
                    _as_bytes(rbuf)[:nb] = copy_result(_as_bytes(sbuf)[:nb])
                self.result[h] = self.result[oh] = DONE
        else:
            mine.setdefault((src, dst), deque()).append((h, buf, count, dtype))
        return h

    def post_send(self, world, src, dst, buf, count, dtype):
        return self._post_p2p(True, world, src, dst, buf, count, dtype)

    def post_recv(self, world, src, dst, buf, count, dtype):
        return self._post_p2p(False, world, src, dst, buf, count, dtype)

    # -- collectives (Sec. 3.3: broadcast, all-reduce) ------------------------
    _ROOTED = ("bcast", "reduce", "gather", "scatter")

    def _post_coll(self, kind, world, rank, root, buf, count, dtype, buf2=None, len1=1, len2=0):
        """buf holds len1*count elements and buf2 (if the kind has one on this rank) len2*count."""
        w = self._world(world)
        n = len(w.members)
        if not (0 <= rank < n) or (kind in self._ROOTED and not (0 <= root < n)):
            raise OracleError("EINVAL", "ranks")
        self._check_buf(buf, count * len1, dtype)
        if len2:
            self._check_buf(buf2, count * len2, dtype)
        if w.state == BROKEN:
            return self._new(BROKEN)
        h = self._new(PENDING)
        seq = w.coll_next[rank]
        w.coll_next[rank] += 1
        idx = seq - w.coll_base
        while len(w.coll) <= idx:
            w.coll.append({})
        slot = w.coll[idx]
        slot[rank] = (h, kind, root, buf, count, dtype, buf2)
        # collectives of a world execute in sequence order once all ranks posted
        while w.coll and len(w.coll[0]) == n:
            self._run_coll(w.coll.popleft(), n)
            w.coll_base += 1
        return h

    def _run_coll(self, slot, n):
        posts = [slot[r] for r in range(n)]
        hs = [p[0] for p in posts]
        sig = {(p[1], p[2], p[4], p[5]) for p in posts}
        if len(sig) != 1:
            for h in hs:
                self.result[h] = MISMATCH
            return
        kind, root, count, dtype = next(iter(sig))
        bufs = [p[3] for p in posts]
        bufs2 = [p[6] for p in posts]
        nb = count * _ITEMSIZE[dtype]
        have = all(b is not None for b in bufs)
        if kind == "bcast" and have:
            raws = [_as_bytes(b)[:nb] for b in bufs]
            out = broadcast_result(raws, root)
            for r in range(n):
                if r != root:
                    raws[r][:] = out[r]
        elif kind in ("allreduce", "reduce") and have:
            raws = [_as_bytes(b)[:nb] for b in bufs]
            s, sabs = allreduce_sum_f64(raws, count, dtype)
            for r in range(n):
                if kind == "allreduce" or r == root:
                    self.reduce_ref[hs[r]] = (s, sabs)
            if dtype == F32:
                outb = s.astype(np.float32).view(np.uint8)
            else:
                outb = f32_to_bf16_bits(s.astype(np.float32)).view(np.uint8)
            for r in range(n):
                if kind == "allreduce" or r == root:
                    raws[r][:] = outb
        elif kind == "allgather" and have and all(b is not None for b in bufs2):
            cat = all_gather_result([_as_bytes(b)[:nb] for b in bufs])  # taken before any rank is written
            for r in range(n):
                _as_bytes(bufs2[r])[: n * nb] = cat
        elif kind == "gather" and have and bufs2[root] is not None:
            _as_bytes(bufs2[root])[: n * nb] = gather_result([_as_bytes(b)[:nb] for b in bufs])
        elif kind == "scatter" and bufs[root] is not None and all(b is not None for b in bufs2):
            src = np.array(_as_bytes(bufs[root])[: n * nb], copy=True)
            for r in range(n):
                _as_bytes(bufs2[r])[:nb] = scatter_result(src, n, r)
        for h in hs:
            self.result[h] = DONE

    def post_broadcast(self, world, rank, root, buf, count, dtype):
        return self._post_coll("bcast", world, rank, root, buf, count, dtype)

    def post_allreduce(self, world, rank, buf, count, dtype):
        return self._post_coll("allreduce", world, rank, 0, buf, count, dtype)

    def post_reduce(self, world, rank, root, buf, count, dtype):
        """buf: count elements; the root's is overwritten with the sum, the others are only read."""
        return self._post_coll("reduce", world, rank, root, buf, count, dtype)

    def post_all_gather(self, world, rank, sendbuf, recvbuf, count, dtype):
        """sendbuf: count elements; recvbuf: n*count elements on every rank."""
        n = len(self._world(world).members)
        return self._post_coll("allgather", world, rank, 0, sendbuf, count, dtype, recvbuf, 1, n)

    def post_gather(self, world, rank, root, sendbuf, recvbuf, count, dtype):
        """sendbuf: count elements; recvbuf: n*count elements, used on the root only."""
        n = len(self._world(world).members)
        is_root = rank == root
        return self._post_coll("gather", world, rank, root, sendbuf, count, dtype, recvbuf if is_root else None,
                               1, n if is_root and recvbuf is not None else 0)

    def post_scatter(self, world, rank, root, sendbuf, recvbuf, count, dtype):
        """sendbuf: n*count elements, used on the root only; recvbuf: count elements on every rank."""
        n = len(self._world(world).members)
        is_root = rank == root
        return self._post_coll("scatter", world, rank, root, sendbuf if is_root else None, count, dtype, recvbuf,
                               n if is_root else 0, 1)

    # -- faults (Sec. 3.1 fault domains; Sec. 3.3 manager aborts pending ops) ---
    def abort_world(self, world):
        w = self._world(world)
        if w.state == BROKEN:
            return
        w.state = BROKEN
        for table in (w.sends, w.recvs):
            for q in table.values():
                for item in q:
                    self.result[item[0]] = BROKEN
            table.clear()
        for slot in w.coll:
            for post in slot.values():
                self.result[post[0]] = BROKEN
        w.coll.clear()

    # -- watchdog (Sec. 3.3 "Watchdog"): workers report their health periodically; one whose
    #    reports have been missing for longer than the timeout is taken to have failed, and the
    #    worlds it belongs to are cleaned up.  Time is an explicit argument here.
    def heartbeat(self, worker, t):
        if not (0 <= worker < self.n_workers):
            raise OracleError("EINVAL", "worker id out of range")
        if worker in self.dead:
            raise OracleError("EBROKEN", "worker has been declared failed")
        self.last_beat[worker] = max(t, self.last_beat.get(worker, t))

    def watchdog_check(self, t, timeout):
        """One inspection at time t: returns the workers newly declared failed (ascending)."""
        late = sorted(k for k, tb in self.last_beat.items() if k not in self.dead and t - tb > timeout)
        for k in late:
            self.dead.add(k)
            self.abort_worker(k)
        return late

    def abort_worker(self, worker):
        if not (0 <= worker < self.n_workers):
            raise OracleError("EINVAL", "worker id out of range")
        members = {wid: w.members for wid, w in self.worlds.items()}
        for wid in sorted(broken_worlds_of_worker(members, worker)):
            self.abort_world(wid)
