"""The five workloads as seeded traces.

Every generator takes the full-size parameters as defaults and lets a caller
shrink shapes and lengths so that a CPU reference finishes in seconds while the
structure (topology, op mix, posting order, abort positions) stays the same.

Shapes follow serving traffic: pipeline-stage activation hand-offs
[batch, seq, hidden] in bf16, tensor-parallel partial sums in fp32, fan-in from
replicated partition workers, and a mixed scale-out soup.
"""

from __future__ import annotations

import math

import numpy as np

from .data import ITEMSIZE, POOL_ELEMS, rng_of
from .trace import Op, Trace

BASE_SEED = 20240708
POISON = 0xA5
_POOL_FROM = 1 << 20  # tensors with at least this many elements are cut from the pool


def _numel(shape):
    n = 1
    for s in shape:
        n *= int(s)
    return n


class _Seeds:
    """Distinct per-buffer seeds derived from the config's seed."""

    def __init__(self, cfg):
        self.base = (BASE_SEED + cfg) * 1_000_003
        self.k = 0
        self.rng = rng_of(BASE_SEED + cfg)

    def next(self):
        self.k += 1
        return self.base + self.k


def _payload_init(kind, dtype, count, seeds):
    """N(0,1)/U(-1,1) tensor: drawn directly when small, cut from the pool when large."""
    if kind == "normal" and count >= _POOL_FROM:
        return ("pool", dtype, int(seeds.rng.integers(0, POOL_ELEMS)))
    return (kind, dtype, seeds.next())


# ---------------------------------------------------------------------------
# config 1: two worlds over three workers, the leader in both
# ---------------------------------------------------------------------------
def config1(n_msgs=200, shape=(8, 1024), window=16):
    """Worker 0 is rank 0 of world 0 = (0, 1) and of world 1 = (0, 2).  Message k
    travels peer -> worker 0 in world k mod 2; for odd floor(k/2) the recv is
    posted before the send, otherwise after.  Then each world does one
    broadcast from rank 0 and one all-reduce."""
    t = Trace("config1", n_workers=3, n_streams=2)
    sd = _Seeds(1)
    count = _numel(shape)
    t.create(0, (0, 1))
    t.create(1, (0, 2))
    dsts = []
    for k in range(n_msgs):
        w = k % 2
        src = t.tensor(count, "f32", ("normal", "f32", sd.next()))
        dst = t.tensor(count, "f32", ("fill", POISON))
        dsts.append(dst)
        if (k // 2) % 2 == 1:
            t.recv(w, 1, 0, dst, count, "f32", stream=w)
            t.send(w, 1, 0, src, count, "f32", stream=w)
        else:
            t.send(w, 1, 0, src, count, "f32", stream=w)
            t.recv(w, 1, 0, dst, count, "f32", stream=w)
        if (k + 1) % window == 0:
            t.wait()
    t.wait()
    for d in dsts:
        t.check(d)
    coll = []
    for w in (0, 1):
        bb = [t.tensor(count, "f32", ("normal", "f32", sd.next())) for _ in range(2)]
        for r in (1, 0):
            t.bcast(w, r, 0, bb[r], count, "f32", stream=w)
        ab = [t.tensor(count, "f32", ("normal", "f32", sd.next())) for _ in range(2)]
        for r in (0, 1):
            t.allreduce(w, r, ab[r], count, "f32", stream=w)
        coll += bb + ab
    t.wait()
    for b in coll:
        t.check(b)
    t.meta.update(shape=tuple(shape), n_msgs=n_msgs)
    return t


# ---------------------------------------------------------------------------
# config 2: pipeline-stage activation hand-off, 8 producer -> consumer worlds
# ---------------------------------------------------------------------------
def config2(shape=(32, 2048, 4096), steps=50, n_worlds=8, pool_k=4, check_steps=None):
    """World i = (worker 2i -> worker 2i+1).  Step s of every world is outstanding
    together; world i posts on stream i.  Sources cycle through pool_k tensors,
    destinations are double-buffered and poisoned before a checked step."""
    t = Trace("config2", n_workers=2 * n_worlds, n_streams=n_worlds)
    sd = _Seeds(2)
    count = _numel(shape)
    if check_steps is None:
        check_steps = range(steps)
    check_steps = set(check_steps)
    src = [[t.tensor(count, "bf16", _payload_init("normal", "bf16", count, sd)) for _ in range(pool_k)]
           for _ in range(n_worlds)]
    dst = [[t.tensor(count, "bf16", ("fill", POISON)) for _ in range(2)] for _ in range(n_worlds)]
    for i in range(n_worlds):
        t.create(i, (2 * i, 2 * i + 1))
    for s in range(steps):
        if s in check_steps:
            for i in range(n_worlds):
                t.restore(dst[i][s % 2])
        for i in range(n_worlds):
            t.send(i, 0, 1, src[i][s % pool_k], count, "bf16", stream=i)
            t.recv(i, 0, 1, dst[i][s % 2], count, "bf16", stream=i)
        if s in check_steps:
            t.wait()
            for i in range(n_worlds):
                t.check(dst[i][s % 2])
        elif s % 2 == 1:
            t.wait()
    t.wait()
    t.meta.update(shape=tuple(shape), steps=steps, n_worlds=n_worlds)
    return t


# ---------------------------------------------------------------------------
# config 3: tensor-parallel partial-sum all-reduce, 4 worlds x 4 ranks
# ---------------------------------------------------------------------------
def config3(shapes=((16, 4096), (16, 14336)), iters=500, n_worlds=4, n_ranks=4, pool_k=4,
            check_iters=None, dtype="f32"):
    """Each iteration every world all-reduces one tensor of each shape; all worlds
    are outstanding together.  Inputs are U(-1,1), pool_k sets per rank, restored
    before reuse because the operation is in place."""
    t = Trace("config3", n_workers=n_worlds * n_ranks, n_streams=n_worlds)
    sd = _Seeds(3)
    if check_iters is None:
        check_iters = range(iters)
    check_iters = set(check_iters)
    counts = [_numel(s) for s in shapes]
    bufs = [[[[t.tensor(c, dtype, ("uniform", dtype, sd.next())) for c in counts]
              for _ in range(pool_k)] for _ in range(n_ranks)] for _ in range(n_worlds)]
    for w in range(n_worlds):
        t.create(w, tuple(range(w * n_ranks, (w + 1) * n_ranks)))
    for it in range(iters):
        k = it % pool_k
        if it >= pool_k:
            for w in range(n_worlds):
                for r in range(n_ranks):
                    for j in range(len(counts)):
                        t.restore(bufs[w][r][k][j])
        for j, c in enumerate(counts):
            for w in range(n_worlds):
                for r in range(n_ranks):
                    t.allreduce(w, r, bufs[w][r][k][j], c, dtype, stream=w)
        t.wait()
        if it in check_iters:
            for w in range(n_worlds):
                for r in range(n_ranks):
                    for j in range(len(counts)):
                        t.check(bufs[w][r][k][j])
    t.meta.update(shapes=tuple(tuple(s) for s in shapes), iters=iters, n_worlds=n_worlds, n_ranks=n_ranks)
    return t


# ---------------------------------------------------------------------------
# config 4: elastic fan-in with a fault
# ---------------------------------------------------------------------------
def config4(shape=(8, 2048, 5120), steps=300, n_worlds=16, abort_worker=7, abort_step=100, pool_k=4,
            check_steps=None):
    """Workers 0..n-1 are replicated partition workers, worker n is the one shared
    consumer; world i = (worker i as rank 0 -> consumer as rank 1).  Steps are
    0-based; `abort_worker` is aborted before anything of step `abort_step` is
    posted, and its world keeps being attempted afterwards."""
    t = Trace("config4", n_workers=n_worlds + 1, n_streams=n_worlds)
    sd = _Seeds(4)
    count = _numel(shape)
    if check_steps is None:
        check_steps = range(steps)
    check_steps = set(check_steps)
    src = [[t.tensor(count, "bf16", _payload_init("normal", "bf16", count, sd)) for _ in range(pool_k)]
           for _ in range(n_worlds)]
    dst = [[t.tensor(count, "bf16", ("fill", POISON)) for _ in range(2)] for _ in range(n_worlds)]
    for i in range(n_worlds):
        t.create(i, (i, n_worlds))
    for s in range(steps):
        if s == abort_step:
            t.abort_worker(abort_worker)
        if s in check_steps:
            for i in range(n_worlds):
                t.restore(dst[i][s % 2])
        for i in range(n_worlds):
            t.send(i, 0, 1, src[i][s % pool_k], count, "bf16", stream=i)
            t.recv(i, 0, 1, dst[i][s % 2], count, "bf16", stream=i)
        if s in check_steps:
            t.wait()
            for i in range(n_worlds):
                t.check(dst[i][s % 2])
        elif s % 2 == 1:
            t.wait()
    t.wait()
    t.meta.update(shape=tuple(shape), steps=steps, n_worlds=n_worlds, abort_worker=abort_worker,
                  abort_step=abort_step)
    return t


# ---------------------------------------------------------------------------
# config 5: mixed scale-out
# ---------------------------------------------------------------------------
def config5(n_ops=10_000, n_worlds=64, n_workers=32, min_bytes=4096, max_bytes=1 << 26, window=64,
            n_aborts=3, check_small=1 << 20, check_fraction=0.05, check_all=False):
    """n_worlds worlds of 2-4 members sampled without replacement; each op picks a
    world uniformly (already-broken ones included), a kind 70/20/10 % send-recv /
    broadcast / all-reduce, fp32 or bf16, a byte size log-uniform in
    [min_bytes, max_bytes] (element counts are not rounded to 16 bytes), ranks
    uniformly, and a seeded posting order of its sides.  n_aborts distinct workers
    are aborted before seeded op indices.  Operations use fresh buffers; up to
    `window` are outstanding together.  Data of an operation is checked when its
    payload is at most check_small bytes, else with probability check_fraction."""
    t = Trace("config5", n_workers=n_workers, n_streams=4)
    sd = _Seeds(5)
    rng = sd.rng
    members = []
    for w in range(n_worlds):
        size = int(rng.integers(2, 5))
        m = tuple(int(x) for x in rng.choice(n_workers, size=size, replace=False))
        members.append(m)
        t.create(w, m)
    victims = [int(x) for x in rng.choice(n_workers, size=n_aborts, replace=False)]
    abort_at = {}
    for v in victims:
        abort_at.setdefault(int(rng.integers(0, n_ops)), []).append(v)
    data_bufs = set()
    live = []  # (buffers, checked) of the current window
    lo, hi = math.log(min_bytes), math.log(max_bytes)
    kinds = np.array(["p2p", "bcast", "allreduce"])

    def close_window():
        t.wait()
        for bufs, checked in live:
            if checked:
                for b in bufs:
                    t.check(b)
        for bufs, _ in live:
            for b in bufs:
                t.free(b)
        live.clear()

    for i in range(n_ops):
        for v in abort_at.get(i, ()):
            t.abort_worker(v)
        w = int(rng.integers(0, n_worlds))
        n = len(members[w])
        kind = str(rng.choice(kinds, p=[0.7, 0.2, 0.1]))
        dtype = "f32" if rng.integers(0, 2) == 0 else "bf16"
        isz = ITEMSIZE[dtype]
        count = int(math.exp(rng.uniform(lo, hi))) // isz
        nbytes = count * isz
        checked = check_all or nbytes <= check_small or rng.random() < check_fraction
        stream = int(rng.integers(0, t.n_streams))
        bufs = []
        if kind == "p2p":
            src, dst = (int(x) for x in rng.choice(n, size=2, replace=False))
            sb = t.tensor(count, dtype, ("pool", dtype, int(rng.integers(0, POOL_ELEMS))))
            db = t.tensor(count, dtype, ("fill", POISON))
            bufs = [sb, db]
            if rng.integers(0, 2) == 0:
                t.send(w, src, dst, sb, count, dtype, stream)
                t.recv(w, src, dst, db, count, dtype, stream)
            else:
                t.recv(w, src, dst, db, count, dtype, stream)
                t.send(w, src, dst, sb, count, dtype, stream)
        else:
            root = int(rng.integers(0, n))
            order = [int(x) for x in rng.permutation(n)]
            for r in range(n):
                if kind == "bcast" and r != root:
                    bufs.append(t.tensor(count, dtype, ("fill", POISON)))
                else:
                    bufs.append(t.tensor(count, dtype, ("pool", dtype, int(rng.integers(0, POOL_ELEMS)))))
            for r in order:
                if kind == "bcast":
                    t.bcast(w, r, root, bufs[r], count, dtype, stream)
                else:
                    t.allreduce(w, r, bufs[r], count, dtype, stream)
        if checked:
            data_bufs.update(bufs)
        live.append((bufs, checked))
        if len(live) == window:
            close_window()
    close_window()
    t.meta.update(members=members, victims=victims, abort_at=abort_at, data_bufs=data_bufs, n_ops=n_ops)
    return t


# ---------------------------------------------------------------------------
# all eight operations of the communicator, mixed
# ---------------------------------------------------------------------------
def collectives_mix(n_ops=400, n_worlds=12, n_workers=16, min_bytes=64, max_bytes=1 << 20, window=24, n_aborts=2,
                    max_ranks=4, seed_offset=6):
    """Worlds of 2..max_ranks members; every op is one of send-recv, broadcast, all-reduce, reduce,
    all-gather, gather, scatter (uniformly), fp32 or bf16, log-uniform size, seeded posting order;
    n_aborts workers are aborted at seeded positions.  Every op uses fresh buffers and is checked."""
    t = Trace("collectives_mix", n_workers=n_workers, n_streams=3)
    sd = _Seeds(seed_offset)
    rng = sd.rng
    members = []
    for w in range(n_worlds):
        size = int(rng.integers(2, max_ranks + 1))
        m = tuple(int(x) for x in rng.choice(n_workers, size=size, replace=False))
        members.append(m)
        t.create(w, m)
    abort_at = {}
    for v in rng.choice(n_workers, size=n_aborts, replace=False):
        abort_at.setdefault(int(rng.integers(n_ops // 3, n_ops)), []).append(int(v))
    live = []
    lo, hi = math.log(min_bytes), math.log(max_bytes)
    kinds = ["p2p", "bcast", "allreduce", "reduce", "allgather", "gather", "scatter"]

    def close_window():
        t.wait()
        for bufs in live:
            for b in bufs:
                t.check(b)
        for bufs in live:
            for b in bufs:
                t.free(b)
        live.clear()

    for i in range(n_ops):
        for v in abort_at.get(i, ()):
            t.abort_worker(v)
        w = int(rng.integers(0, n_worlds))
        n = len(members[w])
        kind = kinds[int(rng.integers(0, len(kinds)))]
        dtype = "f32" if rng.integers(0, 2) == 0 else "bf16"
        isz = ITEMSIZE[dtype]
        count = max(1, int(math.exp(rng.uniform(lo, hi))) // isz)
        stream = int(rng.integers(0, t.n_streams))
        order = [int(x) for x in rng.permutation(n)]
        root = int(rng.integers(0, n))
        draw = lambda c: t.tensor(c, dtype, ("uniform", dtype, sd.next()))
        poison = lambda c: t.tensor(c, dtype, ("fill", POISON))
        bufs = []
        if kind == "p2p":
            src, dst = (int(x) for x in rng.choice(n, size=2, replace=False))
            sb, db = draw(count), poison(count)
            bufs = [sb, db]
            t.recv(w, src, dst, db, count, dtype, stream)
            t.send(w, src, dst, sb, count, dtype, stream)
        elif kind in ("bcast", "allreduce", "reduce"):
            bufs = [draw(count) if (kind != "bcast" or r == root) else poison(count) for r in range(n)]
            for r in order:
                if kind == "bcast":
                    t.bcast(w, r, root, bufs[r], count, dtype, stream)
                elif kind == "allreduce":
                    t.allreduce(w, r, bufs[r], count, dtype, stream)
                else:
                    t.reduce(w, r, root, bufs[r], count, dtype, stream)
        elif kind == "allgather":
            sends = [draw(count) for _ in range(n)]
            recvs = [poison(n * count) for _ in range(n)]
            bufs = sends + recvs
            for r in order:
                t.allgather(w, r, sends[r], recvs[r], count, dtype, stream)
        elif kind == "gather":
            sends = [draw(count) for _ in range(n)]
            recv = poison(n * count)
            bufs = sends + [recv]
            for r in order:
                t.gather(w, r, root, sends[r], recv if r == root else -1, count, dtype, stream)
        else:
            send = draw(n * count)
            recvs = [poison(count) for _ in range(n)]
            bufs = [send] + recvs
            for r in order:
                t.scatter(w, r, root, send if r == root else -1, recvs[r], count, dtype, stream)
        live.append(bufs)
        if len(live) == window:
            close_window()
    close_window()
    t.meta.update(members=members, abort_at=abort_at, n_ops=n_ops)
    return t


# ---------------------------------------------------------------------------
# online instantiation and recovery under load (the paper's Sec. 3.1 / Fig. 2 and Sec. 4.2 / Fig. 5 in shape)
# ---------------------------------------------------------------------------
def online_recovery(count=1_000_000, window=4, rounds=2):
    """The rhombus of Fig. 2: P1 -> {P2, P3} -> P4 with one world per edge, fp32 tensors of `count` elements
    (4 MB in Sec. 4.2).  Workers 0..3 are P1..P4, worker 4 is the replacement P5.

      phase 1  only the P2 path exists (worlds 1 = (P1,P2), 3 = (P2,P4)) and streams windows;
      phase 2  with a window of the P2 path in flight, worlds 2 = (P1,P3) and 4 = (P3,P4) are created
               (online instantiation) and all four worlds stream;
      phase 3  a window is posted in all four worlds, the P3 worlds also get receives whose tensors never
               come; with that window in flight P3 fails: what was matched is delivered, the rest is broken,
               later posts to its worlds are refused, the P2 path streams on;
      phase 4  with a window of the P2 path in flight, P5 takes P3's place through two NEW worlds
               6 = (P1,P5) and 7 = (P5,P4) (Fig. 2(c)); all healthy worlds stream.

    Every destination is checked."""
    t = Trace("online_recovery", n_workers=5, n_streams=2)
    sd = _Seeds(7)
    dsts = []

    def window_of(worlds, orphans=()):
        """One window: `window` messages rank 0 -> rank 1 in each of `worlds`; `orphans` get one recv more."""
        for j in range(window):
            for w in worlds:
                src = t.tensor(count, "f32", _payload_init("normal", "f32", count, sd))
                dst = t.tensor(count, "f32", ("fill", POISON))
                dsts.append(dst)
                if j % 2:
                    t.recv(w, 0, 1, dst, count, "f32", stream=w % 2)
                    t.send(w, 0, 1, src, count, "f32", stream=w % 2)
                else:
                    t.send(w, 0, 1, src, count, "f32", stream=w % 2)
                    t.recv(w, 0, 1, dst, count, "f32", stream=w % 2)
        for w in orphans:
            dst = t.tensor(count, "f32", ("fill", POISON))
            dsts.append(dst)
            t.recv(w, 0, 1, dst, count, "f32", stream=w % 2)

    t.create(1, (0, 1))
    t.create(3, (1, 3))
    for _ in range(rounds):
        window_of((1, 3))
        t.wait()
    window_of((1, 3))
    t.flush()
    t.create(2, (0, 2))  # while the window above is in flight
    t.create(4, (2, 3))
    for _ in range(rounds):
        window_of((1, 2, 3, 4))
        t.wait()
    window_of((1, 2, 3, 4), orphans=(2, 4))
    t.flush()
    t.abort_worker(2)  # P3
    window_of((1, 2, 3, 4))  # worlds 2 and 4 refuse
    t.wait()
    window_of((1, 3))
    t.flush()
    t.create(6, (0, 4))  # P5 joins through new worlds while the P2 path has a window in flight
    t.create(7, (4, 3))
    for _ in range(rounds):
        window_of((1, 3, 6, 7))
        t.wait()
    for d in dsts:
        t.check(d)
    t.meta.update(count=count, window=window, rounds=rounds)
    return t


# ---------------------------------------------------------------------------
# the multi-sender experiment in shape (Sec. 4.3 / Fig. 7)
# ---------------------------------------------------------------------------
def multi_sender(senders, count, multi_world, window=8, n_windows=2):
    """`senders` workers (1..3) each send fp32 tensors of `count` elements to worker 0, `window` messages per
    sender outstanding together.  multi_world: one world per sender, (receiver, sender k), the receiver in all of
    them; otherwise one world holding the receiver and every sender."""
    t = Trace(f"multi_sender_{senders}_{count}_{'mw' if multi_world else 'sw'}", n_workers=senders + 1, n_streams=senders)
    sd = _Seeds(8 + senders)
    if multi_world:
        for k in range(senders):
            t.create(k, (0, 1 + k))
    else:
        t.create(0, tuple(range(senders + 1)))
    dsts = []
    for _ in range(n_windows):
        for j in range(window):
            for k in range(senders):
                w, a = (k, 1) if multi_world else (0, 1 + k)
                src = t.tensor(count, "f32", _payload_init("normal", "f32", count, sd))
                dst = t.tensor(count, "f32", ("fill", POISON))
                dsts.append(dst)
                t.recv(w, a, 0, dst, count, "f32", stream=k)
                t.send(w, a, 0, src, count, "f32", stream=k)
        t.wait()
    for d in dsts:
        t.check(d)
    t.meta.update(senders=senders, count=count, multi_world=multi_world)
    return t


# ---------------------------------------------------------------------------
# single-world baseline of a point-to-point trace
# ---------------------------------------------------------------------------
def single_world_of(trace, drop_aborts=True):
    """The same messages in the same order through ONE world whose ranks are all
    workers (rank == worker id): the single-world setup the paper compares
    against.  Only point-to-point traces can be mapped (a collective changes
    meaning in a bigger world)."""
    members = {}
    out = Trace(trace.name + "_single_world", trace.n_workers, trace.n_streams, dict(trace.bufs), [],
                dict(trace.meta))
    out.create(0, tuple(range(trace.n_workers)))
    for op in trace.ops:
        if op.kind == "create":
            members[op.world] = op.members
        elif op.kind in ("send", "recv"):
            m = members[op.world]
            out.add(Op(op.kind, 0, m[op.a], m[op.b], op.buf, op.count, op.dtype, op.stream))
        elif op.kind in ("bcast", "allreduce", "reduce", "allgather", "gather", "scatter"):
            raise ValueError("single_world_of maps point-to-point traces only")
        elif op.kind == "abort_worker":
            if not drop_aborts:
                out.add(Op("abort_worker", a=op.a))
        elif op.kind == "abort_world":
            if not drop_aborts:
                out.add(Op("abort_world", world=0))
        else:
            out.add(op)
    return out
