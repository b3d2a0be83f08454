"""Trace = a program-ordered list of operations over logical workers and worlds.

Posting operations (send / recv / bcast / allreduce) are identified by their
position in Trace.ops; runners report one terminal status per such position.
Buffers are referred to by integer id; a buffer comes into existence with its
spec's initial bytes the first time an operation names it and lives until a
"free" operation.  "wait" asks the runner to let everything outstanding reach
a terminal state (the reference semantics are sequential, so it means nothing
there); "flush" asks it to start what can be started without waiting for it
(likewise nothing there): what follows in the trace then happens while those
operations are in flight; "check" asks for a snapshot of a buffer at that point of the trace;
"restore" rewrites a buffer with its initial bytes.
"""

from __future__ import annotations

from dataclasses import dataclass, field

from .data import ITEMSIZE, BufSpec

POSTING = ("send", "recv", "bcast", "allreduce", "reduce", "allgather", "gather", "scatter")


@dataclass
class Op:
    kind: str  # create send recv bcast allreduce ... abort_world abort_worker wait flush check restore free
    world: int = -1
    a: int = -1  # p2p: src rank; collectives: posting rank; abort_worker: worker id
    b: int = -1  # p2p: dst rank; bcast: root rank
    buf: int = -1
    count: int = 0
    dtype: str = "f32"
    stream: int = 0  # which of the runner's caller-side streams the post is ordered after
    members: tuple = ()
    buf2: int = -1  # allgather / gather: receive buffer; scatter: receive buffer (buf is then the root's source)


@dataclass
class Trace:
    name: str
    n_workers: int
    n_streams: int = 1
    bufs: dict = field(default_factory=dict)
    ops: list = field(default_factory=list)
    meta: dict = field(default_factory=dict)

    # -- builders -----------------------------------------------------------
    def buf(self, nbytes, init):
        i = len(self.bufs)
        self.bufs[i] = BufSpec(int(nbytes), tuple(init))
        return i

    def tensor(self, count, dtype, init):
        return self.buf(count * ITEMSIZE[dtype], init)

    def add(self, op):
        self.ops.append(op)
        return len(self.ops) - 1

    def create(self, world, members):
        return self.add(Op("create", world=world, members=tuple(members)))

    def send(self, world, src, dst, buf, count, dtype, stream=0):
        return self.add(Op("send", world, src, dst, buf, count, dtype, stream))

    def recv(self, world, src, dst, buf, count, dtype, stream=0):
        return self.add(Op("recv", world, src, dst, buf, count, dtype, stream))

    def bcast(self, world, rank, root, buf, count, dtype, stream=0):
        return self.add(Op("bcast", world, rank, root, buf, count, dtype, stream))

    def allreduce(self, world, rank, buf, count, dtype, stream=0):
        return self.add(Op("allreduce", world, rank, -1, buf, count, dtype, stream))

    def reduce(self, world, rank, root, buf, count, dtype, stream=0):
        return self.add(Op("reduce", world, rank, root, buf, count, dtype, stream))

    def allgather(self, world, rank, sendbuf, recvbuf, count, dtype, stream=0):
        return self.add(Op("allgather", world, rank, -1, sendbuf, count, dtype, stream, (), recvbuf))

    def gather(self, world, rank, root, sendbuf, recvbuf, count, dtype, stream=0):
        """recvbuf is -1 on every rank but the root."""
        return self.add(Op("gather", world, rank, root, sendbuf, count, dtype, stream, (), recvbuf))

    def scatter(self, world, rank, root, sendbuf, recvbuf, count, dtype, stream=0):
        """sendbuf is -1 on every rank but the root."""
        return self.add(Op("scatter", world, rank, root, sendbuf, count, dtype, stream, (), recvbuf))

    def abort_world(self, world):
        return self.add(Op("abort_world", world=world))

    def abort_worker(self, worker):
        return self.add(Op("abort_worker", a=worker))

    def wait(self):
        return self.add(Op("wait"))

    def flush(self):
        return self.add(Op("flush"))

    def check(self, buf):
        return self.add(Op("check", buf=buf))

    def restore(self, buf):
        return self.add(Op("restore", buf=buf))

    def free(self, buf):
        return self.add(Op("free", buf=buf))

    # -- facts about the trace ------------------------------------------------
    def posting_indices(self):
        return [i for i, op in enumerate(self.ops) if op.kind in POSTING]

    def payload_bytes(self):
        """Payload bytes if every operation completed: one S per send/recv pair and
        per collective (counted once on its rank-0 post)."""
        total = 0
        for op in self.ops:
            if op.kind == "recv" or (op.kind in POSTING[2:] and op.a == 0):
                total += op.count * ITEMSIZE[op.dtype]
        return total
