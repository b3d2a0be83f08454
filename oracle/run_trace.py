"""Feed a trace (see workloads.trace) to the CPU oracle.

TEST INFRASTRUCTURE ONLY.  The trace object is read by attribute; the caller
passes the function that turns a buffer spec into bytes, so this module
imports nothing but the oracle and numpy.
"""

from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from .mw_oracle import BROKEN, DONE, OracleError, WorldOracle


@dataclass
class OracleRun:
    status: dict = field(default_factory=dict)  # posting op index -> terminal status
    snapshots: dict = field(default_factory=dict)  # check op index -> bytes (None if data skipped)
    reduce_ref: dict = field(default_factory=dict)  # check op index -> (s, sabs, count, dtype)
    world_state: dict = field(default_factory=dict)  # world id -> state at end of trace
    payload_bytes_done: int = 0


def run_trace(trace, materialize, data_bufs=None):
    """Process `trace` in program order.  Buffers whose id is not in `data_bufs`
    (default: trace.meta['data_bufs'], else all) carry no data: their operations
    still take part in matching and fault handling."""
    if data_bufs is None:
        data_bufs = trace.meta.get("data_bufs")
    orc = WorldOracle(trace.n_workers)
    out = OracleRun()
    live = {}
    handle_of = {}
    last_post = {}  # buf -> posting op index that touched it last
    itemsize = {"f32": 4, "bf16": 2}

    def get(buf):
        if data_bufs is not None and buf not in data_bufs:
            return None
        a = live.get(buf)
        if a is None:
            a = np.array(materialize(trace.bufs[buf]), dtype=np.uint8, copy=True)
            live[buf] = a
        return a

    for idx, op in enumerate(trace.ops):
        k = op.kind
        if k == "create":
            orc.create(op.world, op.members)
        elif k in ("send", "recv", "bcast", "allreduce", "reduce", "allgather", "gather", "scatter"):
            b = get(op.buf) if op.buf >= 0 else None
            b2 = get(op.buf2) if op.buf2 >= 0 else None
            if k == "send":
                h = orc.post_send(op.world, op.a, op.b, b, op.count, op.dtype)
            elif k == "recv":
                h = orc.post_recv(op.world, op.a, op.b, b, op.count, op.dtype)
            elif k == "bcast":
                h = orc.post_broadcast(op.world, op.a, op.b, b, op.count, op.dtype)
            elif k == "allreduce":
                h = orc.post_allreduce(op.world, op.a, b, op.count, op.dtype)
            elif k == "reduce":
                h = orc.post_reduce(op.world, op.a, op.b, b, op.count, op.dtype)
            elif k == "allgather":
                h = orc.post_all_gather(op.world, op.a, b, b2, op.count, op.dtype)
            elif k == "gather":
                h = orc.post_gather(op.world, op.a, op.b, b, b2, op.count, op.dtype)
            else:
                h = orc.post_scatter(op.world, op.a, op.b, b, b2, op.count, op.dtype)
            handle_of[idx] = h
            for bid in (op.buf, op.buf2):
                if bid >= 0:
                    last_post[bid] = idx
        elif k == "abort_world":
            orc.abort_world(op.world)
        elif k == "abort_worker":
            orc.abort_worker(op.a)
        elif k == "check":
            a = get(op.buf)
            out.snapshots[idx] = None if a is None else a.copy()
            p = last_post.get(op.buf)
            if p is not None and trace.ops[p].kind in ("allreduce", "reduce") and orc.status(handle_of[p]) == DONE:
                ref = orc.reduce_ref.get(handle_of[p])
                if ref is not None:
                    out.reduce_ref[idx] = (ref[0], ref[1], trace.ops[p].count, trace.ops[p].dtype)
        elif k == "restore":
            if op.buf in live:
                live[op.buf][:] = materialize(trace.bufs[op.buf])
            last_post.pop(op.buf, None)
        elif k == "free":
            live.pop(op.buf, None)
            last_post.pop(op.buf, None)
        elif k in ("wait", "flush"):
            pass
        else:
            raise OracleError("EINVAL", f"unknown trace op {k}")

    for idx, h in handle_of.items():
        st = orc.status(h)
        out.status[idx] = st
        op = trace.ops[idx]
        if st == DONE and (op.kind == "recv" or (op.kind not in ("send", "recv") and op.a == 0)):
            out.payload_bytes_done += op.count * itemsize[op.dtype]
    out.world_state = {w: orc.world_state(w) for w in orc.worlds}
    return out


__all__ = ["OracleRun", "run_trace", "BROKEN", "DONE"]
