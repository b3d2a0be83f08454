"""Run a workload trace through the library on the GPU.

Harness code: it allocates device buffers (torch is used for memory and streams
only), posts the trace's operations through the C ABI, polls, and returns per-post
terminal states and buffer snapshots.  Every byte that moves between buffers is
moved by the library's kernels.
"""

from __future__ import annotations

import time
from dataclasses import dataclass, field

import numpy as np
import torch

from . import binding as mw

STATE_NAME = {mw.MW_DONE: "done", mw.MW_PENDING: "pending", mw.MW_BROKEN: "broken", mw.MW_EMISMATCH: "mismatch"}
ITEMSIZE = {"f32": 4, "bf16": 2}


@dataclass
class DeviceRun:
    status: dict = field(default_factory=dict)      # posting op index -> "done" / "pending" / "broken" / "mismatch"
    snapshots: dict = field(default_factory=dict)   # check op index -> np.uint8 array
    world_state: dict = field(default_factory=dict)
    seconds: float = 0.0
    payload_bytes_done: int = 0


class DevicePools:
    """The host N(0,1) pools uploaded once; pool-backed buffers are cut from them on the device."""

    def __init__(self, host_pools, device):
        self.host = host_pools
        self.device = device
        self._dev = {}

    def slice(self, dtype, offset, nbytes, out):
        p = self._dev.get(dtype)
        if p is None:
            p = torch.from_numpy(self.host.get(dtype)).to(self.device)
            self._dev[dtype] = p
        total = p.numel()
        start = (offset * ITEMSIZE[dtype]) % total
        done = 0
        while done < nbytes:
            take = min(nbytes - done, total - start)
            out[done:done + take].copy_(p[start:start + take])
            done += take
            start = 0


def _fill(spec, tensor, pools, materialize):
    kind = spec.init[0]
    if kind == "fill":
        tensor.fill_(spec.init[1])
    elif kind == "pool":
        pools.slice(spec.init[1], spec.init[2], spec.nbytes, tensor)
    else:
        tensor.copy_(torch.from_numpy(materialize(spec)))


def wait_all(outstanding, status, timeout_s=120.0):
    """Poll until no posted operation can still make progress; terminal handles leave `outstanding`."""
    mw.mw_flush()
    t0 = time.time()
    while True:
        if outstanding:
            ps = mw.PollSet([h for _, h in outstanding])
            ps.poll()
            keep = []
            for (idx, h), st in zip(outstanding, ps.states):
                if st == mw.MW_PENDING:
                    keep.append((idx, h))
                else:
                    status[idx] = STATE_NAME.get(st, f"error{st}")
            outstanding[:] = keep
        if mw.mw_pending_ops() == 0:
            return
        if time.time() - t0 > timeout_s:
            raise TimeoutError(f"{mw.mw_pending_ops()} operations did not complete within {timeout_s} s")


def run_trace(trace, host_pools, materialize, device=0, snapshots=True, check_fn=None, on_init=None, on_exit=None,
              settle=False):
    """Execute `trace`; returns a DeviceRun.  mw_init / mw_shutdown bracket the run.

    check_fn(idx, op, bufs), if given, is called at every "check" op with the dict of live device
    tensors (buffer id -> uint8 tensor) once everything outstanding has completed; use it with
    snapshots=False to verify large buffers on the device instead of copying them out.
    on_init() / on_exit() run right after mw_init and right before mw_shutdown (e.g. to run the watchdog).
    settle=True finishes every buffer initialisation before the operation that uses it is posted, so that the
    operation finds its caller stream idle and depends on nothing (the resident mailbox kernel serves only such)."""
    dev = torch.device("cuda", device)
    torch.cuda.set_device(dev)
    pools = DevicePools(host_pools, dev)
    streams = [torch.cuda.Stream(device=dev) for _ in range(trace.n_streams)]
    cur = torch.cuda.current_stream(dev)
    out = DeviceRun()
    bufs = {}
    outstanding = []
    touched = False  # buffers were (re)initialised on torch's stream since the last ordering point

    def get(buf):
        nonlocal touched
        t = bufs.get(buf)
        if t is None:
            spec = trace.bufs[buf]
            t = torch.empty(max(spec.nbytes, 1), dtype=torch.uint8, device=dev)[: spec.nbytes]
            _fill(spec, t, pools, materialize)
            bufs[buf] = t
            touched = True
        return t

    mw.mw_init(device, trace.n_workers)
    try:
        if on_init is not None:
            on_init()
        t_start = time.time()
        for idx, op in enumerate(trace.ops):
            k = op.kind
            if k in ("send", "recv", "bcast", "allreduce", "reduce", "allgather", "gather", "scatter"):
                t = get(op.buf) if op.buf >= 0 else None
                t2 = get(op.buf2) if op.buf2 >= 0 else None
                p1 = t.data_ptr() if t is not None else None
                p2 = t2.data_ptr() if t2 is not None else None
                s = streams[op.stream]
                if touched:  # make every caller stream see the initialised bytes
                    if settle:
                        torch.cuda.synchronize(dev)
                    else:
                        for st in streams:
                            st.wait_stream(cur)
                    touched = False
                dt = mw.DTYPES[op.dtype]
                try:
                    if k == "send":
                        h = mw.mw_send(op.world, op.a, op.b, t.data_ptr(), op.count, dt, s.cuda_stream)
                    elif k == "recv":
                        h = mw.mw_recv(op.world, op.a, op.b, t.data_ptr(), op.count, dt, s.cuda_stream)
                    elif k == "bcast":
                        h = mw.mw_broadcast(op.world, op.a, op.b, t.data_ptr(), op.count, dt, s.cuda_stream)
                    elif k == "allreduce":
                        h = mw.mw_allreduce_sum(op.world, op.a, t.data_ptr(), op.count, dt, s.cuda_stream)
                    elif k == "reduce":
                        h = mw.mw_reduce_sum(op.world, op.a, op.b, p1, op.count, dt, s.cuda_stream)
                    elif k == "allgather":
                        h = mw.mw_all_gather(op.world, op.a, p1, p2, op.count, dt, s.cuda_stream)
                    elif k == "gather":
                        h = mw.mw_gather(op.world, op.a, op.b, p1, p2, op.count, dt, s.cuda_stream)
                    else:
                        h = mw.mw_scatter(op.world, op.a, op.b, p1, p2, op.count, dt, s.cuda_stream)
                    outstanding.append((idx, h))
                except mw.MwError as e:
                    if e.code != mw.MW_EBROKEN:
                        raise
                    out.status[idx] = "broken"  # the post itself was refused
            elif k == "create":
                mw.mw_world_create(op.world, list(op.members))
            elif k == "abort_world":
                mw.mw_world_abort(op.world)
            elif k == "abort_worker":
                mw.mw_worker_abort(op.a)
            elif k == "wait":
                wait_all(outstanding, out.status)
            elif k == "flush":
                mw.mw_flush()
            elif k == "check":
                wait_all(outstanding, out.status)
                if snapshots:
                    out.snapshots[idx] = get(op.buf).cpu().numpy().copy()
                if check_fn is not None:
                    get(op.buf)
                    check_fn(idx, op, bufs)
            elif k == "restore":
                wait_all(outstanding, out.status)
                if op.buf in bufs:
                    _fill(trace.bufs[op.buf], bufs[op.buf], pools, materialize)
                    touched = True
            elif k == "free":
                wait_all(outstanding, out.status)
                bufs.pop(op.buf, None)
            else:
                raise ValueError(f"unknown trace op {k}")
        wait_all(outstanding, out.status)
        torch.cuda.synchronize(dev)
        out.seconds = time.time() - t_start
        # whatever is still pending waits for a peer that never posted
        ps = mw.mw_poll_many([h for _, h in outstanding]) if outstanding else []
        for (idx, h), st in zip(outstanding, ps):
            out.status[idx] = STATE_NAME.get(st, f"error{st}")
        for op in trace.ops:
            if op.kind == "create":
                out.world_state[op.world] = "alive" if mw.mw_world_state(op.world) == mw.MW_ALIVE else "broken"
        for idx, st in out.status.items():
            o = trace.ops[idx]
            if st == "done" and (o.kind == "recv" or (o.kind not in ("send", "recv") and o.a == 0)):
                out.payload_bytes_done += o.count * ITEMSIZE[o.dtype]
    finally:
        try:
            if on_exit is not None:
                on_exit()
        finally:
            mw.mw_shutdown()
    return out
