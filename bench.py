"""Benchmark of the multi-world data plane on one MI355X.

Workload: the pipeline-stage activation hand-off -- 8 worlds, each a 2-rank
producer -> consumer pair, bf16 [32, 2048, 4096] payloads (512 MiB), every
world's transfer of a step outstanding together, each world posting on its own
stream.  One step = one pass of the whole path over that batch: 16 posts,
matching, one batched copy launch covering all 8 worlds, device-written
completion flags, host polling.  Payloads are resident in HBM before timing.

Prints ONE JSON line (see README / DESIGN for the fields).
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "multi-world transfer GB/s on 1 MI355X (% of HBM peak); % loss vs single world"
HBM_PEAK_GBPS = 8000.0
SHAPE = (32, 2048, 4096)
N_WORLDS = 8
POOL_K = 4


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--reps", type=int, default=5, help="repetitions of the multi-/single-world comparison")
    ap.add_argument("--cpu-steps", type=int, default=6, help="steps of the workload the CPU oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--shape", type=int, nargs=3, default=list(SHAPE), help=argparse.SUPPRESS)
    return ap.parse_args()


class Workload:
    """Device buffers of the hand-off workload and the loop that drives one run."""

    def __init__(self, torch, mw, shape, device):
        from paper_2407_08980_amd.trace_runner import DevicePools
        from workloads import HostPools
        from workloads.data import POOL_ELEMS, rng_of

        self.torch, self.mw = torch, mw
        self.count = shape[0] * shape[1] * shape[2]
        self.nbytes = self.count * 2
        self.host_pools = HostPools()
        pools = DevicePools(self.host_pools, device)
        rng = rng_of(20240708 + 2)
        self.offsets = [[int(rng.integers(0, POOL_ELEMS)) for _ in range(POOL_K)] for _ in range(N_WORLDS)]
        self.src = []
        self.dst = []
        for w in range(N_WORLDS):
            row = []
            for k in range(POOL_K):
                t = torch.empty(self.nbytes, dtype=torch.uint8, device=device)
                pools.slice("bf16", self.offsets[w][k], self.nbytes, t)
                row.append(t)
            self.src.append(row)
            self.dst.append([torch.full((self.nbytes,), 0xA5, dtype=torch.uint8, device=device) for _ in range(2)])
        self.streams = [torch.cuda.Stream(device=device) for _ in range(N_WORLDS)]
        torch.cuda.synchronize(device)

    def post_step(self, s, world_of, ranks_of):
        """Post step s of every world: the producer's send and the consumer's recv."""
        mw = self.mw
        hs = []
        for w in range(N_WORLDS):
            st = self.streams[w].cuda_stream
            wid = world_of[w]
            a, b = ranks_of[w]
            hs.append(mw.mw_send(wid, a, b, self.src[w][s % POOL_K].data_ptr(), self.count, mw.MW_BF16, st))
            hs.append(mw.mw_recv(wid, a, b, self.dst[w][s % 2].data_ptr(), self.count, mw.MW_BF16, st))
        mw.mw_flush()
        return mw.PollSet(hs)

    @staticmethod
    def wait(ps):
        while ps.poll():  # busy-wait polling, as the paper's communicator does
            pass
        bad = [s for s in ps.states if s != 0]
        if bad:
            raise RuntimeError(f"operations ended in states {bad}")

    def run(self, steps, world_of, ranks_of, first_step=0):
        """Steps are double-buffered: step s+1 is posted while step s is in flight."""
        prev = None
        for s in range(first_step, first_step + steps):
            cur = self.post_step(s, world_of, ranks_of)
            if prev is not None:
                self.wait(prev)
            prev = cur
        if prev is not None:
            self.wait(prev)

    def timed(self, steps, world_of, ranks_of, first_step=0):
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.run(steps, world_of, ranks_of, first_step)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def verify_last(self, steps, first_step=0):
        """received == sent for the last two steps (both destination buffers), on the device."""
        torch = self.torch
        for s in range(max(first_step, first_step + steps - 2), first_step + steps):
            for w in range(N_WORLDS):
                if not torch.equal(self.dst[w][s % 2], self.src[w][s % POOL_K]):
                    raise RuntimeError(f"world {w} step {s}: destination differs from source")


def cpu_baseline(shape, steps):
    """The CPU oracle on the first `steps` steps of the same workload (all 8 worlds), one thread."""
    import numpy as np

    from oracle import BF16, WorldOracle
    from workloads import HostPools
    from workloads.data import POOL_ELEMS, pool_slice, rng_of

    count = shape[0] * shape[1] * shape[2]
    nbytes = count * 2
    pools = HostPools()
    rng = rng_of(20240708 + 2)
    src = [pool_slice(pools.get("bf16"), "bf16", int(rng.integers(0, POOL_ELEMS)), nbytes) for _ in range(N_WORLDS)]
    dst = [np.full(nbytes, 0xA5, dtype=np.uint8) for _ in range(N_WORLDS)]
    orc = WorldOracle(2 * N_WORLDS)
    for w in range(N_WORLDS):
        orc.create(w, (2 * w, 2 * w + 1))
    t0 = time.perf_counter()
    for s in range(steps):
        for w in range(N_WORLDS):
            orc.post_send(w, 0, 1, src[w], count, BF16)
            orc.post_recv(w, 0, 1, dst[w], count, BF16)
    dt = time.perf_counter() - t0
    assert all(st == "done" for st in orc.result)
    return steps * N_WORLDS * nbytes / dt / 1e9, dt


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py measures ONE GPU: logical workers share a single device and there is no inter-GPU path "
              f"(got --gpus {args.gpus})", file=sys.stderr)
        sys.exit(2)
    import torch

    if not torch.cuda.is_available():
        print("bench.py needs the MI355X (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)
    from paper_2407_08980_amd import binding as mw

    mw.lib()
    shape = tuple(args.shape)
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    mw.mw_init(0, 2 * N_WORLDS)
    wl = Workload(torch, mw, shape, dev)
    # multi-world: world w = (worker 2w -> worker 2w+1); single world: one world of all 16 workers
    for w in range(N_WORLDS):
        mw.mw_world_create(w, [2 * w, 2 * w + 1])
    SINGLE = 1000
    mw.mw_world_create(SINGLE, list(range(2 * N_WORLDS)))
    multi = (list(range(N_WORLDS)), [(0, 1)] * N_WORLDS)
    single = ([SINGLE] * N_WORLDS, [(2 * w, 2 * w + 1) for w in range(N_WORLDS)])

    K, W = args.steps, args.warmup
    wl.run(W, *multi)
    mw.mw_profile_enable(True)
    mw.mw_profile_read(mw.KIND_COPY)
    elapsed = wl.timed(K, *multi, first_step=W)
    launches, kernel_ms, op_bytes = mw.mw_profile_read(mw.KIND_COPY)
    mw.mw_profile_enable(False)
    wl.verify_last(K, first_step=W)
    step_payload = N_WORLDS * wl.nbytes
    value = K * step_payload / elapsed / 1e9

    # multi-world overhead against the single-world baseline: same messages, same order, same kernels
    mw_rates, sw_rates = [], []
    for r in range(args.reps):
        sw_rates.append(K * step_payload / wl.timed(K, *single) / 1e9)
        mw_rates.append(K * step_payload / wl.timed(K, *multi) / 1e9)
    wl.verify_last(K)
    mean = lambda v: sum(v) / len(v) if v else float("nan")
    loss_pct = (1.0 - mean(mw_rates) / mean(sw_rates)) * 100.0 if args.reps else None

    alg_bytes_per_launch = 2.0 * op_bytes / max(launches, 1)  # send/recv: one read + one write of the payload
    avg_ms = kernel_ms / max(launches, 1)
    achieved = alg_bytes_per_launch / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
    out = {
        "metric": METRIC,
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(elapsed / K * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {
            "workload": "config 2: pipeline-stage activation hand-off, 8 worlds x (producer -> consumer), "
                        f"bf16 {list(shape)} = {wl.nbytes >> 20} MiB per message, all worlds concurrent on separate "
                        "streams",
            "worlds": N_WORLDS,
            "payload_dtype": "bf16",
            "payload_bytes_per_step": step_payload,
            "steps_in_flight": 2,
        },
        "hbm_traffic_GBps": round(2 * value, 1),
        "pct_of_hbm_peak": round(2 * value / HBM_PEAK_GBPS * 100.0, 2),
        "single_world_GBps": round(mean(sw_rates), 1) if args.reps else None,
        "multi_world_GBps_mean": round(mean(mw_rates), 1) if args.reps else None,
        "loss_vs_single_world_pct": round(loss_pct, 3) if args.reps else None,
        "overhead_reps": args.reps,
        "roofline": {
            "bound": "hbm",
            "kernel": "mw_k_copy",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": None,
            "launches": launches,
            "avg_launch_ms": round(avg_ms, 4),
            "alg_bytes_per_launch": alg_bytes_per_launch,
        },
    }
    mw.mw_shutdown()
    del wl
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        gbps, secs = cpu_baseline(shape, args.cpu_steps)
        out["cpu_baseline"] = {
            "value": round(gbps, 2),
            "unit": "GB/s",
            "cores": 1,
            "kind": "oracle",
            "sample": f"first {args.cpu_steps} steps of the same workload, all {N_WORLDS} worlds "
                      f"({args.cpu_steps * N_WORLDS} messages of {shape[0] * shape[1] * shape[2] * 2 >> 20} MiB), "
                      f"{secs:.1f} s of oracle time; host has {os.cpu_count()} logical CPUs",
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
