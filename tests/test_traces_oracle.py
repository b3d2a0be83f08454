"""The five workload traces through the CPU oracle, at sizes that take seconds.

What is checked is fixed by the workload definitions, not by the oracle:
received == sent for every completed message, the count of completed / broken
operations around the abort, and the closed-form fault set.
"""

import numpy as np

import workloads
from oracle import BROKEN, DONE
from oracle.run_trace import run_trace
from workloads import materialize


def _mat(pools):
    return lambda spec: materialize(spec, pools)


def test_config1_all_messages_arrive_in_both_worlds(host_pools):
    t = workloads.config1()
    r = run_trace(t, _mat(host_pools))
    assert all(s == DONE for s in r.status.values())
    assert len(r.status) == 2 * 200 + 2 * 2 + 2 * 2
    # the k-th destination holds the k-th source: buffers were created src, dst, src, dst, ...
    checks = [i for i, op in enumerate(t.ops) if op.kind == "check"]
    for i in checks[:200]:
        dst = t.ops[i].buf
        assert np.array_equal(r.snapshots[i], materialize(t.bufs[dst - 1]))
    assert r.payload_bytes_done == 200 * 32768 + 4 * 32768


def test_config2_small_every_step_delivers(host_pools):
    t = workloads.config2(shape=(2, 33, 65), steps=6)
    r = run_trace(t, _mat(host_pools))
    assert all(s == DONE for s in r.status.values()) and len(r.status) == 6 * 8 * 2
    assert len(r.snapshots) == 6 * 8
    assert all(not np.all(s == 0xA5) for s in r.snapshots.values())


def test_config3_small_sums_on_all_ranks(host_pools):
    t = workloads.config3(shapes=((3, 17), (5, 11)), iters=6)
    r = run_trace(t, _mat(host_pools))
    assert all(s == DONE for s in r.status.values()) and len(r.status) == 6 * 4 * 4 * 2
    assert len(r.reduce_ref) == len(r.snapshots) == 6 * 4 * 4 * 2
    # restored inputs: iteration 4 reuses set 0, so its sums equal iteration 0's
    snaps = [r.snapshots[i] for i in sorted(r.snapshots)]
    per_iter = len(snaps) // 6
    for a, b in zip(snaps[:per_iter], snaps[4 * per_iter : 5 * per_iter]):
        assert np.array_equal(a, b)


def test_config4_small_only_the_victims_world_breaks(host_pools):
    t = workloads.config4(shape=(2, 8, 20), steps=30, abort_step=10)
    r = run_trace(t, _mat(host_pools))
    by_world = {}
    for i, s in r.status.items():
        by_world.setdefault(t.ops[i].world, []).append(s)
    for w, sts in by_world.items():
        if w == 7:
            assert sts.count(DONE) == 2 * 10 and sts.count(BROKEN) == 2 * 20
            assert sts[: 2 * 10] == [DONE] * 20  # steps 0..9 complete, 10.. are refused
        else:
            assert sts == [DONE] * 60
    assert [w for w, s in r.world_state.items() if s == BROKEN] == [7]


def test_config5_small_statuses_follow_the_fault_closed_form(host_pools):
    t = workloads.config5(n_ops=600, max_bytes=1 << 16, check_all=True)
    r = run_trace(t, _mat(host_pools))
    members = t.meta["members"]
    broken_at = {}  # world -> op index from which it is broken
    for at, victims in t.meta["abort_at"].items():
        for v in victims:
            for w, m in enumerate(members):
                if v in m:
                    broken_at[w] = min(broken_at.get(w, 10 ** 9), at)
    assert broken_at, "seed should abort at least one populated worker"
    # a post is refused iff a worker of its world was aborted earlier in the trace
    dead = set()
    aborts_seen = 0
    for i, op in enumerate(t.ops):
        if op.kind == "abort_worker":
            aborts_seen += 1
            dead.add(op.a)
        if i in r.status:
            want = BROKEN if dead & set(members[op.world]) else DONE
            assert r.status[i] == want, (i, op)
    assert aborts_seen == 3
    assert set(r.status.values()) == {DONE, BROKEN}
    assert len(r.snapshots) > 600


def test_online_recovery_trace_breaks_exactly_the_failed_workers_worlds(host_pools):
    """Fig. 2 in small: the statuses follow from the scenario alone (P3 = worker 2 fails; worlds 2 and 4 contain
    it), and every delivered tensor is its source (buffers are created src, dst per message; orphan receives
    have a destination only)."""
    t = workloads.online_recovery(count=257, window=4, rounds=2)
    r = run_trace(t, _mat(host_pools))
    assert r.world_state == {1: "alive", 3: "alive", 2: BROKEN, 4: BROKEN, 6: "alive", 7: "alive"}
    failed_at = next(i for i, op in enumerate(t.ops) if op.kind == "abort_worker")
    assert t.ops[failed_at].a == 2
    sends = {}  # destination buffer -> source buffer, from the way the generator pairs them
    for i, op in enumerate(t.ops):
        if i not in r.status:
            continue
        in_p3_world = op.world in (2, 4)
        if in_p3_world and i > failed_at:
            assert r.status[i] == BROKEN  # refused
        elif op.kind == "recv" and t.bufs[op.buf - 1].init[0] == "fill":
            assert in_p3_world and r.status[i] == BROKEN  # the orphan receive: its tensor never came
        else:
            assert r.status[i] == DONE, (i, op)
            if op.kind == "recv":
                sends[op.buf] = op.buf - 1
    assert sum(1 for s in r.status.values() if s == BROKEN) == 2 + 2 * 2 * 4
    delivered = 0
    for i, op in enumerate(t.ops):
        if op.kind != "check":
            continue
        if op.buf in sends:
            assert np.array_equal(r.snapshots[i], materialize(t.bufs[sends[op.buf]]))
            delivered += 1
        else:
            assert np.all(r.snapshots[i] == 0xA5)  # nothing was written where nothing was delivered
    assert delivered == len(sends) == (3 * 2 + 2 * 4 + 4 + 2 + 2 + 2 * 4) * 4


def test_multi_sender_traces_deliver_every_tensor_in_both_setups(host_pools):
    for senders in (1, 2, 3):
        for multi in (True, False):
            t = workloads.multi_sender(senders, 1000, multi, window=4, n_windows=2)
            r = run_trace(t, _mat(host_pools))
            assert all(s == DONE for s in r.status.values()) and len(r.status) == 2 * senders * 8
            for i, op in enumerate(t.ops):
                if op.kind == "check":
                    assert np.array_equal(r.snapshots[i], materialize(t.bufs[op.buf - 1]))
