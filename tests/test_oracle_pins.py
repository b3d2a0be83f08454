"""Pins for the CPU oracle: everything here is fixed by the paper or by
mathematics, none of it by the oracle's own formulas.

  send/recv  -- received bytes == sent bytes, FIFO per (world, src, dst)
  broadcast  -- brute force on tiny inputs, root untouched
  all-reduce -- exact rational arithmetic on tiny inputs; integer-valued inputs
                (sum exact in every precision); x and -x cancel to +0; two fp32
                ranks give the correctly rounded sum; all ranks agree
  bf16       -- the format's definition evaluated with integers (golden values)
  faults     -- the worked examples of Fig. 2 and Fig. 4 and the closed form
                broken(k) = {w : k in members(w)}
  polling    -- a recv with no sender stays pending while another world moves
                a thousand tensors (the deadlock scenario of Sec. 3.2)
"""

from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import BF16, BROKEN, DONE, F32, MISMATCH, PENDING, WorldOracle
from oracle.mw_oracle import OracleError

from helpers import golden, read_kv


def u8(a):
    return np.ascontiguousarray(a).view(np.uint8).reshape(-1)


def rand_bytes(n, seed):
    return np.random.default_rng(seed).integers(0, 256, size=n, dtype=np.uint8)


# ---------------------------------------------------------------------------
# bf16 format
# ---------------------------------------------------------------------------
def _bf16_exact(bits):
    """Value of a bf16 pattern from the format's definition, in exact rationals."""
    sign = -1 if bits >> 15 else 1
    e = (bits >> 7) & 0xFF
    m = bits & 0x7F
    assert e != 0xFF
    if e == 0:
        return sign * Fraction(m, 128) * Fraction(2) ** (-126)
    return sign * (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)


def test_bf16_widening_matches_golden_values():
    rows = []
    with open(golden("bf16_values.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                b, v = line.split()
                rows.append((int(b, 16), float(v)))
    assert len(rows) >= 10
    bits = np.array([b for b, _ in rows], dtype=np.uint16)
    got = oracle.bf16_bits_to_f32(bits)
    for (b, v), g in zip(rows, got):
        assert Fraction(float(g)) == _bf16_exact(b), hex(b)
        assert float(g) == v and np.signbit(g) == (b >> 15 == 1), hex(b)


def test_bf16_widening_all_finite_patterns_against_definition():
    bits = np.arange(0, 1 << 16, dtype=np.uint32)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF].astype(np.uint16)
    got = oracle.bf16_bits_to_f32(bits)
    for b, g in zip(bits[::37], got[::37]):
        assert Fraction(float(g)) == _bf16_exact(int(b))


def test_bf16_rounding_is_nearest_even():
    # every bf16 value survives a round trip
    bits = np.arange(0, 1 << 16, dtype=np.uint32)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF].astype(np.uint16)
    assert np.array_equal(oracle.f32_to_bf16_bits(oracle.bf16_bits_to_f32(bits)), bits)
    # ties: 1 + 2^-8 lies halfway between 1 (even) and 1 + 2^-7 -> 1;
    # 1 + 3*2^-8 lies halfway between 1 + 2^-7 (odd) and 1 + 2^-6 -> 1 + 2^-6
    x = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, -(1 + 2.0 ** -8)], dtype=np.float32)
    got = oracle.f32_to_bf16_bits(x)
    assert [hex(v) for v in got] == ["0x3f80", "0x3f82", "0x3f81", "0xbf80"]
    # brute force nearest-even against exact rationals on random draws
    rng = np.random.default_rng(5)
    xs = rng.standard_normal(300).astype(np.float32)
    for xv, b in zip(xs, oracle.f32_to_bf16_bits(xs)):
        fx = Fraction(float(xv))
        cands = [int(b) + d for d in (-1, 0, 1)]
        errs = [abs(_bf16_exact(c) - fx) for c in cands]
        assert errs[1] == min(errs)
        for c, e in zip(cands, errs):
            if c != int(b) and e == errs[1]:
                assert int(b) % 2 == 0  # a tie goes to the even pattern
    assert np.isnan(oracle.bf16_bits_to_f32(oracle.f32_to_bf16_bits(np.array([np.nan], dtype=np.float32))))[0]


# ---------------------------------------------------------------------------
# send / recv
# ---------------------------------------------------------------------------
def test_sendrecv_identity_arbitrary_bit_patterns():
    o = WorldOracle(2)
    o.create(0, (0, 1))
    # NaN payloads, -0, denormals: any byte pattern must survive
    special = np.array([0x7FC00001, 0xFFC12345, 0x80000000, 0x00000001, 0x7F800000, 0x007FFFFF], dtype=np.uint32)
    src = np.concatenate([u8(special), rand_bytes(4 * 1000, 1)])
    keep = src.copy()
    dst = np.full(src.size, 0xA5, dtype=np.uint8)
    hs = o.post_send(0, 0, 1, src, src.size // 4, F32)
    assert o.status(hs) == PENDING  # rendezvous: no receiver yet
    hr = o.post_recv(0, 0, 1, dst, src.size // 4, F32)
    assert o.status(hs) == DONE and o.status(hr) == DONE
    assert np.array_equal(dst, keep) and np.array_equal(src, keep)


def test_sendrecv_partial_buffer_and_bf16_count():
    o = WorldOracle(2)
    o.create(3, (1, 0))
    src = rand_bytes(64, 2)
    dst = np.full(64, 0xA5, dtype=np.uint8)
    o.post_recv(3, 1, 0, dst, 7, BF16)
    o.post_send(3, 1, 0, src, 7, BF16)
    assert np.array_equal(dst[:14], src[:14]) and np.all(dst[14:] == 0xA5)


def test_sendrecv_fifo_order_per_pair_and_independence_across_pairs():
    o = WorldOracle(3)
    o.create(0, (0, 1, 2))
    n = 12
    srcs = [u8(np.array([k, 100 + k], dtype=np.float32)) for k in range(n)]
    dsts = [np.zeros(8, dtype=np.uint8) for _ in range(n)]
    # all sends first (1 -> 0), an unrelated pair in between, then the recvs
    for k in range(n):
        o.post_send(0, 1, 0, srcs[k], 2, F32)
    other_src, other_dst = rand_bytes(8, 3), np.zeros(8, dtype=np.uint8)
    o.post_send(0, 2, 0, other_src, 2, F32)
    for k in range(n):
        o.post_recv(0, 1, 0, dsts[k], 2, F32)
    for k in range(n):
        assert dsts[k].view(np.float32)[0] == k  # k-th recv holds the k-th send
    assert not other_dst.any()
    h = o.post_recv(0, 2, 0, other_dst, 2, F32)
    assert o.status(h) == DONE and np.array_equal(other_dst, other_src)
    # sends of another pair and of the opposite direction, posted EARLIER, are not what a recv of (1 -> 0) gets
    o = WorldOracle(3)
    o.create(0, (0, 1, 2))
    x, y, a = rand_bytes(8, 11), rand_bytes(8, 12), rand_bytes(8, 13)
    hx = o.post_send(0, 2, 0, x, 2, F32)
    hy = o.post_send(0, 0, 1, y, 2, F32)
    da = np.zeros(8, dtype=np.uint8)
    hr = o.post_recv(0, 1, 0, da, 2, F32)
    assert [o.status(h) for h in (hx, hy, hr)] == [PENDING] * 3 and not da.any()
    ha = o.post_send(0, 1, 0, a, 2, F32)
    assert [o.status(h) for h in (hx, hy, hr, ha)] == [PENDING, PENDING, DONE, DONE] and np.array_equal(da, a)


def test_sendrecv_same_pair_in_two_worlds_does_not_cross():
    o = WorldOracle(2)
    o.create(0, (0, 1))
    o.create(1, (0, 1))
    a, b = rand_bytes(16, 4), rand_bytes(16, 5)
    da, db = np.zeros(16, np.uint8), np.zeros(16, np.uint8)
    o.post_send(0, 0, 1, a, 4, F32)
    o.post_send(1, 0, 1, b, 4, F32)
    o.post_recv(1, 0, 1, db, 4, F32)
    o.post_recv(0, 0, 1, da, 4, F32)
    assert np.array_equal(da, a) and np.array_equal(db, b)


def test_mismatched_sides_move_nothing():
    o = WorldOracle(2)
    o.create(0, (0, 1))
    src, dst = rand_bytes(32, 6), np.full(32, 0xA5, np.uint8)
    hs = o.post_send(0, 0, 1, src, 8, F32)
    hr = o.post_recv(0, 0, 1, dst, 4, F32)
    assert o.status(hs) == MISMATCH and o.status(hr) == MISMATCH and np.all(dst == 0xA5)
    hs = o.post_send(0, 0, 1, src, 8, BF16)
    hr = o.post_recv(0, 0, 1, dst, 8, F32)
    assert o.status(hs) == MISMATCH and o.status(hr) == MISMATCH


def test_argument_errors():
    o = WorldOracle(3)
    o.create(0, (0, 1))
    b = np.zeros(16, np.uint8)
    with pytest.raises(OracleError) as e:
        o.create(0, (1, 2))
    assert e.value.code == "EEXIST"
    for bad in [(0, 0, 0), (0, 0, 2), (0, -1, 1)]:
        with pytest.raises(OracleError) as e:
            o.post_send(bad[0], bad[1], bad[2], b, 1, F32)
        assert e.value.code == "EINVAL"
    with pytest.raises(OracleError) as e:
        o.post_send(9, 0, 1, b, 1, F32)
    assert e.value.code == "ENOWORLD"
    with pytest.raises(OracleError):
        o.post_send(0, 0, 1, b, 5, F32)  # buffer too short
    with pytest.raises(OracleError):
        o.create(1, (0, 0))
    with pytest.raises(OracleError):
        o.create(1, (0, 3))


# ---------------------------------------------------------------------------
# broadcast
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n", [2, 3, 4])
def test_broadcast_brute_force(n):
    for root in range(n):
        o = WorldOracle(n)
        o.create(0, tuple(range(n)))
        bufs = [rand_bytes(16 * 4, 10 * n + r) for r in range(n)]
        root_before = bufs[root].copy()
        hs = []
        order = list(range(n))[::-1]
        for r in order:
            if hs:
                assert all(o.status(h) == PENDING for h in hs)
            hs.append(o.post_broadcast(0, r, root, bufs[r], 16, F32))
        assert all(o.status(h) == DONE for h in hs)
        for r in range(n):
            for i in range(64):
                assert bufs[r][i] == root_before[i]


def test_broadcast_root_disagreement_is_mismatch():
    o = WorldOracle(2)
    o.create(0, (0, 1))
    a, b = rand_bytes(8, 1), rand_bytes(8, 2)
    b0 = b.copy()
    h0 = o.post_broadcast(0, 0, 0, a, 2, F32)
    h1 = o.post_broadcast(0, 1, 1, b, 2, F32)
    assert o.status(h0) == MISMATCH and o.status(h1) == MISMATCH and np.array_equal(b, b0)


# ---------------------------------------------------------------------------
# all-reduce
# ---------------------------------------------------------------------------
def _run_allreduce(arrays, dtype):
    n = len(arrays)
    o = WorldOracle(n)
    o.create(0, tuple(range(n)))
    bufs = [u8(a).copy() for a in arrays]
    isz = 4 if dtype == F32 else 2
    count = bufs[0].size // isz
    hs = [o.post_allreduce(0, r, bufs[r], count, dtype) for r in range(n)]
    assert all(o.status(h) == DONE for h in hs)
    return o, hs, bufs


@pytest.mark.parametrize("n", [2, 3, 4])
def test_allreduce_against_exact_rational_sum(n):
    rng = np.random.default_rng(n)
    xs = [rng.standard_normal(16).astype(np.float32) for _ in range(n)]
    o, hs, bufs = _run_allreduce(xs, F32)
    s, sabs = o.reduce_ref[hs[0]]
    for i in range(16):
        exact = sum(Fraction(float(x[i])) for x in xs)
        exact_abs = sum(abs(Fraction(float(x[i]))) for x in xs)
        assert abs(Fraction(float(s[i])) - exact) <= exact_abs * Fraction(n, 2 ** 52)
        assert abs(Fraction(float(sabs[i])) - exact_abs) <= exact_abs * Fraction(n, 2 ** 52)
        # python's own float sum as the brute force
        assert abs(float(s[i]) - sum(float(x[i]) for x in xs)) <= 1e-15 * float(exact_abs)
    # in place, identical on every rank, and the stored tensor is the sum rounded to fp32
    for b in bufs:
        assert np.array_equal(b, bufs[0])
    assert np.array_equal(bufs[0].view(np.float32), s.astype(np.float32))


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("n", [2, 3, 4])
def test_allreduce_integer_inputs_are_exact_in_every_precision(n, dtype):
    rng = np.random.default_rng(100 + n)
    ints = [rng.integers(-16, 17, size=64) for _ in range(n)]  # |sum| <= 64: exact even in bf16
    if dtype == F32:
        arrays = [v.astype(np.float32) for v in ints]
    else:
        arrays = [oracle.f32_to_bf16_bits(v.astype(np.float32)) for v in ints]
    o, hs, bufs = _run_allreduce(arrays, dtype)
    want = sum(ints)
    s, _ = o.reduce_ref[hs[0]]
    assert np.array_equal(s, want.astype(np.float64))
    got = bufs[0].view(np.float32) if dtype == F32 else oracle.bf16_bits_to_f32(bufs[0].view(np.uint16))
    assert np.array_equal(got.astype(np.int64), want)
    ordered = oracle.allreduce_sum_ordered([u8(a) for a in arrays], 64, dtype)
    assert np.array_equal(ordered, bufs[0])  # both summation definitions agree when sums are exact


def test_allreduce_cancellation_gives_plus_zero():
    x = np.random.default_rng(7).standard_normal(32).astype(np.float32)
    o, hs, bufs = _run_allreduce([x, -x], F32)
    assert not bufs[0].any()  # +0.0 is the all-zero pattern
    xb = oracle.f32_to_bf16_bits(x)
    o, hs, bufs = _run_allreduce([xb, xb ^ np.uint16(0x8000)], BF16)
    assert not bufs[0].any()
    assert not oracle.allreduce_sum_ordered([u8(x), u8(-x)], 32, F32).any()


def test_allreduce_two_fp32_ranks_is_the_correctly_rounded_sum():
    rng = np.random.default_rng(8)
    a = (rng.standard_normal(4096) * 10.0 ** rng.integers(-3, 4, 4096)).astype(np.float32)
    b = (rng.standard_normal(4096) * 10.0 ** rng.integers(-3, 4, 4096)).astype(np.float32)
    o, hs, bufs = _run_allreduce([a, b], F32)
    want = a + b  # IEEE float32 addition is correctly rounded; fp64 holds a+b exactly here
    assert np.array_equal(bufs[0].view(np.float32), want)
    assert np.array_equal(oracle.allreduce_sum_ordered([u8(a), u8(b)], 4096, F32).view(np.float32), want)


def test_allreduce_ordered_sum_follows_ascending_rank_order():
    # (1 + 2^-24) + 2^-24 in fp32: ascending order loses both small terms, the
    # reverse order keeps them -- so the order is observable.
    big, tiny = np.float32(1.0), np.float32(2.0 ** -24)
    asc = oracle.allreduce_sum_ordered([u8(np.array([big])), u8(np.array([tiny])), u8(np.array([tiny]))], 1, F32)
    desc = oracle.allreduce_sum_ordered([u8(np.array([tiny])), u8(np.array([tiny])), u8(np.array([big]))], 1, F32)
    assert asc.view(np.float32)[0] == np.float32(1.0)
    assert desc.view(np.float32)[0] == np.float32(1.0 + 2.0 ** -23)
    # python-loop brute force of the same order on random data, bf16 output rounded once
    rng = np.random.default_rng(9)
    xs = [oracle.f32_to_bf16_bits(rng.uniform(-1, 1, 50).astype(np.float32)) for _ in range(4)]
    got = oracle.allreduce_sum_ordered([u8(x) for x in xs], 50, BF16).view(np.uint16)
    for i in range(50):
        acc = np.float32(0)
        vals = [oracle.bf16_bits_to_f32(x[i : i + 1])[0] for x in xs]
        acc = vals[0]
        for v in vals[1:]:
            acc = np.float32(acc + v)
        assert got[i] == oracle.f32_to_bf16_bits(np.array([acc]))[0]


def test_allreduce_tolerance_accepts_any_order_and_rejects_a_dropped_rank():
    rng = np.random.default_rng(10)
    xs = [rng.uniform(-1, 1, 2048).astype(np.float32) for _ in range(4)]
    s, sabs = oracle.allreduce_sum_f64([u8(x) for x in xs], 2048, F32)
    for order in ([0, 1, 2, 3], [3, 2, 1, 0], [2, 0, 3, 1]):
        y = oracle.allreduce_sum_ordered([u8(xs[i]) for i in order], 2048, F32)
        ok, worst = oracle.allreduce_within_tolerance(y, s, sabs, 2048, F32)
        assert ok and worst < 3 * 2.0 ** -24
    dropped = oracle.allreduce_sum_ordered([u8(x) for x in xs[:3]], 2048, F32)
    assert not oracle.allreduce_within_tolerance(dropped, s, sabs, 2048, F32)[0]
    xb = [oracle.f32_to_bf16_bits(x) for x in xs]
    s, sabs = oracle.allreduce_sum_f64([u8(x) for x in xb], 2048, BF16)
    y = oracle.allreduce_sum_ordered([u8(x) for x in xb], 2048, BF16)
    ok, worst = oracle.allreduce_within_tolerance(y, s, sabs, 2048, BF16)
    assert ok and worst <= 2.0 ** -8
    wrong_dtype = oracle.allreduce_sum_ordered([u8(x) for x in xb], 1024, F32)  # bf16 pairs read as fp32
    assert not oracle.allreduce_within_tolerance(wrong_dtype[: 2048 * 2], s, sabs, 2048, BF16)[0]


def test_collectives_run_in_per_world_sequence_order():
    o = WorldOracle(2)
    o.create(0, (0, 1))
    a0, a1 = u8(np.array([1.0], np.float32)).copy(), u8(np.array([2.0], np.float32)).copy()
    b0, b1 = u8(np.array([10.0], np.float32)).copy(), u8(np.array([20.0], np.float32)).copy()
    # rank 0 posts two collectives before rank 1 posts any
    h = [o.post_allreduce(0, 0, a0, 1, F32), o.post_broadcast(0, 0, 1, b0, 1, F32)]
    assert all(o.status(x) == PENDING for x in h)
    h.append(o.post_allreduce(0, 1, a1, 1, F32))
    assert o.status(h[0]) == DONE and o.status(h[1]) == PENDING
    h.append(o.post_broadcast(0, 1, 1, b1, 1, F32))
    assert all(o.status(x) == DONE for x in h)
    assert a0.view(np.float32)[0] == 3.0 and a1.view(np.float32)[0] == 3.0
    assert b0.view(np.float32)[0] == 20.0
    # kind disagreement at the same sequence number
    h0 = o.post_allreduce(0, 0, a0, 1, F32)
    h1 = o.post_broadcast(0, 1, 0, b1, 1, F32)
    assert o.status(h0) == MISMATCH and o.status(h1) == MISMATCH


# ---------------------------------------------------------------------------
# fault domains: the paper's worked examples
# ---------------------------------------------------------------------------
def test_fig2_rhombus_fault_set_and_recovery():
    kv = read_kv(golden("fig2_rhombus.txt"))
    workers = kv["workers"][0].split()
    wid = {name: i for i, name in enumerate(workers)}
    o = WorldOracle(len(workers))
    worlds = {}
    for key, vals in kv.items():
        if key.startswith("world "):
            worlds[key.split()[1]] = [wid[x] for x in vals[0].split()]
    names = sorted(worlds)
    for i, nm in enumerate(names):
        o.create(i, worlds[nm])
    idx = {nm: i for i, nm in enumerate(names)}
    # traffic pending everywhere: the downstream side of every edge waits for a tensor
    bufs = {nm: np.zeros(8, np.uint8) for nm in names}
    pend = {nm: o.post_recv(idx[nm], 0, 1, bufs[nm], 2, F32) for nm in names}
    failed = wid[kv["fail"][0]]
    assert oracle.broken_worlds_of_worker({idx[n]: worlds[n] for n in names}, failed) == {
        idx[n] for n in kv["broken"][0].split()}
    o.abort_worker(failed)
    for nm in kv["broken"][0].split():
        assert o.world_state(idx[nm]) == BROKEN and o.status(pend[nm]) == BROKEN
        assert o.status(o.post_send(idx[nm], 0, 1, np.zeros(8, np.uint8), 2, F32)) == BROKEN  # access refused
    for nm in kv["healthy"][0].split():
        assert o.world_state(idx[nm]) == oracle.ALIVE and o.status(pend[nm]) == PENDING
        src = rand_bytes(8, 11)
        assert o.status(o.post_send(idx[nm], 0, 1, src, 2, F32)) == DONE
        assert o.status(pend[nm]) == DONE and np.array_equal(bufs[nm], src)
    # recovery: NEW worlds with the new worker, the broken ones are not reused
    base = len(names)
    for j, (key, vals) in enumerate((k, v) for k, v in kv.items() if k.startswith("recover world")):
        o.create(base + j, [wid[x] for x in vals[0].split()])
        src, dst = rand_bytes(8, 12 + j), np.zeros(8, np.uint8)
        o.post_send(base + j, 0, 1, src, 2, F32)
        assert o.status(o.post_recv(base + j, 0, 1, dst, 2, F32)) == DONE and np.array_equal(dst, src)


def test_fig4_leader_keeps_receiving_after_peer_dies():
    kv = read_kv(golden("fig4_leader.txt"))
    n_before = int(kv["tensors_sent_by_victim_before_termination"][0])
    o = WorldOracle(3)  # worker 0 = leader, 1 = W1-R1, 2 = W2-R1
    o.create(1, (0, 1))
    o.create(2, (0, 2))
    got = {1: 0, 2: 0}
    recv_handles = {1: [], 2: []}

    def leader_posts_recv(w):
        b = np.zeros(4, np.uint8)
        recv_handles[w].append((o.post_recv(w, 1, 0, b, 1, F32), b))

    def peer_sends(w, k):
        return o.post_send(w, 1, 0, u8(np.array([k], np.float32)), 1, F32)

    # W1's peer sends twice as often as W2's, as in the experiment
    for tick in range(2 * n_before):
        leader_posts_recv(1)
        peer_sends(1, tick)
        if tick % 2 == 1:
            leader_posts_recv(2)
            peer_sends(2, tick // 2)
    leader_posts_recv(2)  # the leader is already waiting for the 11th tensor
    o.abort_worker(2)  # W2-R1 terminated after its 10th tensor
    for tick in range(50):  # the leader goes on with W1
        leader_posts_recv(1)
        assert o.status(peer_sends(1, 1000 + tick)) == DONE
    for w in (1, 2):
        got[w] = sum(o.status(h) == DONE for h, _ in recv_handles[w])
    assert got[2] == int(kv["tensors_received_from_victim"][0]) == n_before
    assert [int(b.view(np.float32)[0]) for h, b in recv_handles[2][:n_before]] == list(range(n_before))
    assert o.status(recv_handles[2][-1][0]) == BROKEN
    assert got[1] == 2 * n_before + 50
    assert o.world_state(1) == kv["world_state_after W1"][0]
    assert o.world_state(2) == kv["world_state_after W2"][0]


def test_config1_topology_exhaustive_fault_sets():
    worlds = {0: (0, 1), 1: (0, 2)}
    expect = {0: {0, 1}, 1: {0}, 2: {1}}
    for victim, broken in expect.items():
        o = WorldOracle(3)
        for w, m in worlds.items():
            o.create(w, m)
        o.abort_worker(victim)
        assert {w for w in worlds if o.world_state(w) == BROKEN} == broken
        assert oracle.broken_worlds_of_worker(worlds, victim) == broken


def test_fault_set_closed_form_on_random_topologies():
    rng = np.random.default_rng(12)
    for trial in range(20):
        nw = int(rng.integers(3, 12))
        worlds = {w: tuple(int(x) for x in rng.choice(nw, size=int(rng.integers(2, min(5, nw + 1))), replace=False))
                  for w in range(int(rng.integers(2, 20)))}
        o = WorldOracle(nw)
        for w, m in worlds.items():
            o.create(w, m)
        victims = [int(x) for x in rng.choice(nw, size=2, replace=False)]
        for v in victims:
            o.abort_worker(v)
        want = {w for w, m in worlds.items() if any(v in m for v in victims)}
        assert {w for w in worlds if o.world_state(w) == BROKEN} == want


def test_completed_ops_stay_done_and_abort_is_idempotent():
    o = WorldOracle(2)
    o.create(0, (0, 1))
    src, dst = rand_bytes(8, 13), np.zeros(8, np.uint8)
    hs, hr = o.post_send(0, 0, 1, src, 2, F32), o.post_recv(0, 0, 1, dst, 2, F32)
    hp = o.post_send(0, 0, 1, src, 2, F32)
    hc = o.post_allreduce(0, 0, np.zeros(8, np.uint8), 2, F32)
    o.abort_world(0)
    o.abort_world(0)
    assert (o.status(hs), o.status(hr), o.status(hp), o.status(hc)) == (DONE, DONE, BROKEN, BROKEN)
    assert np.array_equal(dst, src)


def test_pending_recv_in_one_world_never_blocks_another():
    o = WorldOracle(3)
    o.create(0, (0, 1))
    o.create(1, (0, 2))
    stuck = o.post_recv(0, 1, 0, np.zeros(8, np.uint8), 2, F32)  # its sender never shows up
    for k in range(1000):
        src, dst = rand_bytes(8, 1000 + k), np.zeros(8, np.uint8)
        o.post_recv(1, 1, 0, dst, 2, F32)
        assert o.status(o.post_send(1, 1, 0, src, 2, F32)) == DONE and np.array_equal(dst, src)
        assert o.status(stuck) == PENDING


# ---------------------------------------------------------------------------
# reduce / all-gather / gather / scatter (the communicator's other four operations)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n", [2, 3, 4])
def test_reduce_leaves_the_exact_sum_on_the_root_only(n):
    rng = np.random.default_rng(40 + n)
    for root in range(n):
        xs = [rng.standard_normal(12).astype(np.float32) for _ in range(n)]
        o = WorldOracle(n)
        o.create(0, tuple(range(n)))
        bufs = [u8(x).copy() for x in xs]
        hs = [o.post_reduce(0, r, root, bufs[r], 12, F32) for r in range(n)]
        assert all(o.status(h) == DONE for h in hs)
        s, sabs = o.reduce_ref[hs[root]]
        for i in range(12):
            exact = sum(Fraction(float(x[i])) for x in xs)
            exact_abs = sum(abs(Fraction(float(x[i]))) for x in xs)
            assert abs(Fraction(float(s[i])) - exact) <= exact_abs * Fraction(n, 2 ** 52)
        assert np.array_equal(bufs[root].view(np.float32), s.astype(np.float32))
        for r in range(n):
            if r != root:
                assert np.array_equal(bufs[r], u8(xs[r])) and hs[r] not in o.reduce_ref
    # integer inputs: exact, equal to python's integer sum
    ints = [np.arange(-8, 8) * (r + 1) for r in range(3)]
    o = WorldOracle(3)
    o.create(0, (0, 1, 2))
    bufs = [u8(v.astype(np.float32)).copy() for v in ints]
    for r in range(3):
        o.post_reduce(0, r, 2, bufs[r], 16, F32)
    assert [int(v) for v in bufs[2].view(np.float32)] == [sum(int(v[i]) for v in ints) for i in range(16)]


@pytest.mark.parametrize("n", [2, 3, 4])
def test_all_gather_gather_scatter_brute_force(n):
    count = 5
    send = [rand_bytes(count * 2, 60 + 10 * n + r) for r in range(n)]
    # all-gather: byte j of rank q's tensor lands at q*S + j on every rank
    o = WorldOracle(n)
    o.create(0, tuple(range(n)))
    recv = [np.full(n * count * 2 + 3, 0xA5, np.uint8) for _ in range(n)]
    keep = [s.copy() for s in send]
    hs = [o.post_all_gather(0, r, send[r], recv[r], count, BF16) for r in reversed(range(n))]
    assert all(o.status(h) == DONE for h in hs)
    for r in range(n):
        for q in range(n):
            for j in range(count * 2):
                assert recv[r][q * count * 2 + j] == keep[q][j]
        assert np.all(recv[r][n * count * 2:] == 0xA5) and np.array_equal(send[r], keep[r])
    for root in range(n):
        # gather: the same concatenation, on the root only
        o = WorldOracle(n)
        o.create(0, tuple(range(n)))
        groot = np.full(n * count * 2, 0xA5, np.uint8)
        hs = [o.post_gather(0, r, root, send[r], groot if r == root else None, count, BF16) for r in range(n)]
        assert all(o.status(h) == DONE for h in hs)
        assert np.array_equal(groot, recv[0][: n * count * 2])
        # scatter undoes gather: rank r gets back its own tensor
        back = [np.full(count * 2, 0xA5, np.uint8) for _ in range(n)]
        hs = [o.post_scatter(0, r, root, groot if r == root else None, back[r], count, BF16) for r in range(n)]
        assert all(o.status(h) == DONE for h in hs)
        for r in range(n):
            assert np.array_equal(back[r], keep[r])
            for j in range(count * 2):
                assert oracle.scatter_result(groot, n, r)[j] == groot[r * count * 2 + j]


def test_all_gather_in_place_and_rooted_mismatch():
    n, count = 3, 4
    o = WorldOracle(n)
    o.create(0, (0, 1, 2))
    recv = [rand_bytes(n * count * 4, 90 + r) for r in range(n)]
    mine = [recv[r][r * count * 4 : (r + 1) * count * 4].copy() for r in range(n)]
    # each rank's contribution already sits in its own slot of its receive buffer
    hs = [o.post_all_gather(0, r, recv[r][r * count * 4 : (r + 1) * count * 4], recv[r], count, F32) for r in range(n)]
    assert all(o.status(h) == DONE for h in hs)
    for r in range(n):
        assert np.array_equal(recv[r], np.concatenate(mine))
    b = [rand_bytes(16, r) for r in range(n)]
    hs = [o.post_reduce(0, r, r % 2, b[r], 4, F32) for r in range(n)]  # roots disagree
    assert all(o.status(h) == MISMATCH for h in hs)
    hs = [o.post_gather(0, 0, 0, b[0], np.zeros(48, np.uint8), 4, F32), o.post_scatter(0, 1, 0, None, b[1], 4, F32),
          o.post_gather(0, 2, 0, b[2], None, 4, F32)]  # kinds disagree
    assert all(o.status(h) == MISMATCH for h in hs)
    pend = o.post_all_gather(0, 0, b[0], np.zeros(48, np.uint8), 4, F32)
    o.abort_world(0)
    assert o.status(pend) == BROKEN
