"""Are the oracle's pins sharp?  Each case plants ONE plausible mistake in a copy of the oracle (a dropped
rank, a wrong shift, a transposed operand, a queue served from the wrong end, a fault set that is too large or
too small, ...) and runs the pin tests against that copy in a child process: at least one pin must fail for
every mistake.  The mistakes live in a temporary copy on the CPU; the real oracle and the GPU are not involved."""

import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text in oracle/mw_oracle.py, replacement)
MUTANTS = [
    ("bf16 widened by the wrong shift", "<< np.uint32(16)).view(np.float32)", "<< np.uint32(15)).view(np.float32)"),
    ("bf16 rounding truncates", "(u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)", "(u) >> np.uint64(16)"),
    ("bf16 rounding: ties away from even", "(u + np.uint64(0x7FFF) + lsb)", "(u + np.uint64(0x8000))"),
    ("copy delivers the receiver's own bytes", "_as_bytes(rbuf)[:nb] = copy_result(_as_bytes(sbuf)[:nb])",
     "_as_bytes(sbuf)[:nb] = copy_result(_as_bytes(rbuf)[:nb])"),
    ("copy moves one element too few", "nb = count * _ITEMSIZE[dtype]\n                    _as_bytes(rbuf)",
     "nb = (count - 1) * _ITEMSIZE[dtype]\n                    _as_bytes(rbuf)"),
    ("p2p queue served from the back", "oh, obuf, ocount, odtype = q.popleft()", "oh, obuf, ocount, odtype = q.pop()"),
    ("p2p queues shared by all pairs", "q = theirs.get((src, dst))", "q = next((v for v in theirs.values() if v), None)"),
    ("count disagreement goes unnoticed", "if (ocount, odtype) != (count, dtype):", "if odtype != dtype:"),
    ("broadcast takes rank 0's tensor", "rootb = _as_bytes(bufs[root])", "rootb = _as_bytes(bufs[0])"),
    ("broadcast leaves the last rank out", "                if r != root:\n                    raws[r][:] = out[r]",
     "                if r != root and r != n - 1:\n                    raws[r][:] = out[r]"),
    ("all-reduce drops the last rank", "    for b in bufs:\n        v = _values_f64(_as_bytes(b), count, dtype)",
     "    for b in bufs[:-1] if len(bufs) > 2 else bufs:\n        v = _values_f64(_as_bytes(b), count, dtype)"),
    ("all-reduce subtracts", "        s += v\n", "        s -= v\n"),
    ("ordered sum runs in descending rank order", "    acc = None\n    for b in bufs:", "    acc = None\n    for b in list(bufs)[::-1]:"),
    ("ordered sum accumulates in float64", "(acc + v).astype(np.float32)", "(acc.astype(np.float64) + v)"),
    ("all-reduce leaves rank 0 untouched", "                if kind == \"allreduce\" or r == root:\n                    raws[r][:] = outb",
     "                if (kind == \"allreduce\" and r > 0) or (kind == \"reduce\" and r == root):\n                    raws[r][:] = outb"),
    ("reduce writes every rank", "                if kind == \"allreduce\" or r == root:\n                    raws[r][:] = outb",
     "                raws[r][:] = outb"),
    ("gather concatenates in reverse rank order", "def gather_result(send_bufs):\n    \"\"\"gather: the root receives the ranks' tensors concatenated in rank order.\"\"\"\n    return np.concatenate([_as_bytes(b) for b in send_bufs])",
     "def gather_result(send_bufs):\n    return np.concatenate([_as_bytes(b) for b in send_bufs][::-1])"),
    ("scatter hands out the wrong slice", "raw[rank * k : (rank + 1) * k]", "raw[(n - 1 - rank) * k : (n - rank) * k]"),
    ("collectives of a world run out of sequence", "seq = w.coll_next[rank]\n        w.coll_next[rank] += 1", "seq = w.coll_next[rank]"),
    ("root disagreement goes unnoticed", "sig = {(p[1], p[2], p[4], p[5]) for p in posts}", "sig = {(p[1], p[4], p[5]) for p in posts}\n        posts = [(p[0], p[1], posts[0][2]) + tuple(p[3:]) for p in posts]"),
    ("a failed worker breaks every world", "return {w for w, members in worlds.items() if worker in members}", "return set(worlds)"),
    ("a failed worker breaks only its first world", "return {w for w, members in worlds.items() if worker in members}",
     "return set(sorted(w for w, members in worlds.items() if worker in members)[:1])"),
    ("abort forgets the pending collectives", "        for slot in w.coll:\n            for post in slot.values():\n                self.result[post[0]] = BROKEN\n", ""),
    ("abort forgets the unmatched receives", "for table in (w.sends, w.recvs):", "for table in (w.sends,):"),
    ("abort also fails what was delivered", "        w.state = BROKEN\n        for table in", "        w.state = BROKEN\n        self.result[:] = [BROKEN if r == DONE else r for r in self.result]\n        for table in"),
    ("posts to a broken world are accepted", "        if w.state == BROKEN:  # access to a broken world is refused\n            return self._new(BROKEN)\n", ""),
    ("watchdog compares with >=  instead of >", "t - tb > timeout", "t - tb >= timeout"),
    ("watchdog ignores the latest heartbeat", "self.last_beat[worker] = max(t, self.last_beat.get(worker, t))",
     "self.last_beat.setdefault(worker, t)"),
]


@pytest.fixture(scope="module")
def source():
    return open(os.path.join(ROOT, "oracle", "mw_oracle.py")).read()


def test_every_mutation_is_a_single_edit(source):
    for name, old, new in MUTANTS:
        assert source.count(old) == 1, name


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_a_planted_mistake(tmp_path, source, name, old, new):
    pkg = tmp_path / "oracle"
    shutil.copytree(os.path.join(ROOT, "oracle"), pkg, ignore=shutil.ignore_patterns("__pycache__"))
    (pkg / "mw_oracle.py").write_text(source.replace(old, new))
    env = dict(os.environ, MW_ORACLE_UNDER_TEST=str(tmp_path), PYTHONDONTWRITEBYTECODE="1")
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_watchdog.py"), "-k", "not runtime and not thread"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode == 1, f"no pin noticed: {name}\n{p.stdout[-1500:]}"
    assert "passed" in p.stdout or "failed" in p.stdout  # the run got as far as running tests


def test_the_unmodified_copy_passes(tmp_path):
    shutil.copytree(os.path.join(ROOT, "oracle"), tmp_path / "oracle", ignore=shutil.ignore_patterns("__pycache__"))
    env = dict(os.environ, MW_ORACLE_UNDER_TEST=str(tmp_path), PYTHONDONTWRITEBYTECODE="1")
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_watchdog.py"), "-k", "not runtime and not thread"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode == 0, p.stdout[-1500:]
