"""Are the host-runtime tests sharp?  Each case plants ONE mistake in a copy of csrc/mw_host.cpp (a queue served
from the wrong end, an abort that forgets a class of pending operations, a fence that lets posts through, a
fault set that is too large, ...), builds it with the byte-less device double and runs the host tests -- among
them the random comparison with the oracle -- against that build in a child process: they must fail.
CPU only; the product library and the GPU are not involved."""

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2407_08980_amd", "csrc")

# (name, text in mw_host.cpp, replacement)
MUTANTS = [
    ("point-to-point queue served from the back", "Post other = theirs.front();\n  theirs.pop_front();",
     "Post other = theirs.back();\n  theirs.pop_back();"),
    ("dtype disagreement goes unnoticed", "if (other.count != me.count || other.dtype != me.dtype) {", "if (other.count != me.count) {"),
    ("abort forgets the unmatched receives", "    for (const Post& p : kv.second.recvs) finish_handle(c, p.hslot, MW_BROKEN);\n", ""),
    ("abort forgets the pending collectives", "      if (cl.have[r]) finish_handle(c, cl.post[r].hslot, MW_BROKEN);", "      (void)cl;"),
    ("posts to a broken world are accepted", "  if (count > (SIZE_MAX >> 3)) return MW_EINVAL;\n  if (w.state == MW_BROKEN) return MW_EBROKEN;",
     "  if (count > (SIZE_MAX >> 3)) return MW_EINVAL;"),
    ("all ranks of a world share one collective sequence counter", "uint32_t seq = w.coll_next[rank]++;", "uint32_t seq = w.coll_next[0]++;"),
    ("root disagreement goes unnoticed", "same &= f.kind[r] == f.kind[0] && f.root[r] == f.root[0] &&", "same &= f.kind[r] == f.kind[0] &&"),
    ("a failed worker breaks every world", "  for (uint32_t wi : c.worlds_of_worker[(size_t)worker_id]) {\n    int r = abort_world_locked(c, *c.worlds[wi]);",
     "  for (uint32_t wi = 0; wi < c.worlds.size(); ++wi) {\n    int r = abort_world_locked(c, *c.worlds[wi]);"),
    ("broadcast descriptor starts with rank 0 instead of the root", "      l.buf[at++] = f.post[rt].buf;\n      for (int r = 0; r < n; ++r)\n        if (r != rt) l.buf[at++] = f.post[r].buf;",
     "      for (int r = 0; r < n; ++r) l.buf[at++] = f.post[r].buf;"),
    ("copy descriptor has source and destination swapped", "  l.buf[0] = pair[0].buf;\n  l.buf[1] = pair[1].buf;", "  l.buf[0] = pair[1].buf;\n  l.buf[1] = pair[0].buf;"),
    ("live handles are recycled", "    if (e.status.load(std::memory_order_relaxed) == MW_PENDING) continue;  // still live: never recycle\n", ""),
    ("ring slots are never given back", "  slot_release(w, op.l.slot - w.first_slot);\n  op.state = kOpFree;", "  op.state = kOpFree;"),
    ("completion generation is not advanced", "uint32_t gen = c.slot_gen[slot] + 1;", "uint32_t gen = c.slot_gen[slot] + (slot & 1);"),
    ("matched operations of an aborted world are dropped", "  // Operations that already had all their sides are delivered: launch them now so that they retire.\n  int rc2 = flush_locked(c);",
     "  for (uint32_t opi : c.ready) if (&*c.worlds[c.ops[opi].world] == &w) for (int i = 0; i < c.ops[opi].n_handles; ++i) finish_handle(c, c.ops[opi].handles[i], MW_BROKEN);\n  int rc2 = flush_locked(c);"),
    ("watchdog takes a report exactly as old as the timeout for a miss", "!(now - c.last_beat[k] > timeout)", "!(now - c.last_beat[k] >= timeout)"),
    ("watchdog aborts the worlds of every watched worker", "    for (uint32_t wi : c.worlds_of_worker[k]) abort_world_locked(c, *c.worlds[wi]);",
     "    for (size_t q = 0; q < c.beating.size(); ++q) if (c.beating[q]) for (uint32_t wi : c.worlds_of_worker[q]) abort_world_locked(c, *c.worlds[wi]);"),
    ("a poll without the lock never looks at the completion word", "(fs != kNone && c.dev->flag(fs) != fg && !c.dev->needs_attention())", "(fs != kNone && !c.dev->needs_attention())"),
    ("a poll without the lock takes a launched operation for a complete one", "  if (st != MW_PENDING) {\n    *state = st;\n    return true;\n  }\n  if (op == kNone",
     "  if (st != MW_PENDING || fs != kNone) {\n    *state = fs != kNone ? MW_DONE : st;\n    return true;\n  }\n  if (op == kNone"),
    ("a poll without the lock does not notice work left without a kernel", "(fs != kNone && c.dev->flag(fs) != fg && !c.dev->needs_attention())",
     "(fs != kNone && c.dev->flag(fs) != fg)"),
    ("a poll under the lock does not start a kernel for work left without one",
     "  if (c.dev->needs_attention()) {  // it may sit in the resident kernel's queue with no kernel open: start one\n    int rc = c.dev->attend();\n    if (rc != MW_OK) return rc;\n  }\n",
     ""),
    ("the allocation-free variant pairs a side with a side of its own kind", "posts[j].kind == 1 - p.kind", "posts[j].kind == p.kind"),
    ("the allocation-free variant lets a rank's later collective overtake its earlier one",
     "posts[j].world_id == p.world_id && side[posts[j].a] < 0)\n          side[posts[j].a] = j;",
     "posts[j].world_id == p.world_id)\n          side[posts[j].a] = j;"),
    ("a zero-length message waits for a launch", "  if (count == 0) {\n    finish_handle(c, hs, MW_DONE);\n    finish_handle(c, other.hslot, MW_DONE);\n    return MW_OK;\n  }\n", ""),
]


@pytest.fixture(scope="module")
def source():
    return open(os.path.join(CSRC, "mw_host.cpp")).read()


@pytest.fixture(scope="module")
def builds(tmp_path_factory, source):
    """Every mutant compiled once, a few at a time."""
    out = tmp_path_factory.mktemp("host_mutants")

    def build(i):
        name, old, new = MUTANTS[i]
        assert source.count(old) == 1, name
        d = out / f"m{i}"
        d.mkdir()
        src = d / "mw_host.cpp"
        src.write_text(source.replace(old, new).replace('#include "../../include/mw.h"', f'#include "{ROOT}/include/mw.h"')
                       .replace('#include "mw_internal.hpp"', f'#include "{CSRC}/mw_internal.hpp"'))
        lib = d / "libmw_hostcheck.so"
        p = subprocess.run(["g++", "-O0", "-std=c++17", "-fPIC", "-shared", "-pthread", str(src),
                            os.path.join(CSRC, "mw_device_null.cpp"), "-o", str(lib)],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert p.returncode == 0, p.stdout[-2000:]
        return str(lib)

    with ThreadPoolExecutor(4) as pool:
        return list(pool.map(build, range(len(MUTANTS))))


def _limit_memory():
    import resource

    resource.setrlimit(resource.RLIMIT_AS, (8 << 30, 8 << 30))  # a broken runtime must not eat the machine


def run_host_tests(lib):
    env = dict(os.environ, MW_HOSTCHECK_UNDER_TEST=lib, PYTHONDONTWRITEBYTECODE="1")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "--timeout", "120",
                           os.path.join(ROOT, "tests", "test_host_logic.py"),
                           os.path.join(ROOT, "tests", "test_host_vs_oracle_fuzz.py"),
                           os.path.join(ROOT, "tests", "test_watchdog.py"),
                           os.path.join(ROOT, "tests", "test_host_noalloc.py"),
                           "-k", "not cost and not product_library and not oracle_watchdog"],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600,
                          preexec_fn=_limit_memory)


@pytest.mark.parametrize("i", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_host_tests_catch_a_planted_mistake(builds, i):
    p = run_host_tests(builds[i])
    assert p.returncode != 0, f"not noticed: {MUTANTS[i][0]}\n{p.stdout[-1500:]}"
    assert "failed" in p.stdout or "error" in p.stdout.lower(), p.stdout[-1500:]
