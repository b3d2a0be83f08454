"""The host runtime under AddressSanitizer + UndefinedBehaviorSanitizer (single-threaded random stress of the
whole C ABI) and under ThreadSanitizer (posting threads, a completion thread, heartbeats and the watchdog
thread).  Host code only: the runtime is linked against the byte-less device double."""

import os
import subprocess

import pytest

from helpers import ROOT

CSRC = os.path.join(ROOT, "paper_2407_08980_amd", "csrc")
SRCS = [os.path.join(ROOT, "tests", "host_stress.cpp"), os.path.join(CSRC, "mw_host.cpp"),
        os.path.join(CSRC, "mw_device_null.cpp")]


def _build_and_run(tmp_path, name, flags, args, env=None, srcs=None, opt="-O1"):
    exe = str(tmp_path / name)
    cmd = ["g++", "-std=c++17", opt, "-g", "-fno-omit-frame-pointer", "-pthread"] + flags + (srcs or SRCS) + ["-o", exe]
    b = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert b.returncode == 0, b.stdout
    e = dict(os.environ)
    e.pop("LD_PRELOAD", None)  # sanitizer runtimes must come first in the link order
    e.update(env or {})
    r = subprocess.run([exe] + args, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600, env=e)
    assert r.returncode == 0, r.stdout[-4000:]
    return r.stdout


def test_asan_ubsan_single_thread_stress(tmp_path):
    out = _build_and_run(tmp_path, "host_stress_asan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"],
                         [], {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0"})
    assert out.count("single:") == 3 and "ERROR" not in out


def test_tsan_threads_and_watchdog(tmp_path):
    out = _build_and_run(tmp_path, "host_stress_tsan", ["-fsanitize=thread"], ["threads"],
                         {"TSAN_OPTIONS": "halt_on_error=1"})
    assert "threads:" in out and "WARNING: ThreadSanitizer" not in out


POLL_SRCS = [os.path.join(ROOT, "tests", "poll_contention.cpp")] + SRCS[1:]


def _poll_table(out):
    rows = {}
    for line in out.splitlines():
        if line.startswith("threads"):
            f = line.replace(":", " ").split()
            rows[int(f[1])] = (float(f[2]), float(f[f.index("thread),") + 1]))
    return rows


def test_polls_without_the_lock_are_race_free(tmp_path):
    """Threads busy-polling in-flight operations read the handle table without the library lock while another
    thread posts, launches, completes and recycles entries: ThreadSanitizer must see no race."""
    out = _build_and_run(tmp_path, "poll_contention_tsan", ["-fsanitize=thread"], ["0.05"], {"TSAN_OPTIONS": "halt_on_error=1"},
                         srcs=POLL_SRCS)
    assert set(_poll_table(out)) == {1, 8, 16, 32} and "WARNING: ThreadSanitizer" not in out


def test_busy_polling_threads_do_not_slow_each_other_or_the_posting_thread(tmp_path):
    """The paper's model is one busy-waiting poller per worker (Sec. 3.3).  With 8 and 16 threads spinning on
    mw_poll a poll must stay far below the microseconds one lock hand-over costs (behind one lock it measured 1.1 us at
    8 threads, 1.9 us at 16 and 3.2 us at 32, and a posting thread's round went from 4.5 us to 26 us)."""
    out = _build_and_run(tmp_path, "poll_contention", [], ["0.2"], srcs=POLL_SRCS, opt="-O2")
    rows = _poll_table(out)
    assert rows[1][0] < 500 and rows[8][0] < 1000 and rows[16][0] < 2000, out
    if (os.cpu_count() or 1) >= 8:
        assert rows[8][1] < 4 * max(rows[1][1], 2000.0), out  # the thread that makes progress is not starved
