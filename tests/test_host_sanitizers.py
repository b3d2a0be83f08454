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


def _build_and_run(tmp_path, name, flags, args, env=None):
    exe = str(tmp_path / name)
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-pthread"] + flags + SRCS + ["-o", exe]
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
