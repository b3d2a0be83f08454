"""The mailbox protocol without a GPU: the library's own host side (csrc/mw_mailbox.hpp) against threads that play
the resident kernel (tests/mailbox_model.cpp) -- kernels that close by idling out, by the host's request and by
their lifetime while the host keeps submitting, and launches that are refused now and then.  Every chunk of every descriptor must be executed exactly once, by the
worker that owns it, and every kernel thread must end; ThreadSanitizer must see no race in the host-side protocol."""

import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "mailbox_model.cpp")
INC = ["-I", os.path.join(ROOT, "paper_2407_08980_amd", "csrc"), "-I", os.path.join(ROOT, "include")]


def _run(tmp_path, name, flags, seconds, env=None):
    exe = str(tmp_path / name)
    subprocess.run(["g++", "-std=c++17", "-pthread", *flags, *INC, SRC, "-o", exe], check=True, capture_output=True, text=True)
    p = subprocess.run([exe, str(seconds)], capture_output=True, text=True, timeout=300, env={**os.environ, **(env or {})})
    assert p.returncode == 0, p.stdout + p.stderr
    return p.stdout + p.stderr


def _closes(out):
    rows = []
    for line in out.splitlines():
        if line.startswith("seed"):
            f = line.replace(",", " ").replace(")", " ").split()
            rows.append((int(f[f.index("idle") + 1]), int(f[f.index("stop") + 1]), int(f[f.index("life") + 1])))
    return rows


def test_every_chunk_is_executed_exactly_once_whatever_ends_the_kernels(tmp_path):
    out = _run(tmp_path, "mailbox_model", ["-O2"], 1.5)
    assert "all chunks executed exactly once" in out
    rows = _closes(out)
    assert len(rows) == 3
    # each way a kernel can end was exercised: idling out, the host's request, the lifetime
    assert sum(r[0] for r in rows) > 0 and sum(r[1] for r in rows) > 0 and sum(r[2] for r in rows) > 0, out
    # ... and launches of the kernel were refused now and then: the descriptors stayed queued and were served later
    refused = [line for line in out.splitlines() if "launches refused" in line]
    assert len(refused) == 1 and int(refused[0].split()[0]) > 0, out


def test_the_host_side_of_the_mailbox_is_race_free(tmp_path):
    out = _run(tmp_path, "mailbox_model_tsan", ["-O1", "-g", "-fsanitize=thread"], 0.6, {"TSAN_OPTIONS": "halt_on_error=1"})
    assert "all chunks executed exactly once" in out and "WARNING: ThreadSanitizer" not in out
