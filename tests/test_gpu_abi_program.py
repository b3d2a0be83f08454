"""A compiled program that uses the C ABI directly (tests/abi_check.cpp: no Python, no torch in its process)."""

import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_compiled_program_drives_the_library_through_the_c_abi():
    from paper_2407_08980_amd import build

    exe = build.ABI_CHECK
    assert os.path.exists(exe), "not built: run `python -m paper_2407_08980_amd.build`"
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert p.returncode == 0 and "abi_check ok" in p.stdout, p.stdout[-2000:]


def test_header_is_plain_c(tmp_path):
    """include/mw.h must be usable from C99 (no C++ in the boundary)."""
    src = tmp_path / "t.c"
    src.write_text('#include "mw.h"\nint f(void) { mw_handle h = 0; return mw_poll(h) + (int)sizeof(mw_post_desc); }\n')
    p = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", "-I", os.path.join(ROOT, "include"),
                        str(src)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert p.returncode == 0, p.stdout


@pytest.mark.gpu
def test_the_latency_program_moves_the_right_bytes_in_both_modes():
    """pingpong.bin: single messages through the resident mailbox kernel and launched; it checks the payload itself.
    The timing is printed, not judged -- except that a message through the mailbox must not take longer than a launched
    one by more than measurement noise (the mailbox exists to save the launch)."""
    import json

    from paper_2407_08980_amd import build

    assert os.path.exists(build.PINGPONG), "run `python -m paper_2407_08980_amd.build`"
    p = subprocess.run([build.PINGPONG, "--iters", "500", "--sizes", "4,4096,32768,40000"], capture_output=True, text=True, timeout=120)
    assert p.returncode == 0, p.stdout[-1000:] + p.stderr[-1000:]
    rows = [json.loads(line) for line in p.stdout.splitlines() if line.startswith("{")]
    assert [(r["bytes"], r["mailbox"]) for r in rows] == [(b, m) for m in (1, 0) for b in (4, 4096, 32768, 40000)]
    by = {(r["bytes"], r["mailbox"]): r["total_us"]["median"] for r in rows}
    print(by)
    assert by[(32768, 1)] < by[(32768, 0)] * 1.1


@pytest.mark.gpu
def test_the_latency_programs_tensor_parallel_loop_runs_in_both_forms():
    import json

    from paper_2407_08980_amd import build

    p = subprocess.run([build.PINGPONG, "--tp", "--iters", "300"], capture_output=True, text=True, timeout=180)
    assert p.returncode == 0, p.stdout[-1000:] + p.stderr[-1000:]
    rows = [json.loads(line) for line in p.stdout.splitlines() if line.startswith("{")]
    assert [(r["mailbox"], r["iterations_in_flight"]) for r in rows] == [(m, d) for m in (1, 0) for d in (1, 2, 3, 4)]
    print({(r["mailbox"], r["iterations_in_flight"]): r["us_per_iteration"] for r in rows})
    assert all(0 < r["us_per_iteration"] < 1000 for r in rows)


@pytest.mark.gpu
def test_the_latency_programs_window_loop_moves_the_right_bytes():
    import json

    from paper_2407_08980_amd import build

    p = subprocess.run([build.PINGPONG, "--windows", "--iters", "300"], capture_output=True, text=True, timeout=180)
    assert p.returncode == 0, p.stdout[-1000:] + p.stderr[-1000:]  # (it checks the payload itself)
    rows = [json.loads(line) for line in p.stdout.splitlines() if line.startswith("{")]
    assert [(r["mailbox"], r["windows_in_flight"]) for r in rows] == [(m, d) for m in (1, 0) for d in (1, 2)]
    print({(r["mailbox"], r["windows_in_flight"]): r["us_per_message"] for r in rows})
