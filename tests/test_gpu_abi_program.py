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
