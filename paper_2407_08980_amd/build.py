"""Compile the native libraries in-tree.

  libmw.so            the product: host runtime + HIP kernels for gfx950
  libmw_hostcheck.so  host runtime + a device test double that moves no bytes
                      (used only by the CPU tests of the host state machine)
  pingpong.bin        post-to-done time of one message through the C ABI (no interpreter in the loop)
"""

from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmw.so")
LIB_HOSTCHECK = os.path.join(HERE, "libmw_hostcheck.so")
ABI_CHECK = os.path.join(HERE, "abi_check.bin")  # tests/abi_check.cpp: a program that uses the C ABI directly
PINGPONG = os.path.join(HERE, "pingpong.bin")    # pingpong.cpp: post-to-done time of one message, from C

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=default",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def source_id():
    """First 16 hex digits of the SHA-256 over the native sources and the public header, in name order."""
    import hashlib

    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp", ".hpp")))
    files.append(os.path.join(os.path.dirname(HERE), "include", "mw.h"))
    for f in files:
        h.update(os.path.basename(f).encode() + b"\0")
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def _build_id_flag():
    return '-DMW_BUILD_ID="%s"' % source_id()


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if p.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build_product():
    srcs = [os.path.join(CSRC, "mw_device.hip"), os.path.join(CSRC, "mw_host.cpp")]
    return _run([HIPCC] + HIP_FLAGS + [_build_id_flag()] + srcs + ["-o", LIB])


def build_hostcheck():
    srcs = [os.path.join(CSRC, "mw_host.cpp"), os.path.join(CSRC, "mw_device_null.cpp")]
    return _run(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread", "-Wall", _build_id_flag()] + srcs + ["-o", LIB_HOSTCHECK])


def library_id(path):
    """Build identity stored in a built library, or None if it cannot be read."""
    import ctypes

    try:
        lib = ctypes.CDLL(path)
        lib.mw_build_id.restype = ctypes.c_char_p
        return lib.mw_build_id().decode()
    except (OSError, AttributeError):
        return None


def fresh_hostcheck():
    """Path of the host-check library, rebuilt first if it is missing or was made from other sources.  (A stale
    copy must be replaced before this process loads it: a loaded library is not reloaded from a new file.)"""
    import multiprocessing as mp

    stale = not os.path.exists(LIB_HOSTCHECK)
    if not stale:
        with mp.get_context("spawn").Pool(1) as pool:  # read the id in a child so the old file is never mapped here
            stale = pool.apply(library_id, (LIB_HOSTCHECK,)) != source_id()
    if stale:
        build_hostcheck()
    return LIB_HOSTCHECK


def build_abi_check():
    """The test program of the C ABI, linked against the product library beside it."""
    src = os.path.join(os.path.dirname(HERE), "tests", "abi_check.cpp")
    return _run([HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wno-unused-command-line-argument", src, "-o", ABI_CHECK,
                 "-L" + HERE, "-lmw", "-Wl,-rpath,$ORIGIN"])


def build_pingpong():
    """The latency tool, linked against the product library beside it."""
    return _run([HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wno-unused-command-line-argument", "-Wno-unused-result",
                 os.path.join(HERE, "pingpong.cpp"), "-o", PINGPONG, "-L" + HERE, "-lmw", "-Wl,-rpath,$ORIGIN"])


def build_all():
    out = build_product()
    out += build_hostcheck()
    out += build_abi_check()
    out += build_pingpong()
    return out


if __name__ == "__main__":
    sys.stdout.write(build_all())
    print("built", LIB, "and", LIB_HOSTCHECK)
