"""Compile the native libraries in-tree.

  libmw.so            the product: host runtime + HIP kernels for gfx950
  libmw_hostcheck.so  host runtime + a device test double that moves no bytes
                      (used only by the CPU tests of the host state machine)
"""

from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmw.so")
LIB_HOSTCHECK = os.path.join(HERE, "libmw_hostcheck.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=default",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if p.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build_product():
    srcs = [os.path.join(CSRC, "mw_device.hip"), os.path.join(CSRC, "mw_host.cpp")]
    return _run([HIPCC] + HIP_FLAGS + srcs + ["-o", LIB])


def build_hostcheck():
    srcs = [os.path.join(CSRC, "mw_host.cpp"), os.path.join(CSRC, "mw_device_null.cpp")]
    return _run(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread", "-Wall"] + srcs + ["-o", LIB_HOSTCHECK])


def build_all():
    out = build_product()
    out += build_hostcheck()
    return out


if __name__ == "__main__":
    sys.stdout.write(build_all())
    print("built", LIB, "and", LIB_HOSTCHECK)
