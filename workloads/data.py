"""Seeded tensor contents.

Draws come from numpy's Philox counter-based generator keyed by an integer
seed, so a buffer's bytes depend only on its spec.  bf16 tensors are float32
draws rounded to nearest-even and stored as 16-bit patterns.

Large payloads (hundreds of MiB) are cut from a fixed pool of N(0,1) draws at
a seeded element offset (wrapping around): drawing tens of GiB of fresh
normals on the host would dominate every run without changing what the data
plane sees, which is opaque bytes with the value distribution of activations.
"""

from __future__ import annotations

from dataclasses import dataclass

import numpy as np

ITEMSIZE = {"f32": 4, "bf16": 2}
POOL_ELEMS = 1 << 24  # elements per pool (64 MiB of f32, 32 MiB of bf16)
POOL_SEED = {"f32": 0x6D775F66, "bf16": 0x6D775F62}


def rng_of(seed):
    return np.random.Generator(np.random.Philox(key=int(seed)))


def round_to_bf16_bits(x32):
    """float32 -> bf16 bit patterns, round to nearest, ties to even (finite inputs)."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def _encode(x32, dtype):
    if dtype == "f32":
        return np.ascontiguousarray(x32, dtype=np.float32).view(np.uint8)
    return round_to_bf16_bits(x32).view(np.uint8)


@dataclass(frozen=True)
class BufSpec:
    """One device buffer: its size and the recipe for its initial bytes.

    init is one of
      ("normal", dtype, seed)        N(0,1)
      ("uniform", dtype, seed)       U(-1,1)
      ("ints", dtype, seed, bound)   integers in [-bound, bound] (exact sums)
      ("bytes", seed)                uniform random bytes (arbitrary bit patterns)
      ("fill", byte)                 constant byte (0xA5 poison for destinations)
      ("pool", dtype, offset)        N(0,1) pool slice starting at element offset
    """

    nbytes: int
    init: tuple

    @property
    def dtype(self):
        return self.init[1] if self.init[0] in ("normal", "uniform", "ints", "pool") else None


class HostPools:
    """Lazily drawn N(0,1) pools, one per dtype, shared by every pool-backed buffer."""

    def __init__(self):
        self._pools = {}

    def get(self, dtype):
        p = self._pools.get(dtype)
        if p is None:
            x = rng_of(POOL_SEED[dtype]).standard_normal(POOL_ELEMS, dtype=np.float32)
            p = _encode(x, dtype)
            self._pools[dtype] = p
        return p


def pool_slice(pool_bytes, dtype, offset, nbytes):
    """Bytes of a pool-backed tensor: element j is pool[(offset + j) mod POOL_ELEMS]."""
    isz = ITEMSIZE[dtype]
    total = POOL_ELEMS * isz
    start = (offset % POOL_ELEMS) * isz
    out = np.empty(nbytes, dtype=np.uint8)
    done = 0
    while done < nbytes:
        take = min(nbytes - done, total - start)
        out[done : done + take] = pool_bytes[start : start + take]
        done += take
        start = 0
    return out


def materialize(spec, pools=None):
    """Initial contents of a buffer as a fresh 1-D uint8 array of spec.nbytes."""
    kind = spec.init[0]
    n = spec.nbytes
    if kind == "fill":
        return np.full(n, spec.init[1], dtype=np.uint8)
    if kind == "bytes":
        return rng_of(spec.init[1]).integers(0, 256, size=n, dtype=np.uint8)
    dtype = spec.init[1]
    count = n // ITEMSIZE[dtype]
    assert count * ITEMSIZE[dtype] == n, "typed buffers hold whole elements"
    if kind == "pool":
        pools = pools or HostPools()
        return pool_slice(pools.get(dtype), dtype, spec.init[2], n)
    rng = rng_of(spec.init[2])
    if kind == "normal":
        x = rng.standard_normal(count, dtype=np.float32)
    elif kind == "uniform":
        x = (rng.random(count, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)
    elif kind == "ints":
        b = int(spec.init[3])
        x = rng.integers(-b, b + 1, size=count).astype(np.float32)
    else:
        raise ValueError(f"unknown init {kind}")
    return np.array(_encode(x, dtype), copy=True)
