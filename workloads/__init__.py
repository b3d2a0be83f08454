"""Seeded synthetic inputs and operation traces for the five workloads.

This package only draws random numbers and lays out lists of operations.  It
contains none of the data plane's arithmetic or matching logic and imports
neither the GPU library nor the CPU oracle; both consume what it emits.
"""

from .data import BufSpec, HostPools, materialize  # noqa: F401
from .trace import Op, Trace  # noqa: F401
from .configs import (  # noqa: F401
    BASE_SEED,
    config1,
    config2,
    config3,
    config4,
    config5,
    collectives_mix,
    online_recovery,
    multi_sender,
    single_world_of,
)
