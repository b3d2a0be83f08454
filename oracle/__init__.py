"""CPU oracle for the multi-world tensor data plane.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this
package: it exists so that tests, the smoke check and the benchmark's
CPU-baseline leg can compare the GPU library's results with a plain, slow,
obviously correct restatement of what the paper's worlds compute.  It is
numpy-only, shares no code with the HIP path and never imports it.
"""

from .mw_oracle import (  # noqa: F401
    ALIVE,
    BROKEN,
    DONE,
    MISMATCH,
    PENDING,
    F32,
    BF16,
    WorldOracle,
    copy_result,
    broadcast_result,
    allreduce_sum_f64,
    allreduce_sum_ordered,
    allreduce_within_tolerance,
    reduce_result_f64,
    all_gather_result,
    gather_result,
    scatter_result,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    broken_worlds_of_worker,
)
