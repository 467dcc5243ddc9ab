"""fp64 CPU oracle for padded bidirectional sigmoid attention -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares no code with the HIP library and never imports it.
"""
from .sigmoid_attn_oracle import (  # noqa: F401
    build,
    threads,
    fwd,
    bwd,
    matrices,
    fwd_rows,
    bwd_q_rows,
    bwd_kv_rows,
    valid_flops,
    cross_fwd,
    cross_bwd,
)
