"""fp64 CPU oracle for varlen packed attention.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares nothing with the HIP path and never imports it.
"""
from .binding import (  # noqa: F401
    build,
    fwd,
    fwd_rows,
    bwd,
    bwd_q_rows,
    bwd_kv_rows,
    merge,
    num_threads,
)
