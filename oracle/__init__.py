"""fp64 CPU oracle of the OBCache scoring / selection / compaction path.

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only the tests, the smoke check and the
benchmark's cpu_baseline leg may import this package.  It shares nothing with
the HIP library and never imports it.
"""
from .binding import (  # noqa: F401
    attn_score,
    build,
    compact,
    num_threads,
    score,
    adaptive_cap,
    select,
    select_adaptive,
    select_pooled,
    select_protected,
    vatp_score,
    window_attention,
)
