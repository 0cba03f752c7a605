"""fp64 CPU oracle (test infrastructure only; see taper_oracle.c).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It never imports the GPU package.
"""
from .oracle import (  # noqa: F401
    OracleInts,
    attention,
    attention_segments,
    attention_slots,
    kv_append,
    resolve_segments,
    build,
    resolve,
)
