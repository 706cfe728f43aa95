"""TEST INFRASTRUCTURE -- plain CPU oracle for the gradient aggregate + statistics path.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may use this package.
It shares no code with the HIP path and never imports it.
"""
from .dynamix_oracle import (  # noqa: F401
    HEAD,
    IDX,
    adam_step,
    aggregate_stats,
    build,
    max_threads,
    sgd_momentum_step,
    sgd_step,
    stats_count,
    widen,
)
