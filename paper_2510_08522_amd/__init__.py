"""MI355X-native gradient aggregate + statistics hot path (HIP kernels behind a C ABI)."""
from .binding import (  # noqa: F401
    DYNAMIX_BF16,
    DYNAMIX_F32,
    DYNAMIX_K_MAX,
    DYNAMIX_STATS_HEAD,
    STAT,
    DynamixError,
    dynamix_grad_aggregate_stats,
    dynamix_grad_aggregate_stats_ex,
    dynamix_plan_describe,
    dynamix_release_cached,
    dynamix_stats_count,
    dynamix_timing_begin,
    dynamix_timing_count,
    dynamix_timing_read,
    dynamix_status_string,
)
