"""Batched critical-path evaluation of data-flow DAGs on AMD MI355X.

The work is done by ``libcpeval.so`` (hand-written HIP for gfx950, C ABI in
``include/cpeval.h``).  This package is the thin binding: argument marshalling
with ctypes, PyTorch tensors for device memory and streams.
"""
from .binding import (  # noqa: F401
    CpError,
    CpGraph,
    CpProfile,
    OUT_PARTITION_MAJOR,
    OUT_VERTEX_MAJOR,
    PLAN_AUTO,
    PLAN_COLUMN_SLICE,
    PLAN_RESIDENT_WINDOW,
    PLAN_SHARED_WINDOW_2,
    PLAN_STREAMED_WINDOW,
    PLAN_SHARED_WINDOW_4,
    PLAN_WAVE_COLUMN,
    POLICY_FIFO,
    POLICY_PCT,
    cost_compact,
    cost_magic,
    cp_critical_path,
    cp_pct_order,
    cp_ranks,
    cp_search,
    cp_seed_partition,
    cp_simulate,
    cp_validate,
    cp_eval,
    cp_eval_static,
    error_string,
    load_library,
)
