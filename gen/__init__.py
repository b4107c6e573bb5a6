"""Seeded synthetic inputs (cluster snapshots and arrival traces).

This package only draws random problem data: shapes, distributions and
structure of the workloads.  It holds none of the scheduling method's
arithmetic, and is the one module both the CPU oracle's tests and the HIP
path's tests/bench feed from.
"""
from .configs import (  # noqa: F401
    TYPE_CPU, TYPE_GPU, TYPE_API,
    MODEL_NONE, MODEL_AMDAHL, MODEL_TABLE,
    make_config, make_random_problem, make_trace, subset_problem, slice_problem, with_fixed_dop, with_core_maps, with_extra_quotas,
    random_trace, trace_with_aux, trace_with_services, trace_with_pooled_gpus, with_shared_nodes,
    PROBLEM_ARRAYS, TRACE_ARRAYS,
)
