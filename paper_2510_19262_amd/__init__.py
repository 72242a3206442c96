"""railsched: batched LPT rail spraying of MoE all-to-all traffic on one MI355X.

Thin ctypes binding over librailsched.so (hand-written HIP kernels for gfx950).
Every step of the path runs in those kernels; this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    Topo, RailschedError, lib_path, load, version, strerror,
    route_topk, traffic_matrix, traffic_matrix_workspace_bytes, check_capacity, chunk_total, route_traffic, route_traffic_workspace_bytes, chunk_sort, chunk_count, lpt_spray, lpt_spray_workspace_bytes, eval, evaluate,
    chunk_sort_workspace_bytes, eval_workspace_bytes, schedule, schedule_static, STATIC_SCRATCH_BYTES, schedule_workspace_bytes, Plan, transpose_matrix, assign_policy, POLICIES, port_round_robin,
)
