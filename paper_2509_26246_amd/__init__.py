"""libslimattn: sliced, asymmetric-unit causal attention for one MI355X (gfx950).

The package is a thin ctypes binding over the C-ABI library declared in include/slimattn.h.
Every step of the hot path runs in the library's HIP kernels; Python only marshals arguments.
Importing the package does not load the library; the first call does, and fails loudly if it
has not been built (python -m paper_2509_26246_amd.build).
"""
from .binding import (SlimAttnError, Tables, build_slices, build_slices_from_bounds, build_units, validate, solve_partition, solve_bottlenecks, dag_timeline, dag_build_1f1b, dag_buffers_1f1b, dag_memory, candidate_unit_counts, search_unit_count, shape_supported,
                      slice_pairs, flops_fwd, flops_bwd, tables_create, bwd_workspace_bytes, fwd, bwd, bwd_static, bwd_released_rows, STATIC_SCRATCH_BYTES, strerror,
                      version, load_library, POLICY_KINDS, F32, BF16, FLAG_PER_UNIT_LAUNCH, FLAG_STATS_PREPASS, CHECK_FORWARD,
                      CHECK_BACKWARD, CHECK_ORDER, EXPORTED_SYMBOLS, profile_enable, profile_read,
                      profile_read_launches, KERNEL_CLASSES)

__all__ = ["SlimAttnError", "Tables", "build_slices", "build_slices_from_bounds", "build_units", "validate", "solve_partition", "solve_bottlenecks", "dag_timeline", "dag_build_1f1b", "dag_buffers_1f1b", "dag_memory", "candidate_unit_counts", "search_unit_count", "shape_supported",
           "slice_pairs", "flops_fwd", "flops_bwd", "tables_create", "bwd_workspace_bytes", "fwd", "bwd", "bwd_static", "bwd_released_rows", "STATIC_SCRATCH_BYTES",
           "strerror", "version", "load_library", "POLICY_KINDS", "F32", "BF16", "FLAG_PER_UNIT_LAUNCH", "FLAG_STATS_PREPASS",
           "CHECK_FORWARD", "CHECK_BACKWARD", "CHECK_ORDER", "EXPORTED_SYMBOLS", "profile_enable", "profile_read",
           "profile_read_launches", "KERNEL_CLASSES"]
