"""MI355X-native MGRIT-FAS (layer-parallel multigrid) solver for residual networks.

The product is the C-ABI library `libmgrit.so` (HIP kernels for gfx950, see include/mgrit.h);
this package is its thin Python binding.
"""
from .binding import (  # noqa: F401
    MgritError, mgrit_problem_t, make_problem, problem_from_workload, lib,
    mgrit_level_map, mgrit_workspace_bytes, mgrit_adjoint_workspace_bytes,
    mgrit_fas_forward, mgrit_fas_adjoint, mgrit_residual_norm, mgrit_trace_begin, mgrit_trace_end,
    mgrit_fas_forward_static, MGRIT_STATIC_SCRATCH_BYTES,
    mgrit_fc_layers_t, make_fc_layers, mgrit_workspace_bytes_mixed, mgrit_adjoint_workspace_bytes_mixed,
    mgrit_fas_forward_mixed, mgrit_fas_adjoint_mixed, mgrit_residual_norm_mixed,
)
