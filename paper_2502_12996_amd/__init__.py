"""MI355X-native optimizer sweep of DiLoCo with eager outer updates (arXiv 2502.12996).

`binding` wraps the C-ABI library (HIP kernels for gfx950), `workloads` holds the
synthetic benchmark configurations and seeded input generators, `build` compiles the
library in-tree.  The shared library is loaded on first use and there is no fallback.
"""
from . import binding, workloads  # noqa: F401
from .binding import (SWEEP_READ, SWEEP_RMW, SWEEP_WRITE, BF16, COMM_BF16, COMM_EXMY, STATE_NO_MEAN, STATE_TILE, DELAYED, EAGER, F32, DilocoError, inner_adamw, outer_eager,  # noqa: F401
                      outer_eager_packed, outer_eager_overlap2, outer_eager_pingpong, outer_sync, pack_state, packed_state_elems, packed_window,
                      reset_packed, unpack_state, reset, sim_loss_workspace, sim_quadratic_inner, sim_quadratic_phase,
                      sim_quadratic_loss, sim_quadratic_loss_static, sim_stream_copy, sim_stream_rmw, sim_stream_sweep, stream_boundary_count, stream_due,
                      stream_offset, strerror, tune, tune_get, version)
