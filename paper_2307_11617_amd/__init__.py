"""R-FAST activation rounds on MI355X: thin ctypes binding over librfast.so.

Nothing here computes: every step of the round runs in the HIP kernels.  The
library must have been built (python -m paper_2307_11617_amd.build); loading
fails loudly otherwise."""
from .binding import (RFAST_FIELDS, RFast, RFastError, RfastProblem, lib, rfast_check, rfast_common_roots, rfast_create,  # noqa: F401
                      rfast_destroy, rfast_diagnostics, rfast_diagnostics_static, rfast_init, rfast_kernel_time, rfast_last_error,
                      rfast_profile_enable, rfast_read_state, rfast_rebase, rfast_set_rebase_interval, rfast_set_optimizer, rfast_set_gamma_schedule, rfast_sync_round, rfast_sync_run, rfast_round, rfast_run, rfast_run_generated, rfast_run_events, rfast_use_graphs, rfast_use_blocks, rfast_block_info, rfast_set_tile_group, rfast_workspace_bytes,
                      rfast_write_state)
