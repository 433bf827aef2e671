"""MI355X-native Dynamic Beam Allocation step (Post & Vilar 2018, Alg. 2).

The product is libdba.so (HIP, gfx950) declared in include/dba.h; this package
is its ctypes binding.  PyTorch is used by callers only to own device memory
and streams.
"""
from .binding import (DBA_EHIP, DBA_EINVAL, DBA_ENOMEM, DBA_ESTATE, DBA_FLAG_DEAD,  # noqa: F401
                      DBA_FLAG_FINISHED, DBA_LOGP_BF16, DBA_LOGP_F16, DBA_LOGP_F32, DBA_MAX_BEAM,
                      DBA_MAX_CONS_TOKENS, DBA_NOALLOC_MAX_ROWS, DBA_OK, DBA_OPT_ADJUSTMENT,
                      DBA_OPT_MERGE_WAVES, DBA_OPT_NORMALIZE_FINISHED, DBA_OPT_PRUNE_THRESHOLD, DBA_OPT_TRACK_COMPLETED, DBA_STOP_ALL, DBA_STOP_ANY,
                      DbaError, dba_debug_allocate, dba_debug_row_max, dba_debug_wave_select, dba_destroy, dba_finalize,
                      dba_get_finished, dba_get_state, dba_init, dba_last_error, dba_set_option, dba_step,
                      dba_step_fmt, dba_step_noalloc, dba_steps_done, dba_workspace_bytes, load)
