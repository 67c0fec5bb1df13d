"""PSO-PS synchronization step on one MI355X: hand-written HIP kernels behind
a C-ABI library, with a thin ctypes binding."""

from .binding import (PSO_PS_EALIGN, PSO_PS_EHIP, PSO_PS_EINVAL, PSO_PS_ELIMIT, PSO_PS_ENOMEM,  # noqa: F401
                      PSO_PS_OK, PSO_PS_SINGLE_LAUNCH_MAX_K, PSO_PS_SINGLE_LAUNCH_MAX_PARAMS,
                      PSO_PS_STATIC_MAX_K, PsoPsError, pso_ps_average, pso_ps_create,
                      pso_ps_destroy, pso_ps_inertia, pso_ps_last_hip_error, pso_ps_last_selection,
                      pso_ps_pointer_table, pso_ps_schedule, pso_ps_set_launch,
                      pso_ps_set_single_launch, pso_ps_set_variant, pso_ps_source_hash,
                      pso_ps_strerror, pso_ps_sync, pso_ps_sync_begin, pso_ps_sync_finish,
                      pso_ps_sync_history, pso_ps_sync_rows, pso_ps_sync_rows_history,
                      pso_ps_sync_segments, pso_ps_sync_segments_history, pso_ps_sync_static)
