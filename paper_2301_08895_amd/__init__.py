"""MI355X-native ABS parameter-server round (libabs) and its thin Python binding.

The product is the C-ABI library `libabs.so` (see include/abs.h); this package
only loads it and marshals arguments.  There is no CPU fallback: importing
`binding` without a built library raises.
"""
from .binding import (AbsConfig, AbsError, abs_config_bytes, abs_workspace_size, abs_create,
                      abs_round, abs_get_model, abs_evaluate, abs_trace, abs_rounds_done, abs_kernel_stats,
                      abs_last_error, abs_destroy, abs_draw_time_ticks, abs_draw_batch_rows,
                      make_config, trace_stride, Simulation, library_path,
                      abs_batch_create, abs_batch_round, abs_batch_destroy, abs_batch_workspace_size, Batch,
                      abs_mlp_round_plan, abs_evaluate_static, abs_calibrate_mfma)

__all__ = ["AbsConfig", "AbsError", "abs_config_bytes", "abs_workspace_size", "abs_create",
           "abs_round", "abs_get_model", "abs_evaluate", "abs_trace", "abs_rounds_done", "abs_kernel_stats",
           "abs_last_error", "abs_destroy", "abs_draw_time_ticks", "abs_draw_batch_rows",
           "make_config", "trace_stride", "Simulation", "library_path",
           "abs_batch_create", "abs_batch_round", "abs_batch_destroy", "abs_batch_workspace_size", "Batch",
           "abs_mlp_round_plan", "abs_evaluate_static", "abs_calibrate_mfma"]
