"""MI355X-native selective-recompute prefill (hot path of VLCache, arxiv 2512.12977).

Thin ctypes binding over libvlcache.so (hand-written HIP kernels behind a C ABI).  Every step of
the path runs inside the library; this package only marshals arguments.  Importing the package
does not load the library; the first call does, and raises if it has not been built
(`python -m paper_2512_12977_amd.build`).
"""
from .binding import (VlcError, lib, lib_path, last_error, VLC_F32, VLC_BF16,
                      vlc_plan_layer_rates, vlc_plan_layer_rates_blocks, vlc_plan_token_indices, vlc_plan_reuse_rows, vlc_plan_next_rows, vlc_plan_budget_steps,
                      vlc_gather_rows, vlc_rope_shift_kv, vlc_rope_shift_kv_layers, shift_job_table, vlc_scatter_kv, vlc_sparse_q_attention,
                      vlc_layer_workspace_bytes, vlc_layer_workspace_layout, vlc_layer_forward,
                      vlc_layer_forward_timed, vlc_layer_forward_chained, LAYER_STAGES, vlc_first_token_workspace_bytes, vlc_first_token,
                      vlc_first_token_noalloc, vlc_first_token_noalloc_max_bytes,
                      vlc_mean_squared_error, vlc_mean_squared_error_workspace_bytes, vlc_probe_mfma_bf16,
                      Segment, LayerShape, LayerWeights, LayerPlan, ShiftJob)

__all__ = ["VlcError", "lib", "lib_path", "last_error", "VLC_F32", "VLC_BF16",
           "vlc_plan_layer_rates", "vlc_plan_layer_rates_blocks", "vlc_plan_token_indices", "vlc_plan_reuse_rows", "vlc_plan_next_rows", "vlc_plan_budget_steps",
           "vlc_gather_rows", "vlc_rope_shift_kv", "vlc_rope_shift_kv_layers", "shift_job_table", "vlc_scatter_kv", "vlc_sparse_q_attention",
           "vlc_layer_workspace_bytes", "vlc_layer_workspace_layout", "vlc_layer_forward", "vlc_layer_forward_timed", "vlc_layer_forward_chained", "LAYER_STAGES",
           "vlc_first_token_workspace_bytes", "vlc_first_token", "vlc_first_token_noalloc",
           "vlc_first_token_noalloc_max_bytes", "vlc_mean_squared_error",
           "vlc_mean_squared_error_workspace_bytes", "vlc_probe_mfma_bf16",
           "Segment", "LayerShape", "LayerWeights", "LayerPlan", "ShiftJob"]
