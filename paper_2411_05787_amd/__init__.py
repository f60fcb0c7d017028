"""RefreshKV decode-attention hot path for AMD MI355X (gfx950).

A thin ctypes binding over ``librefreshkv.so`` (hand-written HIP; C ABI declared in
``include/refreshkv.h``).  Every function here only marshals arguments: all arithmetic runs
in the HIP kernels.  PyTorch tensors are used as device memory and for the current stream.

Importing this package loads the shared library and fails if it has not been built
(``python paper_2411_05787_amd/build.py``): there is no CPU fallback.
"""
from .binding import (LIB_PATH, RkError, Geom, Workspace, lib, version, status_string, workspace_bytes,
                      rk_workspace_init, rk_full_attn, rk_full_attn_scores, rk_topk_select, rk_full_attn_select, rk_full_attn_pool, rk_select_pooled, rk_score_select, rk_window_select,
                      rk_gather_small_kv,
                      rk_partial_attn, rk_partial_attn_static, rk_partial_attn_static_bytes, rk_partial_attn_fixed, rk_partial_attn_lazy, rk_partial_attn_triggered, rk_query_sim, rk_mark_refresh, rk_calibration_copy, rk_calibration_read, rk_debug_set_slice_spin, rk_decode_step, rk_decode_step_overlapped, rk_refresh_batched, rk_full_attn_deferred, rk_decode_step_batched, layer_state, EXPORTS,
                      rk_h2o_append, rk_h2o_update, rk_h2o_step, h2o_state,
                      RK_AGG_MAX, RK_AGG_MEAN, RK_AGG_FIRST)
from .schedule import RefreshKVLayer, RefreshKVModel, RefreshKVStack

__all__ = ["LIB_PATH", "RkError", "Geom", "Workspace", "lib", "version", "status_string",
           "workspace_bytes", "rk_workspace_init", "rk_full_attn", "rk_full_attn_scores", "rk_topk_select",
           "rk_full_attn_select", "rk_full_attn_pool", "rk_select_pooled", "rk_score_select", "rk_window_select",
           "rk_gather_small_kv", "rk_partial_attn", "rk_partial_attn_static", "rk_partial_attn_static_bytes", "rk_partial_attn_fixed", "rk_partial_attn_lazy", "rk_partial_attn_triggered", "rk_query_sim", "rk_mark_refresh", "rk_calibration_copy", "rk_calibration_read", "rk_debug_set_slice_spin",
           "EXPORTS", "rk_h2o_append", "rk_h2o_update", "rk_h2o_step", "h2o_state",
           "rk_decode_step", "rk_decode_step_overlapped", "rk_refresh_batched", "rk_full_attn_deferred", "rk_decode_step_batched", "layer_state", "RK_AGG_MAX", "RK_AGG_MEAN", "RK_AGG_FIRST", "RefreshKVLayer", "RefreshKVModel", "RefreshKVStack"]
