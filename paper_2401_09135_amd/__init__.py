"""Asynchronous Local-SGD hot path on MI355X: thin Python binding over libals.so.

The binding only marshals arguments (ctypes) and uses torch for device memory and streams;
every step of the path runs inside the library's HIP kernels.  Importing this package fails
loudly if the library has not been built (``python paper_2401_09135_amd/build.py``).
"""
from .binding import (RULE_BUFFER, RULE_DN, OuterRule, ALS_DTYPE_BF16, ALS_DTYPE_F32, AlsError, Config, Context, VEC, dylu_schedule,
                      k_adamw, k_attention_bwd, k_attention_fwd, k_dn_group, k_gemm, k_gemm_ex, k_gemm_static_ws, k_gemm_dw_grouped, k_gemm_dw_grouped_ws_bytes, STATIC_WS_BYTES, lib, lr_schedule, shard_sample, lib_path,
                      param_count, param_count_decayed, param_offsets, prof_collect, prof_enable, set_gemm_tile)
from .driver import run_async

__all__ = ["RULE_BUFFER", "RULE_DN", "OuterRule", "ALS_DTYPE_BF16", "ALS_DTYPE_F32", "AlsError", "Config", "Context", "VEC",
           "dylu_schedule", "k_adamw", "k_attention_bwd", "k_attention_fwd", "k_dn_group", "k_gemm", "k_gemm_ex", "k_gemm_static_ws", "k_gemm_dw_grouped", "k_gemm_dw_grouped_ws_bytes", "STATIC_WS_BYTES",
           "lib", "lib_path", "param_count", "param_count_decayed", "param_offsets", "prof_collect", "prof_enable", "run_async", "set_gemm_tile"]
