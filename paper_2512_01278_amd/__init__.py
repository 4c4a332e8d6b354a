"""PillarAttn hot path for MI355X: hand-written HIP kernels behind a C ABI.

`binding` mirrors include/pillar.h one to one; `build` compiles csrc/ with
hipcc for gfx950.  Importing this package loads nothing: the shared library
is opened on first use and its absence is an error, never a fallback.
"""
from . import binding
from .binding import (PILLAR_FLAG_EXACT_SCORES, PILLAR_FLAG_GENERIC_KERNELS, KvCache, DeviceWorkload, PillarError, upload_workload, pillar_version,
                      pillar_workspace_bytes, pillar_verify_attn, pillar_verify_select, pillar_verify_hetero, pillar_mixed_step, pillar_select_topk,
                      pillar_sparse_decode, pillar_sparse_decode_static, pillar_window_indices, pillar_extend_indices, pillar_append_kv, pillar_profile_enable, pillar_profile_reset,
                      pillar_profile_read, pillar_set_option, pillar_bench_read, status_string)

__all__ = ["binding", "PILLAR_FLAG_EXACT_SCORES", "PILLAR_FLAG_GENERIC_KERNELS", "KvCache", "DeviceWorkload", "PillarError", "upload_workload", "pillar_version",
           "pillar_workspace_bytes", "pillar_verify_attn", "pillar_verify_select", "pillar_verify_hetero", "pillar_mixed_step", "pillar_select_topk", "pillar_sparse_decode", "pillar_sparse_decode_static", "pillar_window_indices", "pillar_extend_indices", "pillar_append_kv",
           "pillar_profile_enable", "pillar_profile_reset", "pillar_profile_read", "pillar_set_option", "pillar_bench_read", "status_string"]
