"""fp64 CPU oracle of the PillarAttn hot path (test infrastructure only)."""
from .pillar_oracle import (decode_tensor, e4m3_table, gather_request,
                            verify_attn, select_topk, sparse_decode, run_all,
                            window_indices, extend_indices, append_kv, mixed_step)

__all__ = ["decode_tensor", "e4m3_table", "gather_request", "verify_attn",
           "select_topk", "sparse_decode", "run_all", "window_indices", "extend_indices", "append_kv", "mixed_step"]
