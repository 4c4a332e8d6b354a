"""Device buffers of one PillarAttn round and the calls of that round, for the
benchmark, the smoke check and the tests.  Marshalling only: it uploads a host
workload, allocates the outputs and the workspace with torch, and calls the
entry points of the C ABI through the binding.  Nothing here computes."""
from __future__ import annotations

import torch

from . import binding as pa

_TORCH = {"f32": torch.float32, "bf16": torch.bfloat16}


class GpuRun:
    """Uploads a workload once and runs stages on it."""

    def __init__(self, w, device="cuda:0", flags=0):
        self.w = w
        self.dev = torch.device(device)
        self.dw = pa.upload_workload(w, device)
        kv = self.dw.kv
        kv.flags = flags                       # PILLAR_FLAG_* of every call made through this object
        B, Hq, Hkv, D, n_q = w.B, w.Hq, w.Hkv, w.D, w.n_q
        self.max_budget = max(1, int(w.budgets.max()))
        nbytes = pa.pillar_workspace_bytes(kv, w.spec_k, self.max_budget)
        assert nbytes > 0
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
        qd = _TORCH[w.q_dtype]
        self.out = torch.full((B, n_q, Hq, D), float("nan"), dtype=qd, device=self.dev)
        self.lse = torch.full((B, n_q, Hq), float("nan"), dtype=torch.float32, device=self.dev)
        self.score_stride = (w.max_seq_len + 63) // 64 * 64
        self.scores = torch.full((B, Hkv, self.score_stride), float("nan"), dtype=torch.float32, device=self.dev)
        self.indices = torch.full((B, Hkv, self.max_budget), -7, dtype=torch.int32, device=self.dev)
        self.counts = torch.full((B,), -7, dtype=torch.int32, device=self.dev)
        self.d_out = torch.full((B, Hq, D), float("nan"), dtype=qd, device=self.dev)
        self.d_lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=self.dev)

    def verify(self, with_scores=True, with_lse=True):
        pa.pillar_verify_attn(self.dw.kv, self.dw.q, self.w.spec_k, self.out,
                              self.lse if with_lse else None, self.scores if with_scores else None,
                              self.workspace)

    def verify_select(self, with_scores=True, with_lse=True):
        pa.pillar_verify_select(self.dw.kv, self.dw.q, self.w.spec_k, self.out, self.lse if with_lse else None,
                                self.scores if with_scores else None, self.dw.budgets, self.max_budget,
                                self.indices, self.counts, self.workspace)

    def topk(self, scores=None):
        pa.pillar_select_topk(self.scores if scores is None else scores, self.dw.kv.seq_lens, self.dw.budgets,
                              self.w.max_seq_len, self.max_budget, self.indices, self.counts, self.workspace)

    def decode(self, indices=None, counts=None):
        pa.pillar_sparse_decode(self.dw.kv, self.dw.q_draft, self.indices if indices is None else indices,
                                self.counts if counts is None else counts, self.max_budget, self.d_out,
                                self.d_lse, self.workspace)

    def run_all(self, fused_select=False):
        if fused_select:
            self.verify_select()
        else:
            self.verify()
            self.topk()
        self.decode()
        torch.cuda.synchronize()
