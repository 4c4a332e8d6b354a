"""ctypes binding of libpillar.so: argument marshalling only.

Every function here has the name and the argument order of its C entry point
(include/pillar.h).  Tensors are torch tensors on the GPU, used as typed
device pointers; nothing is computed in Python.  If the library has not been
built, importing succeeds but every call raises: there is no fallback path.  The measurement helpers of
include/pillar_bench.h are bound here too.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpillar.so")

PILLAR_OK, PILLAR_EINVAL, PILLAR_EUNSUPPORTED, PILLAR_EWORKSPACE, PILLAR_EHIP, PILLAR_ETOOLARGE = 0, -1, -2, -3, -4, -5
PILLAR_F32, PILLAR_BF16, PILLAR_FP8_E4M3 = 0, 1, 2
PILLAR_FLAG_EXACT_SCORES, PILLAR_FLAG_GENERIC_KERNELS = 1, 2
DTYPE_CODE = {"f32": PILLAR_F32, "bf16": PILLAR_BF16, "fp8_e4m3": PILLAR_FP8_E4M3}

EXPORTS = ("pillar_version", "pillar_status_string", "pillar_workspace_bytes", "pillar_verify_attn",
           "pillar_verify_select", "pillar_verify_hetero", "pillar_mixed_step", "pillar_select_topk", "pillar_sparse_decode", "pillar_sparse_decode_static", "pillar_window_indices",
           "pillar_extend_indices", "pillar_append_kv", "pillar_profile_enable", "pillar_profile_reset",
           "pillar_profile_read", "pillar_set_option", "pillar_bench_read")


class pillar_kv_t(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("page_size", C.c_int32), ("q_dtype", C.c_int32),
        ("kv_dtype", C.c_int32), ("sm_scale", C.c_float),
        ("k_pool", C.c_void_p), ("v_pool", C.c_void_p),
        ("stride_page", C.c_int64), ("stride_head", C.c_int64), ("stride_slot", C.c_int64),
        ("k_scale", C.c_void_p), ("v_scale", C.c_void_p),
        ("num_pages", C.c_int32), ("block_table_stride", C.c_int32),
        ("block_table", C.c_void_p), ("seq_lens", C.c_void_p),
        ("max_seq_len", C.c_int32), ("flags", C.c_int32),
    ]


class pillar_kernel_time(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64), ("total_ms", C.c_double)]


class PillarError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load() -> C.CDLL:
    """Load libpillar.so (built by paper_2512_01278_amd.build).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2512_01278_amd.build` first; "
                           "there is no fallback implementation")
    lib = C.CDLL(LIB_PATH)
    lib.pillar_version.restype = C.c_int
    lib.pillar_status_string.restype = C.c_char_p
    lib.pillar_status_string.argtypes = [C.c_int]
    lib.pillar_workspace_bytes.restype = C.c_size_t
    lib.pillar_workspace_bytes.argtypes = [C.POINTER(pillar_kv_t), C.c_int32, C.c_int32]
    lib.pillar_verify_attn.restype = C.c_int
    lib.pillar_verify_attn.argtypes = [C.POINTER(pillar_kv_t), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.pillar_verify_select.restype = C.c_int
    lib.pillar_verify_select.argtypes = [C.POINTER(pillar_kv_t), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
    lib.pillar_verify_hetero.restype = C.c_int
    lib.pillar_verify_hetero.argtypes = [C.POINTER(pillar_kv_t), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
    lib.pillar_mixed_step.restype = C.c_int
    lib.pillar_mixed_step.argtypes = [C.POINTER(pillar_kv_t), C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.pillar_select_topk.restype = C.c_int
    lib.pillar_select_topk.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                       C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                       C.c_void_p]
    lib.pillar_sparse_decode.restype = C.c_int
    lib.pillar_sparse_decode.argtypes = [C.POINTER(pillar_kv_t), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.pillar_sparse_decode_static.restype = C.c_int
    lib.pillar_sparse_decode_static.argtypes = [C.POINTER(pillar_kv_t), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                                C.c_void_p, C.c_void_p, C.c_void_p]
    lib.pillar_append_kv.restype = C.c_int
    lib.pillar_append_kv.argtypes = [C.POINTER(pillar_kv_t), C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
    lib.pillar_window_indices.restype = C.c_int
    lib.pillar_window_indices.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
    lib.pillar_extend_indices.restype = C.c_int
    lib.pillar_extend_indices.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                          C.c_void_p]
    lib.pillar_bench_read.restype = C.c_int
    lib.pillar_bench_read.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.pillar_set_option.restype = C.c_int
    lib.pillar_set_option.argtypes = [C.c_char_p, C.c_int64]
    lib.pillar_profile_enable.restype = None
    lib.pillar_profile_enable.argtypes = [C.c_int]
    lib.pillar_profile_reset.restype = None
    lib.pillar_profile_read.restype = C.c_int
    lib.pillar_profile_read.argtypes = [C.POINTER(pillar_kernel_time), C.c_int]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().pillar_status_string(int(status)).decode()


def pillar_version() -> int:
    return load().pillar_version()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


@dataclass
class KvCache:
    """The torch tensors behind one pillar_kv_t (all on one GPU)."""
    k_pool: torch.Tensor           # [num_pages, Hkv, P, D]; bf16 / f32 / uint8 (fp8 codes)
    v_pool: torch.Tensor
    block_table: torch.Tensor      # int32 [B, max_pages]
    seq_lens: torch.Tensor         # int32 [B]
    num_q_heads: int
    q_dtype: str
    kv_dtype: str
    sm_scale: float
    max_seq_len: int
    k_scale: Optional[torch.Tensor] = None
    v_scale: Optional[torch.Tensor] = None
    flags: int = 0                 # OR of PILLAR_FLAG_*

    def c_struct(self) -> pillar_kv_t:
        kp = self.k_pool
        s = pillar_kv_t()
        s.batch = self.block_table.shape[0]
        s.num_q_heads = self.num_q_heads
        s.num_kv_heads = kp.shape[1]
        s.head_dim = kp.shape[3]
        s.page_size = kp.shape[2]
        s.q_dtype = DTYPE_CODE[self.q_dtype]
        s.kv_dtype = DTYPE_CODE[self.kv_dtype]
        s.sm_scale = self.sm_scale
        s.k_pool = kp.data_ptr()
        s.v_pool = self.v_pool.data_ptr()
        s.stride_page, s.stride_head, s.stride_slot = kp.stride(0), kp.stride(1), kp.stride(2)
        s.k_scale = _ptr(self.k_scale)
        s.v_scale = _ptr(self.v_scale)
        s.num_pages = kp.shape[0]
        s.block_table_stride = self.block_table.stride(0)
        s.block_table = self.block_table.data_ptr()
        s.seq_lens = self.seq_lens.data_ptr()
        s.max_seq_len = self.max_seq_len
        s.flags = self.flags
        return s


def pillar_workspace_bytes(kv: KvCache, spec_len_k: int, max_budget: int) -> int:
    s = kv.c_struct()
    return int(load().pillar_workspace_bytes(C.byref(s), spec_len_k, max_budget))


def _check(rc: int, where: str) -> None:
    if rc != PILLAR_OK:
        raise PillarError(rc, where)


def pillar_verify_attn(kv: KvCache, q: torch.Tensor, spec_len_k: int, out: torch.Tensor,
                       lse: Optional[torch.Tensor], scores: Optional[torch.Tensor],
                       workspace: torch.Tensor, stream=None) -> None:
    s = kv.c_struct()
    stride = scores.stride(1) if scores is not None else 0
    rc = load().pillar_verify_attn(C.byref(s), q.data_ptr(), spec_len_k, out.data_ptr(), _ptr(lse), _ptr(scores),
                                   stride, workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                   _stream(stream))
    _check(rc, "pillar_verify_attn")


def pillar_verify_select(kv: KvCache, q: torch.Tensor, spec_len_k: int, out: torch.Tensor,
                         lse: Optional[torch.Tensor], scores: Optional[torch.Tensor], budgets: torch.Tensor,
                         max_budget: int, indices: torch.Tensor, counts: torch.Tensor,
                         workspace: torch.Tensor, stream=None) -> None:
    s = kv.c_struct()
    stride = scores.stride(1) if scores is not None else 0
    rc = load().pillar_verify_select(C.byref(s), q.data_ptr(), spec_len_k, out.data_ptr(), _ptr(lse), _ptr(scores),
                                     stride, budgets.data_ptr(), max_budget, indices.data_ptr(), counts.data_ptr(),
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                     _stream(stream))
    _check(rc, "pillar_verify_select")


def pillar_verify_hetero(kv: KvCache, q: torch.Tensor, spec_len_max: int, spec_lens: torch.Tensor, out: torch.Tensor,
                         lse: Optional[torch.Tensor], scores: Optional[torch.Tensor], workspace: torch.Tensor,
                         budgets: Optional[torch.Tensor] = None, max_budget: int = 0,
                         indices: Optional[torch.Tensor] = None, counts: Optional[torch.Tensor] = None, stream=None) -> None:
    s = kv.c_struct()
    stride = scores.stride(1) if scores is not None else 0
    rc = load().pillar_verify_hetero(C.byref(s), q.data_ptr(), spec_len_max, spec_lens.data_ptr(), out.data_ptr(), _ptr(lse),
                                     _ptr(scores), stride, _ptr(budgets), max_budget, _ptr(indices), _ptr(counts),
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "pillar_verify_hetero")


def pillar_mixed_step(kv: KvCache, verify_ids: Optional[torch.Tensor], draft_ids: Optional[torch.Tensor], q_verify: torch.Tensor,
                      spec_len_k: int, out_verify: torch.Tensor, lse_verify: Optional[torch.Tensor], scores: Optional[torch.Tensor],
                      budgets: torch.Tensor, max_budget: int, indices: torch.Tensor, counts: torch.Tensor, q_draft: torch.Tensor,
                      out_draft: torch.Tensor, lse_draft: Optional[torch.Tensor], workspace: torch.Tensor, stream=None) -> None:
    s = kv.c_struct()
    stride = scores.stride(1) if scores is not None else 0
    nv = 0 if verify_ids is None else verify_ids.numel()
    nd = 0 if draft_ids is None else draft_ids.numel()
    rc = load().pillar_mixed_step(C.byref(s), _ptr(verify_ids), nv, _ptr(draft_ids), nd, q_verify.data_ptr(), spec_len_k,
                                  out_verify.data_ptr(), _ptr(lse_verify), _ptr(scores), stride, budgets.data_ptr(), max_budget,
                                  indices.data_ptr(), counts.data_ptr(), q_draft.data_ptr(), out_draft.data_ptr(), _ptr(lse_draft),
                                  workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "pillar_mixed_step")


def pillar_select_topk(scores: torch.Tensor, seq_lens: torch.Tensor, budgets: torch.Tensor,
                       max_seq_len: int, max_budget: int, indices: torch.Tensor, counts: torch.Tensor,
                       workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    B, Hkv = scores.shape[0], scores.shape[1]
    wsz = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().pillar_select_topk(scores.data_ptr(), scores.stride(1), seq_lens.data_ptr(), budgets.data_ptr(),
                                   B, Hkv, max_seq_len, max_budget, indices.data_ptr(), counts.data_ptr(),
                                   _ptr(workspace), wsz, _stream(stream))
    _check(rc, "pillar_select_topk")


def pillar_sparse_decode(kv: KvCache, q: torch.Tensor, indices: torch.Tensor, counts: torch.Tensor,
                         max_budget: int, out: torch.Tensor, lse: Optional[torch.Tensor],
                         workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    s = kv.c_struct()
    wsz = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().pillar_sparse_decode(C.byref(s), q.data_ptr(), indices.data_ptr(), counts.data_ptr(), max_budget,
                                     out.data_ptr(), _ptr(lse), _ptr(workspace), wsz, _stream(stream))
    _check(rc, "pillar_sparse_decode")


def pillar_sparse_decode_static(kv: KvCache, q: torch.Tensor, indices: torch.Tensor, counts: torch.Tensor,
                                max_budget: int, out: torch.Tensor, lse: Optional[torch.Tensor], stream=None) -> None:
    s = kv.c_struct()
    rc = load().pillar_sparse_decode_static(C.byref(s), q.data_ptr(), indices.data_ptr(), counts.data_ptr(), max_budget,
                                            out.data_ptr(), _ptr(lse), _stream(stream))
    _check(rc, "pillar_sparse_decode_static")


def pillar_append_kv(kv: KvCache, k_new: torch.Tensor, v_new: torch.Tensor, stream=None) -> None:
    s = kv.c_struct()
    _check(load().pillar_append_kv(C.byref(s), k_new.data_ptr(), v_new.data_ptr(), k_new.shape[1], _stream(stream)),
           "pillar_append_kv")


def pillar_window_indices(seq_lens: torch.Tensor, budgets: torch.Tensor, num_kv_heads: int, sink_tokens: int,
                          max_budget: int, indices: torch.Tensor, counts: torch.Tensor, stream=None) -> None:
    rc = load().pillar_window_indices(seq_lens.data_ptr(), budgets.data_ptr(), seq_lens.shape[0], num_kv_heads, sink_tokens,
                                      max_budget, indices.data_ptr(), counts.data_ptr(), _stream(stream))
    _check(rc, "pillar_window_indices")


def pillar_extend_indices(indices: torch.Tensor, counts: torch.Tensor, first_new: torch.Tensor, n_new: torch.Tensor,
                          stream=None) -> None:
    rc = load().pillar_extend_indices(indices.data_ptr(), counts.data_ptr(), first_new.data_ptr(), n_new.data_ptr(),
                                      indices.shape[0], indices.shape[1], indices.shape[2], _stream(stream))
    _check(rc, "pillar_extend_indices")


def pillar_bench_read(buf: torch.Tensor, n_chunks: int, chunk_bytes: int, order: Optional[torch.Tensor], blocks: int,
                      sink: torch.Tensor, stream=None) -> None:
    _check(load().pillar_bench_read(buf.data_ptr(), n_chunks, chunk_bytes, _ptr(order), blocks, sink.data_ptr(), _stream(stream)),
           "pillar_bench_read")


def pillar_set_option(name: str, value: int) -> None:
    _check(load().pillar_set_option(name.encode(), int(value)), f"pillar_set_option({name})")


def pillar_profile_enable(on: bool) -> None:
    load().pillar_profile_enable(1 if on else 0)


def pillar_profile_reset() -> None:
    load().pillar_profile_reset()


def pillar_profile_read() -> dict:
    """{kernel name: (launches, total ms)} since the last reset (synchronises)."""
    arr = (pillar_kernel_time * 64)()
    n = load().pillar_profile_read(arr, 64)
    return {arr[i].name.decode(): (int(arr[i].launches), float(arr[i].total_ms)) for i in range(min(n, 64))}


# ---- device residency of a host-side workload (typed uploads, no arithmetic) ----
_TORCH_VIEW = {"f32": torch.float32, "bf16": torch.bfloat16, "fp8_e4m3": torch.uint8}


def _upload(x, dtype: str, device) -> torch.Tensor:
    t = torch.from_numpy(x)
    if dtype == "bf16":
        t = t.view(torch.int16).to(device).view(torch.bfloat16)
    else:
        t = t.to(device)
    return t


@dataclass
class DeviceWorkload:
    kv: KvCache
    q: torch.Tensor
    q_draft: torch.Tensor
    budgets: torch.Tensor
    spec_k: int
    max_budget: int


def upload_workload(w, device="cuda:0") -> DeviceWorkload:
    """Copy the arrays of a host workload (see gen/workloads.py for the layout)
    to the GPU unchanged; bf16 bit patterns are re-viewed as torch.bfloat16."""
    kv = KvCache(
        k_pool=_upload(w.k_pool, w.kv_dtype, device), v_pool=_upload(w.v_pool, w.kv_dtype, device),
        block_table=torch.from_numpy(w.block_table).to(device), seq_lens=torch.from_numpy(w.seq_lens).to(device),
        num_q_heads=w.Hq, q_dtype=w.q_dtype, kv_dtype=w.kv_dtype, sm_scale=float(w.sm_scale),
        max_seq_len=int(w.seq_lens.max()),
        k_scale=None if w.k_scale is None else torch.from_numpy(w.k_scale).to(device),
        v_scale=None if w.v_scale is None else torch.from_numpy(w.v_scale).to(device))
    return DeviceWorkload(kv=kv, q=_upload(w.q, w.q_dtype, device), q_draft=_upload(w.q_draft, w.q_dtype, device),
                          budgets=torch.from_numpy(w.budgets).to(device), spec_k=w.spec_k,
                          max_budget=int(w.budgets.max()))
