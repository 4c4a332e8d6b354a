"""Seeded synthetic workloads shaped like the decode steps the paper measures.

The paper evaluates on reasoning traces of real models (Section 5.1); neither
the datasets nor the weights are available, so random tensors with the same
shapes, length mix and score structure stand in for them:

* shapes follow the Qwen3-8B attention layer the paper serves (8 KV heads of
  dimension 128, bf16; Section 4.4 footnote) at batch 128 (Section 1);
* ragged context lengths follow the spread of output lengths in Table 1;
* a few "pillar" key positions per KV head carry a larger norm, and the first
  tokens act as attention sinks, so that a small set of tokens dominates the
  attention mass (Section 3.2: about 5 % of the tokens dominate the output).

Nothing here computes attention.  The only numeric work is drawing normals
and *encoding* them into the storage formats (bf16 bit patterns, OCP fp8
e4m3 bytes with one fp32 scale per page and KV head).

Layout of every tensor (C order):
  q        [B, k+1, Hq, D]     query rows of the k+1 speculative positions
  q_draft  [B, Hq, D]          query row of one draft step
  k_pool   [num_pages, Hkv, P, D]
  v_pool   [num_pages, Hkv, P, D]
  k_scale  [num_pages, Hkv]    fp32, fp8 pools only
  block_table [B, max_pages]   int32 page ids, -1 beyond a request's pages
  seq_lens [B]                 int32, counts the k+1 speculative tokens too
  budgets  [B]                 int32 sparsity budget K of each request
bf16 tensors are numpy uint16 arrays of bit patterns, fp8 tensors uint8.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 251201278 * 10


# ----------------------------------------------------------------------------
# storage-format encoders (inputs only; decoding belongs to each consumer)
# ----------------------------------------------------------------------------
def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    r = np.where(nan, 0x7FC0, r)
    return r.astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (b.astype(np.uint32) << 16).view(np.float32)


def e4m3_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Encode float32 as OCP fp8 e4m3 (bias 7, max 448, no inf), round to
    nearest even, saturating.  NaN maps to 0x7F."""
    x = np.asarray(x, dtype=np.float32)
    sign = (np.signbit(x)).astype(np.uint8) << 7
    a = np.minimum(np.abs(x).astype(np.float64), 448.0)
    nan = np.isnan(x)
    a = np.where(nan, 0.0, a)
    _, e = np.frexp(a)                      # a = m * 2**e with m in [0.5, 1)
    e = e - 1                               # floor(log2 a) for a > 0
    e = np.maximum(e, -6)                   # subnormals share the 2**-6 binade
    step = np.ldexp(1.0, e - 3)
    qv = np.rint(a / step) * step           # rint = half to even
    qv = np.minimum(qv, 448.0)
    _, e2 = np.frexp(qv)
    e2 = e2 - 1
    normal = qv >= 2.0 ** -6
    mant_n = np.rint((qv / np.ldexp(1.0, np.where(normal, e2, 0)) - 1.0) * 8.0)
    code_n = ((np.where(normal, e2, 0) + 7).astype(np.int64) << 3) | mant_n.astype(np.int64)
    code_s = np.rint(qv * 512.0).astype(np.int64)      # multiples of 2**-9
    code = np.where(normal, code_n, code_s).astype(np.uint8)
    code = np.where(nan, np.uint8(0x7F), code | sign)
    return code.astype(np.uint8)


# ----------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    P: int
    spec_k: int
    q_dtype: str                 # "f32" | "bf16"
    kv_dtype: str                # "f32" | "bf16" | "fp8_e4m3"
    sm_scale: float
    num_pages: int
    seq_lens: np.ndarray
    budgets: np.ndarray
    block_table: np.ndarray
    q: np.ndarray
    q_draft: np.ndarray
    k_pool: np.ndarray
    v_pool: np.ndarray
    k_scale: Optional[np.ndarray] = None
    v_scale: Optional[np.ndarray] = None
    seed: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def n_q(self) -> int:
        return self.spec_k + 1

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def max_seq_len(self) -> int:
        return int(self.seq_lens.max()) if self.B else 0

    @property
    def max_budget(self) -> int:
        return int(self.budgets.max()) if self.B else 0

    def kv_elem_bytes(self) -> int:
        return {"f32": 4, "bf16": 2, "fp8_e4m3": 1}[self.kv_dtype]

    def q_elem_bytes(self) -> int:
        return {"f32": 4, "bf16": 2}[self.q_dtype]

    # Bytes the method itself has to move (what the roofline fraction is
    # quoted on): every KV row once plus one fp32 score per (token, KV head)
    # for verification; the selected rows plus their indices for a draft step.
    def verify_bytes(self) -> int:
        tok = int(self.seq_lens.astype(np.int64).sum())
        kv = tok * self.Hkv * 2 * self.D * self.kv_elem_bytes()
        sc = tok * self.Hkv * 4
        qo = 2 * self.B * self.n_q * self.Hq * self.D * self.q_elem_bytes()
        scale = 0
        if self.kv_dtype == "fp8_e4m3":
            pages = int(np.sum((self.seq_lens.astype(np.int64) + self.P - 1) // self.P))
            scale = pages * self.Hkv * 8
        return kv + sc + qo + scale

    def selected_rows(self) -> int:
        return int(np.minimum(self.budgets, self.seq_lens).astype(np.int64).sum())

    def draft_bytes(self) -> int:
        rows = self.selected_rows() * self.Hkv
        kv = rows * (2 * self.D * self.kv_elem_bytes() + 4)
        qo = 2 * self.B * self.Hq * self.D * self.q_elem_bytes()
        return kv + qo

    def topk_bytes(self) -> int:
        tok = int(self.seq_lens.astype(np.int64).sum())
        return tok * self.Hkv * 4 + self.selected_rows() * self.Hkv * 4


def _e4m3_fast(x: np.ndarray) -> np.ndarray:
    """Same codes as e4m3_bits_from_f32 (a test checks it), through torch's
    cast when torch is importable: the numpy encoder is slow on large pools."""
    try:
        import torch
    except Exception:                                    # pragma: no cover
        return e4m3_bits_from_f32(x)
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).clamp_(-448.0, 448.0)
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def _encode(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_from_f32(x)
    raise ValueError(dtype)


_POISON = {"f32": np.float32(np.nan), "bf16": np.uint16(0x7FC0), "fp8_e4m3": np.uint8(0x7F)}
_STORE = {"f32": np.float32, "bf16": np.uint16, "fp8_e4m3": np.uint8}


def make_custom(*, name: str, seed: int, B: int, Hq: int, Hkv: int, D: int, P: int,
                spec_k: int, q_dtype: str, kv_dtype: str, seq_lens, budgets,
                pool_factor: float = 1.25, exact_pool: bool = False,
                pillar_frac: float = 0.02, pillar_gain: float = 3.0,
                pillars_per_request: int = 0, sink_tokens: int = 0,
                sink_gain: float = 4.0, poison: bool = True,
                extra_table_cols: int = 0, allow_short: bool = False) -> Workload:
    """Draw one workload.  Draw order (fixed, so a seed names the tensors):
    block table, Q, then per request K, V and pillar positions, then Q_draft.

    pillar positions: either `pillars_per_request` positions per request
    shared by all KV heads, or an independent Bernoulli(pillar_frac) choice
    per (request, KV head, position); their key rows are scaled by
    `pillar_gain`.  The first `sink_tokens` key rows of every request are
    scaled by `sink_gain` on every head.

    Unused pages, and the slots of a request's last page beyond its length,
    are filled with NaN patterns when `poison` is set: a consumer that reads
    a row it has no right to read produces NaN somewhere.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    budgets = np.asarray(budgets, dtype=np.int32)
    assert seq_lens.shape == (B,) and budgets.shape == (B,)
    # a context holds its own speculative tokens; `allow_short` lifts that for the tests of shorter ones
    assert Hq % Hkv == 0 and np.all(seq_lens >= (1 if allow_short else spec_k + 1))
    n_q = spec_k + 1
    pages_per = (seq_lens.astype(np.int64) + P - 1) // P
    need = int(pages_per.sum())
    num_pages = need if exact_pool else max(need, int(math.ceil(need * pool_factor)))
    max_pages = int(pages_per.max()) + extra_table_cols if B else 0

    perm = rng.permutation(num_pages)[:need].astype(np.int32)
    block_table = np.full((B, max_pages), -1, dtype=np.int32)
    off = 0
    for b in range(B):
        n = int(pages_per[b])
        block_table[b, :n] = perm[off:off + n]
        off += n

    q = _encode(rng.standard_normal((B, n_q, Hq, D), dtype=np.float32), q_dtype)

    store = _STORE[kv_dtype]
    shape = (num_pages, Hkv, P, D)
    if poison:
        k_pool = np.full(shape, _POISON[kv_dtype], dtype=store)
        v_pool = np.full(shape, _POISON[kv_dtype], dtype=store)
    else:
        k_pool = np.zeros(shape, dtype=store)
        v_pool = np.zeros(shape, dtype=store)
    k_scale = v_scale = None
    if kv_dtype == "fp8_e4m3":
        fill = np.float32(np.nan) if poison else np.float32(1.0)
        k_scale = np.full((num_pages, Hkv), fill, dtype=np.float32)
        v_scale = np.full((num_pages, Hkv), fill, dtype=np.float32)

    for b in range(B):
        L = int(seq_lens[b])
        n = int(pages_per[b])
        pages = block_table[b, :n]
        kb = rng.standard_normal((n, Hkv, P, D), dtype=np.float32)
        vb = rng.standard_normal((n, Hkv, P, D), dtype=np.float32)
        gain = np.ones((n * P, Hkv), dtype=np.float32)
        if pillars_per_request > 0:
            pos = rng.choice(L, size=min(pillars_per_request, L), replace=False)
            gain[pos, :] *= pillar_gain
        elif pillar_frac > 0:
            gain[rng.random((n * P, Hkv)) < pillar_frac] *= pillar_gain
        if sink_tokens > 0:
            gain[:min(sink_tokens, L), :] *= sink_gain
        # [n*P, Hkv] -> [n, Hkv, P, 1]
        kb *= gain.reshape(n, P, Hkv).transpose(0, 2, 1)[..., None]
        tail = n * P - L
        if kv_dtype == "fp8_e4m3":
            if tail:
                kb[-1, :, P - tail:, :] = 0.0
                vb[-1, :, P - tail:, :] = 0.0
            for src, pool, scale in ((kb, k_pool, k_scale), (vb, v_pool, v_scale)):
                amax = np.abs(src).max(axis=(2, 3))
                sc = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
                enc = _e4m3_fast(src / sc[:, :, None, None])
                if tail and poison:
                    enc[-1, :, P - tail:, :] = _POISON[kv_dtype]
                pool[pages] = enc
                scale[pages] = sc
        else:
            ek = _encode(kb, kv_dtype)
            ev = _encode(vb, kv_dtype)
            if tail and poison:
                ek[-1, :, P - tail:, :] = _POISON[kv_dtype]
                ev[-1, :, P - tail:, :] = _POISON[kv_dtype]
            k_pool[pages] = ek
            v_pool[pages] = ev

    q_draft = _encode(rng.standard_normal((B, Hq, D), dtype=np.float32), q_dtype)

    return Workload(name=name, B=B, Hq=Hq, Hkv=Hkv, D=D, P=P, spec_k=spec_k,
                    q_dtype=q_dtype, kv_dtype=kv_dtype, sm_scale=1.0 / math.sqrt(D),
                    num_pages=num_pages, seq_lens=seq_lens, budgets=budgets,
                    block_table=block_table, q=q, q_draft=q_draft,
                    k_pool=k_pool, v_pool=v_pool, k_scale=k_scale, v_scale=v_scale,
                    seed=seed)


# ----------------------------------------------------------------------------
# The five measured configurations.
# ----------------------------------------------------------------------------
CONFIGS = {
    1: "tiny: B=2, 4/1 heads, D=64, fp32, L={300,512}, P=16, k=3, K=64",
    2: "qwen3-8b layer: B=32, 32/8 heads, D=128, bf16, L=4096, P=16, k=4, K=256",
    3: "paper-shaped decode step: B=128, 32/8 heads, D=128, bf16, L~U[1024,8192], P=16, k=4, K=5% (multiple of 64)",
    4: "long reasoning: B=16, 32/8 heads, D=128, bf16, L~U[24576,32768], P=64, k=8, K=2048",
    5: "larger model, fp8 KV: B=64, 64/8 heads, D=128, q bf16, kv fp8 e4m3, L~lognormal(median 8192) in [512,32768], P=16, k=4, K=512",
}


def make_workload(cfg: int, *, batch: Optional[int] = None, poison: bool = True) -> Workload:
    """Build configuration `cfg` (1..5).  `batch` truncates the request count
    (the per-request draws of the lengths stay those of the full batch), used
    to time the oracle on a bounded sample."""
    seed = BASE_SEED + cfg
    lrng = np.random.Generator(np.random.PCG64(seed ^ 0x5EED))
    if cfg == 1:
        B = 2
        lens = np.array([300, 512], dtype=np.int32)
        kw = dict(Hq=4, Hkv=1, D=64, P=16, spec_k=3, q_dtype="f32", kv_dtype="f32",
                  budgets=np.full(B, 64), exact_pool=True, pillar_frac=0.0,
                  pillars_per_request=8, pillar_gain=4.0)
    elif cfg == 2:
        B = 32
        lens = np.full(B, 4096, dtype=np.int32)
        kw = dict(Hq=32, Hkv=8, D=128, P=16, spec_k=4, q_dtype="bf16", kv_dtype="bf16",
                  budgets=np.full(B, 256), pool_factor=2.0)
    elif cfg == 3:
        B = 128
        lens = lrng.integers(1024, 8193, size=B).astype(np.int32)
        bud = (64 * np.ceil(0.05 * lens / 64.0)).astype(np.int32)
        kw = dict(Hq=32, Hkv=8, D=128, P=16, spec_k=4, q_dtype="bf16", kv_dtype="bf16",
                  budgets=bud, sink_tokens=4)
    elif cfg == 4:
        B = 16
        lens = lrng.integers(24576, 32769, size=B).astype(np.int32)
        kw = dict(Hq=32, Hkv=8, D=128, P=64, spec_k=8, q_dtype="bf16", kv_dtype="bf16",
                  budgets=np.full(B, 2048), sink_tokens=4, pillar_frac=0.01)
    elif cfg == 5:
        B = 64
        z = lrng.standard_normal(B)
        lens = np.clip(np.rint(np.exp(math.log(8192.0) + 0.6 * z)), 512, 32768).astype(np.int32)
        kw = dict(Hq=64, Hkv=8, D=128, P=16, spec_k=4, q_dtype="bf16", kv_dtype="fp8_e4m3",
                  budgets=np.full(B, 512))
    else:
        raise ValueError(f"config {cfg} not in 1..5")
    if batch is not None and batch < B:
        B = batch
        lens = lens[:B]
        kw["budgets"] = np.asarray(kw["budgets"])[:B]
    w = make_custom(name=f"config{cfg}", seed=seed, B=B, seq_lens=lens, poison=poison, **kw)
    w.meta["config"] = cfg
    w.meta["description"] = CONFIGS[cfg]
    return w
