"""CPU oracle for the PillarAttn hot path.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the HIP kernels are compared against.  It is plain
numpy in float64, written from the paper's description (Section 4.1, and the
page-size-1 view of sparse attention in Section 4.2) and shares nothing with
the GPU code: no kernels, headers, tables or helpers.  Only tests, the smoke
check and the benchmark's CPU-baseline leg may import it; the product path
never does.

What each function computes (the method's results are exactly defined
quantities, so the oracle is the definition written out):

  verify_attn    Section 4.1, "Overhead-free identification": full softmax
                 attention of the k+1 speculative query positions over the
                 whole KV-Cache of a request, causal among the new tokens,
                 plus the attention-score statistic: the softmax probabilities
                 averaged over the k+1 queries and over the query heads of
                 one GQA group.
  select_topk    Section 4.1: Top-K on those averaged scores gives the
                 critical tokens of each (request, KV head).
  sparse_decode  Sections 1 and 4.2: attention of one draft query restricted
                 to the selected rows (paged attention at page size 1).

Readings of points the paper leaves open (each is also listed in the design
notes): the statistic averages over all k+1 verification rows with a uniform
1/R weight, masked entries counting as zero, so it sums to one over a
request's tokens; the context length includes the k+1 speculative tokens;
selection is per (request, KV head) with budget min(K, L); ties go to the
lower position; indices are returned in ascending position order.

Pins (tests/test_oracle_*.py): an independent pure-Python triple loop on tiny
inputs, a hand-derived rational example, closed forms (identical keys, one
dominant key, context of only the speculative tokens), the invariants the
definitions imply, and torch's float64 scaled_dot_product_attention on the
un-paged tensors.  The paper prints no numeric example of this path, so
beyond those pins parity is unpinned by the paper itself.
"""
from __future__ import annotations

import numpy as np

__all__ = ["decode_tensor", "e4m3_table", "gather_request", "verify_attn",
           "select_topk", "sparse_decode", "run_all", "mixed_step"]


# ---------------------------------------------------------------------------
# storage formats -> float64 (exact)
# ---------------------------------------------------------------------------
def e4m3_table() -> np.ndarray:
    """All 256 values of OCP fp8 e4m3 (bias 7): normals (1+m/8)*2**(e-7),
    subnormals (m/8)*2**-6, no infinities, S.1111.111 is NaN."""
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        s = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            v = np.nan
        elif e == 0:
            v = s * (m / 8.0) * 2.0 ** -6
        else:
            v = s * (1.0 + m / 8.0) * 2.0 ** (e - 7)
        t[code] = v
    return t


_E4M3 = e4m3_table()


def decode_tensor(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored tensor -> float64.  bf16 arrives as uint16 bit patterns, fp8 as
    uint8 codes; both widen exactly."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return (np.asarray(x, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if dtype == "fp8_e4m3":
        return _E4M3[np.asarray(x, dtype=np.uint8)]
    raise ValueError(dtype)


def gather_request(w, b: int):
    """Un-page request b: K, V as float64 [L, Hkv, D].  Token t lives in page
    block_table[b, t // P], slot t % P."""
    L = int(w.seq_lens[b])
    P = w.P
    t = np.arange(L)
    pages = w.block_table[b, t // P]
    slots = t % P
    k = decode_tensor(w.k_pool[pages, :, slots, :], w.kv_dtype)      # [L, Hkv, D]
    v = decode_tensor(w.v_pool[pages, :, slots, :], w.kv_dtype)
    if w.kv_dtype == "fp8_e4m3":
        k = k * w.k_scale[pages].astype(np.float64)[:, :, None]
        v = v * w.v_scale[pages].astype(np.float64)[:, :, None]
    return k, v


# ---------------------------------------------------------------------------
def verify_attn(w, requests=None, spec_lens=None):
    """Full attention of the verification step and the score statistic.

    Returns out [B, k+1, Hq, D], lse [B, k+1, Hq] (natural log) and
    scores [B, Hkv, max L] (zero beyond a request's length), all float64.
    Query i of request b sits at position L_b-(k+1)+i and sees keys 0..that
    position.  scores[b, g, t] is the mean over the R=(k+1)*G rows of group g
    of the softmax probability the row puts on token t (zero where masked).

    spec_lens (optional, one per request, each <= k): requests speculate
    different numbers of tokens (Section 5.4 allows heterogeneous
    configurations).  Request b then has k_b+1 queries, the first k_b+1 of its
    k+1 query slots, query i at position L_b-(k_b+1)+i; its mean runs over
    (k_b+1)*G rows; out and lse of the unused slots stay zero.

    A context shorter than its queries (L_b < k_b+1; the paper's contexts
    always hold their own speculative tokens, so this is a reading for an
    input outside its range): a query at a negative position sees no token,
    its probabilities are all zero, its out row is zero, its lse is -inf, and
    it still counts in R, so such a request's scores sum to less than one.
    """
    B, n_q_max, Hq, Hkv, D = w.B, w.n_q, w.Hq, w.Hkv, w.D
    G = Hq // Hkv
    Lmax = int(w.seq_lens.max()) if B else 0
    q_all = decode_tensor(w.q, w.q_dtype)
    out = np.zeros((B, n_q_max, Hq, D))
    lse = np.zeros((B, n_q_max, Hq))
    scores = np.zeros((B, Hkv, Lmax))
    for b in (range(B) if requests is None else requests):
        L = int(w.seq_lens[b])
        n_q = n_q_max if spec_lens is None else int(spec_lens[b]) + 1
        R = n_q * G
        k, v = gather_request(w, b)
        pos = L - n_q + np.arange(n_q)                    # position of query i
        visible = np.arange(L)[None, :] <= pos[:, None]   # [n_q, L]
        for g in range(Hkv):
            kg = k[:, g, :]                               # [L, D]
            vg = v[:, g, :]
            qg = q_all[b, :n_q, g * G:(g + 1) * G, :]     # [n_q, G, D]
            s = w.sm_scale * np.einsum("ihd,td->iht", qg, kg)      # [n_q, G, L]
            s = np.where(visible[:, None, :], s, -np.inf)
            seen = visible.any(axis=-1)[:, None, None]    # False for a query whose position is negative
            m = np.where(seen, s.max(axis=-1, keepdims=True), 0.0)
            e = np.exp(s - m)
            l = e.sum(axis=-1, keepdims=True)
            p = e / np.where(seen, l, 1.0)                # rows sum to one (to zero when nothing is seen)
            out[b, :n_q, g * G:(g + 1) * G, :] = np.einsum("iht,td->ihd", p, vg)
            with np.errstate(divide="ignore"):
                lse[b, :n_q, g * G:(g + 1) * G] = (m + np.log(l))[..., 0]
            scores[b, g, :L] = p.sum(axis=(0, 1)) / R
    return out, lse, scores


def select_topk(scores, seq_lens, budgets, max_budget=None):
    """Top-K positions per (request, KV head).

    K' = min(budget_b, L_b) positions of largest score among 0..L_b-1, ties to
    the lower position, returned ascending; indices [B, Hkv, max_budget] padded
    with -1, counts [B] = K'.
    """
    scores = np.asarray(scores)
    B, Hkv = scores.shape[0], scores.shape[1]
    if max_budget is None:
        max_budget = int(np.max(budgets)) if B else 0
    idx = np.full((B, Hkv, max_budget), -1, dtype=np.int32)
    counts = np.zeros(B, dtype=np.int32)
    for b in range(B):
        L = int(seq_lens[b])
        kk = min(int(budgets[b]), L, max_budget)
        counts[b] = kk
        for g in range(Hkv):
            order = np.argsort(-scores[b, g, :L], kind="stable")
            idx[b, g, :kk] = np.sort(order[:kk])
    return idx, counts


def sparse_decode(w, indices, counts, requests=None):
    """Draft attention over the selected rows only.

    out [B, Hq, D], lse [B, Hq]: softmax over j < counts[b] of
    sm_scale * <q_draft[b, h], K[b, indices[b, g, j], g]>, no mask.
    """
    B, Hq, Hkv, D = w.B, w.Hq, w.Hkv, w.D
    G = Hq // Hkv
    qd = decode_tensor(w.q_draft, w.q_dtype)
    out = np.zeros((B, Hq, D))
    lse = np.full((B, Hq), -np.inf)
    for b in (range(B) if requests is None else requests):
        n = int(counts[b])
        if n == 0:
            continue
        k, v = gather_request(w, b)
        for g in range(Hkv):
            sel = np.asarray(indices[b, g, :n], dtype=np.int64)
            ks = k[sel, g, :]
            vs = v[sel, g, :]
            for h in range(g * G, (g + 1) * G):
                s = w.sm_scale * (ks @ qd[b, h])
                m = s.max()
                e = np.exp(s - m)
                l = e.sum()
                out[b, h] = (e / l) @ vs
                lse[b, h] = m + np.log(l)
    return out, lse


def run_all(w):
    """verify -> top-K -> one draft step, as one PillarAttn round runs them."""
    out, lse, scores = verify_attn(w)
    idx, counts = select_topk(scores, w.seq_lens, w.budgets)
    d_out, d_lse = sparse_decode(w, idx, counts)
    return dict(out=out, lse=lse, scores=scores, indices=idx, counts=counts,
                draft_out=d_out, draft_lse=d_lse)


def mixed_step(w, verify_ids, draft_ids, indices, counts):
    """One iteration of a unified batch (Section 4.2, "Unified Batch Scheduler" and "Fused Sparse and Full
    Attention"): in the same iteration some requests are in their verification phase and the others in a draft
    phase.  Every request in `verify_ids` runs the verification attention on its k+1 queries and then selects
    its critical tokens anew (its rows of `indices` / `counts` are replaced); every request in `draft_ids` runs
    one sparse draft step on the lists it already has.  Nothing else is touched: the result is, request by
    request, what verify_attn + select_topk or sparse_decode give for that request alone.

    Returns a dict: out, lse, scores (verification; zeros for other requests), indices, counts (updated copies),
    draft_out, draft_lse (zeros / -inf for other requests).
    """
    verify_ids = [int(b) for b in verify_ids]
    draft_ids = [int(b) for b in draft_ids]
    assert not set(verify_ids) & set(draft_ids), "a request is in one phase at a time"
    out, lse, scores = verify_attn(w, requests=verify_ids)
    idx = np.array(indices, dtype=np.int32, copy=True)
    cnt = np.array(counts, dtype=np.int32, copy=True)
    if verify_ids:
        sub = np.asarray(verify_ids)
        new_idx, new_cnt = select_topk(scores[sub], w.seq_lens[sub], w.budgets[sub], max_budget=idx.shape[2])
        idx[sub], cnt[sub] = new_idx, new_cnt
    # the draft requests use the lists they came with (a request is never in both sets)
    d_out, d_lse = sparse_decode(w, indices, counts, requests=draft_ids)
    return dict(out=out, lse=lse, scores=scores, indices=idx, counts=cnt, draft_out=d_out, draft_lse=d_lse)


# ---------------------------------------------------------------------------
def window_indices(seq_lens, budgets, num_kv_heads, sink_tokens, max_budget=None):
    """Static 'attention sinks + recent window' selection: the sliding-window
    draft that the paper's related work and baselines use in place of a
    dynamic pattern (Sections 1 and 3.3; the MagicDec-style baselines of
    Section 5).  Per request K' = min(budget, L, max_budget); the list holds
    the first min(sink_tokens, K') positions and the last K' minus that many,
    ascending, the same for every KV head, padded with -1; counts = K'.
    """
    seq_lens = np.asarray(seq_lens)
    B = len(seq_lens)
    if max_budget is None:
        max_budget = int(np.max(budgets)) if B else 0
    idx = np.full((B, num_kv_heads, max_budget), -1, dtype=np.int32)
    counts = np.zeros(B, dtype=np.int32)
    for b in range(B):
        L = int(seq_lens[b])
        kk = min(int(budgets[b]), L, max_budget)
        ns = min(int(sink_tokens), kk)
        positions = list(range(ns)) + list(range(L - (kk - ns), L))
        counts[b] = kk
        idx[b, :, :kk] = np.asarray(positions, dtype=np.int32)[None, :]
    return idx, counts


def extend_indices(indices, counts, first_new, n_new):
    """Tokens generated after the last verification have no score yet; a draft
    step must still see them (a reading: the paper is silent).  Appends the
    positions first_new[b] .. first_new[b] + n_new[b] - 1 to every head's list
    of request b, as many as still fit, and returns the new lists and counts.
    """
    idx = np.array(indices, dtype=np.int32, copy=True)
    cnt = np.array(counts, dtype=np.int32, copy=True)
    cap = idx.shape[2]
    for b in range(idx.shape[0]):
        c = int(cnt[b])
        n = max(0, min(int(n_new[b]), cap - c))
        idx[b, :, c:c + n] = (int(first_new[b]) + np.arange(n, dtype=np.int32))[None, :]
        cnt[b] = c + n
    return idx, cnt


def append_kv(w, k_pool, v_pool, k_new, v_new):
    """Writes the K/V rows of the n newest tokens of every request into paged
    pools (the verification attends to speculative tokens whose rows are already
    in the cache: append, then attend).  k_new, v_new: [B, n, Hkv, D] in the
    pool's storage type; row i of request b belongs at position L_b - n + i, i.e.
    page block_table[b, pos // P], slot pos % P.  Returns new pools.
    """
    k_out, v_out = np.array(k_pool, copy=True), np.array(v_pool, copy=True)
    n = k_new.shape[1]
    for b in range(w.B):
        L = int(w.seq_lens[b])
        for i in range(n):
            pos = L - n + i
            page, slot = int(w.block_table[b, pos // w.P]), pos % w.P
            k_out[page, :, slot, :] = k_new[b, i]
            v_out[page, :, slot, :] = v_new[b, i]
    return k_out, v_out

