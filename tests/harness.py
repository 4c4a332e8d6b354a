"""Shared helpers of the GPU parity tests: run the three stages through the
C ABI on a host workload and compare with the CPU oracle."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2512_01278_amd as pa
from paper_2512_01278_amd.runner import GpuRun

# Tolerances (the bf16 / fp8 ones are the stated targets of this build; the
# fp32 ones follow from fp32 accumulation over <= 32768 terms: a few 1e-6
# relative on the logits and outputs).
OUT_TOL = {  # kv dtype -> (max abs, rel L2)
    "f32": (2e-5, 2e-6),
    "bf16": (2e-2, 5e-3),
    "fp8_e4m3": (6e-2, 5e-3),
}
SCORE_REL = 1e-3
SCORE_FLOOR = 1e-20
# The default matrix-core verification keeps every row's exponential as a 16-bit value whose exponent
# reaches down to 2^-62 of the row's running maximum; a smaller probability (all of them are below 2^-62
# themselves) is dropped.  Where a test drives probabilities that low on purpose it grants this much
# absolute slack on top of the relative bound (reading R19 of the design notes); everywhere else the
# bound is the relative one alone.
SCORE_FLUSH = 2.0 ** -62
LSE_ABS = 2e-4
TIE_BAND = 1e-3


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def check_out(got: np.ndarray, want: np.ndarray, kv_dtype: str, what: str):
    assert not np.isnan(got).any(), f"{what}: NaN in GPU output"
    tol_abs, tol_l2 = OUT_TOL[kv_dtype]
    err = np.abs(got - want).max()
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
    assert err <= tol_abs, f"{what}: max abs error {err:.3e} > {tol_abs}"
    assert rel <= tol_l2, f"{what}: rel L2 error {rel:.3e} > {tol_l2}"
    return err, rel


def check_scores(got: np.ndarray, want: np.ndarray, seq_lens, requests, what: str, abs_slack: float = 0.0):
    worst = 0.0
    for b in requests:
        L = int(seq_lens[b])
        g_, w_ = got[b, :, :L], want[b, :, :L]
        assert not np.isnan(g_).any(), f"{what}: NaN score, request {b}"
        rel = np.maximum(np.abs(g_ - w_) - abs_slack, 0.0) / np.maximum(w_, SCORE_FLOOR)
        worst = max(worst, float(rel.max()))
        assert rel.max() <= SCORE_REL, f"{what}: score rel error {rel.max():.3e} at request {b}"
    return worst


def check_topk_exact(indices: np.ndarray, counts: np.ndarray, gpu_scores_f32: np.ndarray, seq_lens, budgets,
                     requests, what: str):
    """Integer work is bit-exact: the selection on the SAME fp32 scores must
    equal the oracle's stable-sort selection, ties included."""
    sub = np.asarray(requests)
    want_idx, want_cnt = oracle.select_topk(gpu_scores_f32[sub].astype(np.float64), np.asarray(seq_lens)[sub],
                                            np.asarray(budgets)[sub], max_budget=indices.shape[2])
    assert np.array_equal(counts[sub], want_cnt), f"{what}: counts differ"
    assert np.array_equal(indices[sub], want_idx), f"{what}: index lists differ from the stable-sort selection"


def check_topk_against_oracle_scores(indices, counts, oracle_scores, seq_lens, budgets, requests, what: str):
    """GPU selection (from GPU scores) vs oracle selection (from fp64 scores):
    the sets agree except for tokens whose score is within TIE_BAND relative
    of the K-th largest score, where either choice is correct."""
    swaps = 0
    for b in requests:
        L = int(seq_lens[b])
        kk = min(int(budgets[b]), L)
        assert counts[b] == kk
        for g in range(indices.shape[1]):
            got = indices[b, g, :kk]
            assert np.all(np.diff(got) > 0) and got.min() >= 0 and got.max() < L, f"{what}: list not ascending/in range"
            s = oracle_scores[b, g, :L]
            want = np.argsort(-s, kind="stable")[:kk]
            kth = s[want[-1]]
            diff = np.setxor1d(got, want)
            swaps += len(diff)
            if len(diff):
                assert np.all(np.abs(s[diff] - kth) <= TIE_BAND * kth), \
                    f"{what}: request {b} head {g}: sets differ outside the tie band"
    return swaps


def compare_with_oracle(w, run: GpuRun, requests=None, what=""):
    """Full element-wise parity of one round on `requests` (default: all)."""
    requests = list(range(w.B)) if requests is None else list(requests)
    want_out, want_lse, want_scores = oracle.verify_attn(w, requests=requests)
    out, lse, scores = to_f64(run.out), to_f64(run.lse), to_f64(run.scores)
    idx, counts = run.indices.cpu().numpy(), run.counts.cpu().numpy()
    rep = {}
    rep["out"] = check_out(out[requests], want_out[requests], w.kv_dtype, what + " verify out")
    lse_err = np.abs(lse[requests] - want_lse[requests]).max()
    assert lse_err <= LSE_ABS, f"{what}: lse error {lse_err:.3e}"
    rep["lse"] = lse_err
    rep["scores"] = check_scores(scores, want_scores, w.seq_lens, requests, what)
    check_topk_exact(idx, counts, run.scores.cpu().numpy()[:, :, :w.max_seq_len], w.seq_lens, w.budgets, requests, what)
    rep["swaps"] = check_topk_against_oracle_scores(idx, counts, want_scores, w.seq_lens, w.budgets, requests, what)
    # the draft step is compared on the index lists the GPU produced
    want_d, want_dl = oracle.sparse_decode(w, idx, counts, requests=requests)
    d_out, d_lse = to_f64(run.d_out), to_f64(run.d_lse)
    rep["draft"] = check_out(d_out[requests], want_d[requests], w.kv_dtype, what + " draft out")
    dl_err = np.abs(d_lse[requests] - want_dl[requests]).max()
    assert dl_err <= LSE_ABS, f"{what}: draft lse error {dl_err:.3e}"
    return rep
