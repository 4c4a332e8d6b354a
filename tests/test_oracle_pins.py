"""Pins for the CPU oracle: it is checked against things other than itself.

Each test names what fixes the expected value: a hand-derived example, an
independent pure-Python writing of the same definitions, a closed form, an
invariant, or a library routine on the un-paged tensors.
"""
import copy
import json
import math
import os

import numpy as np
import pytest

import gen
import oracle
from tests import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny(seed, **kw):
    d = dict(name="tiny", seed=seed, B=2, Hq=4, Hkv=2, D=8, P=4, spec_k=1,
             q_dtype="f32", kv_dtype="f32", seq_lens=[9, 14], budgets=[3, 5])
    d.update(kw)
    return gen.make_custom(**d)


# ---------------------------------------------------------------- golden ----
def hand_workload():
    with open(os.path.join(GOLDEN, "hand_rational.json")) as f:
        g = json.load(f)
    sh = g["shape"]
    w = gen.make_custom(name="hand", seed=1, B=1, Hq=2, Hkv=1, D=2, P=2, spec_k=1,
                        q_dtype="f32", kv_dtype="f32", seq_lens=[3], budgets=[2],
                        exact_pool=True, pillar_frac=0.0)
    w.sm_scale = sh["sm_scale"]
    w.block_table[:] = np.array(g["block_table"], dtype=np.int32)
    eye = np.eye(2, dtype=np.float32)
    w.q[0, :, :, :] = eye[None]
    w.q_draft[0] = eye
    for t in range(3):
        page, slot = g["block_table"][0][t // 2], t % 2
        w.k_pool[page, 0, slot] = np.log(np.array(g["k_logs"][t], dtype=np.float64)).astype(np.float32)
        w.v_pool[page, 0, slot] = np.array(g["v"][t], dtype=np.float32)
    return w, g["expect"]


def test_hand_rational_example():
    w, e = hand_workload()
    r = oracle.run_all(w)
    np.testing.assert_allclose(r["out"][0], np.array(e["out"]), rtol=0, atol=2e-7)
    np.testing.assert_allclose(np.exp(r["lse"][0]), np.array(e["lse_exp"]), rtol=3e-7)
    np.testing.assert_allclose(r["scores"][0, 0] * 16, np.array(e["scores_times_16"]), rtol=3e-7)
    assert r["indices"][0, 0].tolist() == e["indices"] and r["counts"].tolist() == [e["budget"]]
    np.testing.assert_allclose(r["draft_out"][0], np.array(e["draft_out"]), atol=2e-7)
    np.testing.assert_allclose(np.exp(r["draft_lse"][0]), np.array(e["draft_lse_exp"]), rtol=3e-7)


# ----------------------------------------------------------- brute force ----
@pytest.mark.parametrize("seed,kw", [
    (11, dict()),
    (12, dict(P=1, spec_k=0, Hq=2, Hkv=2, seq_lens=[1, 7], budgets=[1, 7])),
    (13, dict(P=16, spec_k=3, Hq=4, Hkv=1, D=16, seq_lens=[40, 4], budgets=[6, 9])),
    (14, dict(q_dtype="bf16", kv_dtype="bf16", B=3, seq_lens=[5, 17, 33], budgets=[2, 4, 40])),
    (15, dict(q_dtype="bf16", kv_dtype="fp8_e4m3", Hq=8, Hkv=1, spec_k=2, seq_lens=[12, 21], budgets=[4, 4])),
])
def test_matches_pure_python_loops(seed, kw):
    w = tiny(seed, **kw)
    r = oracle.run_all(w)
    bo, bl, bs = brute.verify(w)
    np.testing.assert_allclose(r["out"], np.array(bo), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(r["lse"], np.array(bl), rtol=1e-11, atol=1e-12)
    for b in range(w.B):
        L = int(w.seq_lens[b])
        for g in range(w.Hkv):
            np.testing.assert_allclose(r["scores"][b, g, :L], np.array(bs[b][g]), rtol=1e-11, atol=1e-15)
            assert np.all(r["scores"][b, g, L:] == 0)
            kk = int(r["counts"][b])
            assert kk == min(int(w.budgets[b]), L)
            assert r["indices"][b, g, :kk].tolist() == brute.topk(bs[b][g], kk)
            assert np.all(r["indices"][b, g, kk:] == -1)
    so, sl = brute.sparse(w, r["indices"], r["counts"])
    np.testing.assert_allclose(r["draft_out"], np.array(so), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(r["draft_lse"], np.array(sl), rtol=1e-11, atol=1e-12)


def test_context_shorter_than_its_queries():
    """A request with fewer tokens than query rows (outside the paper's range: a reading).  Queries at
    negative positions see nothing: zero output, lse -inf, no share of the statistic.  Pinned by the
    pure-Python loops and by a closed form: with L = 1 only the last query sees token 0, with
    probability one, so out = V[0], lse = its one logit and score[0] = G / R = 1 / (k+1)."""
    w = tiny(16, B=2, spec_k=3, Hq=4, Hkv=2, D=8, seq_lens=[2, 1], budgets=[2, 1], allow_short=True)
    out, lse, scores = oracle.verify_attn(w)
    bo, bl, bs = brute.verify(w)
    np.testing.assert_allclose(out, np.array(bo), rtol=1e-11, atol=1e-12)
    np.testing.assert_array_equal(np.isneginf(lse), np.isneginf(np.array(bl)))
    fin = np.isfinite(lse)
    np.testing.assert_allclose(lse[fin], np.array(bl)[fin], rtol=1e-11, atol=1e-12)
    for b in range(w.B):
        L = int(w.seq_lens[b])
        for g in range(w.Hkv):
            np.testing.assert_allclose(scores[b, g, :L], np.array(bs[b][g]), rtol=1e-11, atol=1e-15)
    # closed form, request 1 (L = 1, four query slots)
    assert np.all(out[1, :3] == 0) and np.all(np.isneginf(lse[1, :3]))
    k0, v0 = oracle.gather_request(w, 1)
    for h in range(w.Hq):
        g = h // w.G
        np.testing.assert_allclose(out[1, 3, h], v0[0, g], rtol=1e-12)
        q = oracle.decode_tensor(w.q, w.q_dtype)[1, 3, h]
        assert abs(lse[1, 3, h] - w.sm_scale * float(q @ k0[0, g])) < 1e-12
    np.testing.assert_allclose(scores[1, :, 0], 1.0 / w.n_q, rtol=1e-12)
    # request 0 (L = 2): rows 2 and 3 are live, the sum of its scores is 2/4
    np.testing.assert_allclose(scores[0, :, :2].sum(-1), 0.5, rtol=1e-12)


def test_config1_matches_pure_python_loops_on_one_head_row():
    # config 1 itself, sampled: one (request, query, head) row by hand
    w = gen.make_workload(1)
    out, lse, scores = oracle.verify_attn(w)
    b, i, h = 1, 2, 3
    L = int(w.seq_lens[b]); last = L - w.n_q + i
    K = [brute.kv_row(w, "k", b, t, 0) for t in range(last + 1)]
    V = [brute.kv_row(w, "v", b, t, 0) for t in range(last + 1)]
    q = [float(x) for x in w.q[b, i, h]]
    s = [w.sm_scale * sum(a * c for a, c in zip(q, row)) for row in K]
    mx = max(s); den = sum(math.exp(x - mx) for x in s)
    o = [sum(math.exp(s[t] - mx) / den * V[t][d] for t in range(last + 1)) for d in range(w.D)]
    np.testing.assert_allclose(out[b, i, h], o, rtol=1e-11, atol=1e-13)
    assert abs(lse[b, i, h] - (mx + math.log(den))) < 1e-12


# ------------------------------------------------------------ invariants ----
@pytest.mark.parametrize("cfg_kw", [dict(), dict(q_dtype="bf16", kv_dtype="bf16"),
                                    dict(q_dtype="bf16", kv_dtype="fp8_e4m3")])
def test_scores_are_a_distribution(cfg_kw):
    w = tiny(21, B=3, seq_lens=[6, 31, 64], budgets=[2, 2, 2], spec_k=3, **cfg_kw)
    out, lse, scores = oracle.verify_attn(w)
    assert np.all(scores >= 0)
    np.testing.assert_allclose(scores.sum(-1), 1.0, rtol=1e-13)
    for b in range(w.B):
        L = int(w.seq_lens[b])
        # every row sees tokens up to the first query's position: none is zero
        assert np.all(scores[b, :, :L - w.n_q + 1] > 0)
        # the last token is seen by the last query's rows only
        assert np.all(scores[b, :, L - 1] <= 1.0 / w.n_q + 1e-15)


def test_sparse_with_every_index_equals_full_attention():
    # Section 4.2: at page size 1 sparse and full attention are one pipeline
    w = tiny(22, spec_k=0, seq_lens=[13, 30], budgets=[13, 30])
    w.q_draft = w.q[:, 0].copy()
    out, lse, scores = oracle.verify_attn(w)
    idx, counts = oracle.select_topk(scores, w.seq_lens, w.budgets)
    assert counts.tolist() == [13, 30]
    assert idx[0, 0, :13].tolist() == list(range(13))          # K >= L keeps all
    d_out, d_lse = oracle.sparse_decode(w, idx, counts)
    np.testing.assert_allclose(d_out, out[:, 0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(d_lse, lse[:, 0], rtol=1e-12, atol=1e-14)


def test_order_of_indices_does_not_matter():
    w = tiny(23, seq_lens=[20, 25], budgets=[7, 9])
    r = oracle.run_all(w)
    rng = np.random.default_rng(0)
    idx = r["indices"].copy()
    for b in range(w.B):
        n = int(r["counts"][b])
        for g in range(w.Hkv):
            idx[b, g, :n] = rng.permutation(idx[b, g, :n])
    o2, l2 = oracle.sparse_decode(w, idx, r["counts"])
    np.testing.assert_allclose(o2, r["draft_out"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(l2, r["draft_lse"], rtol=1e-12)


def test_reshuffling_pages_changes_nothing():
    w = tiny(24, seq_lens=[11, 19], budgets=[4, 4], pool_factor=2.0)
    r1 = oracle.run_all(w)
    rng = np.random.default_rng(5)
    perm = rng.permutation(w.num_pages)                # new id of old page p
    inv = np.argsort(perm)
    w.k_pool = w.k_pool[inv].copy(); w.v_pool = w.v_pool[inv].copy()
    w.block_table = np.where(w.block_table >= 0, perm[np.maximum(w.block_table, 0)], -1).astype(np.int32)
    r2 = oracle.run_all(w)
    for key in r1:
        assert np.array_equal(r1[key], r2[key]), key


# ---------------------------------------------------------- closed forms ----
def test_identical_keys_give_uniform_attention():
    w = tiny(31, B=1, Hq=4, Hkv=1, spec_k=2, seq_lens=[10], budgets=[3])
    w.k_pool[:] = w.k_pool[w.block_table[0, 0], 0, 0][None, None, None, :]
    out, lse, scores = oracle.verify_attn(w)
    k, v = oracle.gather_request(w, 0)
    n_q, L = 3, 10
    for i in range(n_q):
        last = L - n_q + i
        mean_v = v[:last + 1, 0].mean(axis=0)
        for h in range(4):
            np.testing.assert_allclose(out[0, i, h], mean_v, rtol=1e-12, atol=1e-14)
    want = np.zeros(L)
    for i in range(n_q):
        last = L - n_q + i
        want[:last + 1] += 1.0 / (last + 1)
    np.testing.assert_allclose(scores[0, 0], want / n_q, rtol=1e-12)


def test_one_dominant_key_returns_its_value_row():
    w = tiny(32, B=1, Hq=2, Hkv=1, D=8, spec_k=1, seq_lens=[12], budgets=[1])
    w.q[0, :, :, :] = w.q[0, 0, 0]                     # all rows share one query
    qv = w.q[0, 0, 0].astype(np.float64)
    t_star = 5
    page, slot = w.block_table[0, t_star // w.P], t_star % w.P
    w.k_pool[page, 0, slot] = (200.0 * qv / np.linalg.norm(qv)).astype(np.float32)
    out, lse, scores = oracle.verify_attn(w)
    k, v = oracle.gather_request(w, 0)
    np.testing.assert_allclose(out[0], np.broadcast_to(v[t_star, 0], out[0].shape), atol=1e-9)
    assert abs(scores[0, 0, t_star] - 1.0) < 1e-9
    idx, counts = oracle.select_topk(scores, w.seq_lens, w.budgets)
    assert idx[0, 0, 0] == t_star


def test_context_of_only_the_speculative_tokens_is_a_causal_triangle():
    w = tiny(33, B=1, Hq=1, Hkv=1, spec_k=3, seq_lens=[4], budgets=[4])
    out, lse, scores = oracle.verify_attn(w)
    k, v = oracle.gather_request(w, 0)
    np.testing.assert_allclose(out[0, 0, 0], v[0, 0], rtol=1e-13)   # first row sees one key
    assert abs(lse[0, 0, 0] - w.sm_scale * float(k[0, 0] @ oracle.decode_tensor(w.q, "f32")[0, 0, 0])) < 1e-12
    assert scores[0, 0, 3] <= 0.25 and scores[0, 0, 0] >= 0.25 * (1 + 0)   # token 0 gets all of row 0


# -------------------------------------------------------- library routine ----
def test_torch_sdpa_float64_on_unpaged_tensors():
    torch = pytest.importorskip("torch")
    w = tiny(41, B=2, Hq=4, Hkv=2, D=16, spec_k=2, q_dtype="bf16", kv_dtype="bf16",
             seq_lens=[23, 37], budgets=[5, 6])
    r = oracle.run_all(w)
    G = w.G
    qf = gen.f32_from_bf16_bits(w.q).astype(np.float64)
    qd = gen.f32_from_bf16_bits(w.q_draft).astype(np.float64)
    for b in range(w.B):
        L = int(w.seq_lens[b])
        t = np.arange(L)
        pages, slots = w.block_table[b, t // w.P], t % w.P
        k = gen.f32_from_bf16_bits(w.k_pool[pages, :, slots]).astype(np.float64)    # [L, Hkv, D]
        v = gen.f32_from_bf16_bits(w.v_pool[pages, :, slots]).astype(np.float64)
        kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(G, dim=0)       # [Hq, L, D]
        vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(G, dim=0)
        qt = torch.from_numpy(qf[b]).permute(1, 0, 2)                               # [Hq, n_q, D]
        pos = L - w.n_q + torch.arange(w.n_q)
        mask = torch.arange(L)[None, :] <= pos[:, None]
        o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask, scale=w.sm_scale)
        np.testing.assert_allclose(r["out"][b], o.permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)
        n = int(r["counts"][b])
        for g in range(w.Hkv):
            sel = torch.from_numpy(r["indices"][b, g, :n].astype(np.int64))
            qh = torch.from_numpy(qd[b, g * G:(g + 1) * G])[:, None, :]            # [G, 1, D]
            ks = torch.from_numpy(k[:, g])[sel][None].expand(G, -1, -1)
            vs = torch.from_numpy(v[:, g])[sel][None].expand(G, -1, -1)
            o = torch.nn.functional.scaled_dot_product_attention(qh, ks, vs, scale=w.sm_scale)
            np.testing.assert_allclose(r["draft_out"][b, g * G:(g + 1) * G], o[:, 0].numpy(), rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ top-K ----
def test_topk_with_exact_ties_takes_lower_positions():
    scores = np.zeros((1, 2, 12))
    scores[0, 0] = [.1, .3, .3, .05, .3, .3, .0, .2, .2, .2, .01, .3]
    scores[0, 1] = 0.5                                   # all equal
    idx, counts = oracle.select_topk(scores, np.array([12]), np.array([4]))
    assert idx[0, 0].tolist() == [1, 2, 4, 5]            # five 0.3s: the lowest four
    assert idx[0, 1].tolist() == [0, 1, 2, 3]
    idx, counts = oracle.select_topk(scores, np.array([10]), np.array([7]), max_budget=9)
    assert idx[0, 0].tolist() == [1, 2, 4, 5, 7, 8, 9, -1, -1] and counts.tolist() == [7]
    assert brute.topk(list(scores[0, 0, :10]), 7) == [1, 2, 4, 5, 7, 8, 9]


def test_topk_is_a_threshold_set():
    rng = np.random.default_rng(3)
    s = rng.random((3, 2, 200)) ** 8
    lens = np.array([200, 150, 17]); bud = np.array([20, 200, 5])
    idx, counts = oracle.select_topk(s, lens, bud)
    assert counts.tolist() == [20, 150, 5]
    for b in range(3):
        for g in range(2):
            sel = idx[b, g, :counts[b]]
            assert np.all(np.diff(sel) > 0) and sel.max() < lens[b]
            rest = np.setdiff1d(np.arange(lens[b]), sel)
            if len(rest):
                assert s[b, g, sel].min() >= s[b, g, rest].max()


# -------------------------------------------------------------------- fp8 ----
def test_e4m3_table_against_format_and_library():
    torch = pytest.importorskip("torch")
    t = oracle.e4m3_table()
    assert t[0x7E] == 448.0 and t[0x01] == 2.0 ** -9 and t[0x08] == 2.0 ** -6 and t[0x38] == 1.0
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and t[0x80] == 0 and np.signbit(t[0x80])
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(t, lib, equal_nan=True)
    finite = ~np.isnan(t)
    # the generator's encoder inverts the table on every finite code ...
    codes = np.arange(256, dtype=np.uint8)[finite]
    back = gen.e4m3_bits_from_f32(t[finite].astype(np.float32))
    assert np.array_equal(back & 0x7F, codes & 0x7F) and np.array_equal(back[t[finite] != 0], codes[t[finite] != 0])
    # ... and agrees with the library's rounding on random values
    x = np.random.default_rng(0).standard_normal(20000).astype(np.float32) * 100
    x = np.concatenate([x, np.array([0.0, 448.0, 1e9, -1e9, 2.0 ** -10, 3 * 2.0 ** -10, 0.0009765625 * 1.5], dtype=np.float32)])
    want = torch.from_numpy(np.clip(x, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(gen.e4m3_bits_from_f32(x), want)


def test_bf16_roundtrip_against_library():
    torch = pytest.importorskip("torch")
    x = np.random.default_rng(1).standard_normal(10000).astype(np.float32)
    bits = gen.bf16_bits_from_f32(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    assert np.array_equal(oracle.decode_tensor(bits, "bf16"), torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy())


# ---------------------------------------------------------------- index lists
def test_window_list_is_topk_of_a_sink_plus_recency_score():
    """'Sinks + recent window' is the Top-K of a score that puts the sinks first and then grows with
    the position: checked against the (separately pinned) Top-K routine, and against hand-written lists."""
    seq_lens = np.array([5, 40, 17, 3], dtype=np.int32)
    budgets = np.array([8, 12, 17, 2], dtype=np.int32)
    sink = 4
    idx, cnt = oracle.window_indices(seq_lens, budgets, 3, sink, max_budget=16)
    scores = np.zeros((4, 3, 40))
    for b, L in enumerate(seq_lens):
        scores[b, :, :L] = (np.arange(L) + 1.0) / (L + 1.0)
        scores[b, :, :min(sink, L)] = 2.0 + np.arange(min(sink, L))[::-1]     # sink 0 highest
    ref_idx, ref_cnt = oracle.select_topk(scores, seq_lens, budgets, max_budget=16)
    assert np.array_equal(cnt, ref_cnt) and np.array_equal(idx, ref_idx)
    assert cnt.tolist() == [5, 12, 16, 2]
    assert idx[1, 0, :12].tolist() == [0, 1, 2, 3, 32, 33, 34, 35, 36, 37, 38, 39]
    assert idx[3, 2, :2].tolist() == [0, 1] and idx[3, 2, 2] == -1          # budget below the sink count: sinks only
    assert idx[0, 1, :5].tolist() == [0, 1, 2, 3, 4]                        # budget above the length: everything


def test_extend_indices_by_hand():
    idx = np.full((2, 2, 6), -1, dtype=np.int32)
    idx[0, :, :3] = [1, 4, 7]
    idx[1, :, :5] = [0, 1, 2, 3, 9]
    cnt = np.array([3, 5], dtype=np.int32)
    new_idx, new_cnt = oracle.extend_indices(idx, cnt, first_new=[10, 20], n_new=[2, 3])
    assert new_cnt.tolist() == [5, 6]                                        # the second list has room for one only
    assert new_idx[0, 1].tolist() == [1, 4, 7, 10, 11, -1]
    assert new_idx[1, 0].tolist() == [0, 1, 2, 3, 9, 20]
    assert idx[0, 0, 3] == -1                                                # inputs untouched


def test_append_kv_restores_rows_read_back_through_the_block_table():
    """Cut the newest rows out of a generated pool (poison them), append them again: the pool is back
    bit for bit, and what gather_request (a different code path) reads is what was appended."""
    w = gen.make_custom(name="append", seed=77, B=3, Hq=4, Hkv=2, D=8, P=4, spec_k=2, q_dtype="f32", kv_dtype="f32",
                        seq_lens=[3, 9, 14], budgets=[2, 2, 2])
    n = 3
    k_new = np.zeros((w.B, n, w.Hkv, w.D), dtype=w.k_pool.dtype)
    v_new = np.zeros_like(k_new)
    k_cut, v_cut = w.k_pool.copy(), w.v_pool.copy()
    for b in range(w.B):
        k, v = oracle.gather_request(w, b)                  # [L, Hkv, D] float64, exact for f32 storage
        L = int(w.seq_lens[b])
        k_new[b], v_new[b] = k[L - n:], v[L - n:]
        for pos in range(L - n, L):
            page, slot = int(w.block_table[b, pos // w.P]), pos % w.P
            k_cut[page, :, slot, :] = np.nan
            v_cut[page, :, slot, :] = np.nan
    k_back, v_back = oracle.append_kv(w, k_cut, v_cut, k_new, v_new)
    assert np.array_equal(k_back.view(np.uint32), w.k_pool.view(np.uint32))
    assert np.array_equal(v_back.view(np.uint32), w.v_pool.view(np.uint32))
    assert np.isnan(k_cut).sum() > np.isnan(w.k_pool).sum()    # the cut really removed something


def test_per_request_speculative_lengths_reduce_to_uniform_runs():
    """A request that speculates k_b tokens inside a batch laid out for k must get exactly what a batch
    laid out for k_b gives it (same K/V, same first k_b+1 queries, shifted positions), and k_b = 0 is the
    sparse decode over every token."""
    w = gen.make_custom(name="hetero", seed=31, B=3, Hq=4, Hkv=2, D=8, P=4, spec_k=3, q_dtype="f32", kv_dtype="f32",
                        seq_lens=[9, 14, 6], budgets=[2, 2, 2])
    spec = np.array([1, 3, 0])
    out, lse, scores = oracle.verify_attn(w, spec_lens=spec)
    assert np.allclose(scores.sum(-1), 1.0, atol=1e-12)
    for b in range(w.B):
        kb = int(spec[b])
        sub = copy.copy(w)                               # same pools and tables, queries re-laid for k_b
        sub.spec_k = kb
        sub.q = w.q[:, :kb + 1].copy()
        o2, l2, s2 = oracle.verify_attn(sub, requests=[b])
        assert np.array_equal(o2[b], out[b, :kb + 1]) and np.array_equal(l2[b], lse[b, :kb + 1])
        assert np.array_equal(s2[b], scores[b])
        assert not out[b, kb + 1:].any() and not lse[b, kb + 1:].any()
    # k_b = 0: one query at the last position sees everything = sparse decode over all tokens
    b = 2
    L = int(w.seq_lens[b])
    idx = np.full((w.B, w.Hkv, L), -1, dtype=np.int32)
    idx[b] = np.arange(L)
    cnt = np.zeros(w.B, dtype=np.int32)
    cnt[b] = L
    wd = copy.copy(w)
    wd.q_draft = w.q[:, 0].copy()
    d_out, d_lse = oracle.sparse_decode(wd, idx, cnt, requests=[b])
    assert np.allclose(d_out[b], out[b, 0], atol=1e-12) and np.allclose(d_lse[b], lse[b, 0], atol=1e-12)



# ---------------------------------------------------- mixed draft / verify batch ----
def test_mixed_step_reduces_to_the_two_pure_batches():
    """A unified batch is, request by request, one of the two pure batches: everything verifying equals
    verify_attn + select_topk, everything drafting equals sparse_decode, and a mixed batch equals, for each
    request, the pure result of its phase computed for that request alone (both pure functions are pinned
    above); requests of the other phase keep their lists and get no output."""
    w = tiny(41, B=5, spec_k=2, Hq=4, Hkv=2, D=16, seq_lens=[9, 40, 17, 33, 5], budgets=[3, 8, 4, 6, 2],
             q_dtype="bf16", kv_dtype="bf16")
    rng = np.random.default_rng(3)
    old_idx = np.full((w.B, w.Hkv, 8), -1, dtype=np.int32)
    old_cnt = np.array([2, 5, 0, 6, 1], dtype=np.int32)
    for b in range(w.B):
        for g in range(w.Hkv):
            old_idx[b, g, :old_cnt[b]] = np.sort(rng.choice(int(w.seq_lens[b]), size=old_cnt[b], replace=False))
    full = oracle.run_all(w)
    allv = oracle.mixed_step(w, range(w.B), [], old_idx, old_cnt)
    np.testing.assert_array_equal(allv["out"], full["out"])
    np.testing.assert_array_equal(allv["scores"], full["scores"])
    np.testing.assert_array_equal(allv["indices"][:, :, :full["indices"].shape[2]], full["indices"])
    np.testing.assert_array_equal(allv["counts"], full["counts"])
    want_d, want_dl = oracle.sparse_decode(w, old_idx, old_cnt)
    alld = oracle.mixed_step(w, [], range(w.B), old_idx, old_cnt)
    np.testing.assert_array_equal(alld["draft_out"], want_d)
    np.testing.assert_array_equal(alld["indices"], old_idx)
    ver, dra = [3, 0], [4, 1, 2]
    mix = oracle.mixed_step(w, ver, dra, old_idx, old_cnt)
    for b in ver:
        np.testing.assert_array_equal(mix["out"][b], full["out"][b])
        np.testing.assert_array_equal(mix["lse"][b], full["lse"][b])
        kk = int(full["counts"][b])
        assert mix["counts"][b] == kk and np.array_equal(mix["indices"][b, :, :kk], full["indices"][b, :, :kk])
        assert np.all(mix["draft_out"][b] == 0)
    for b in dra:
        np.testing.assert_array_equal(mix["draft_out"][b], want_d[b])
        np.testing.assert_array_equal(mix["draft_lse"][b], want_dl[b])
        assert mix["counts"][b] == old_cnt[b] and np.array_equal(mix["indices"][b], old_idx[b])
        assert np.all(mix["out"][b] == 0) and np.all(mix["scores"][b] == 0)
    with pytest.raises(AssertionError):
        oracle.mixed_step(w, [1], [1], old_idx, old_cnt)
