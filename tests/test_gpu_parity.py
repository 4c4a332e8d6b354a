"""GPU parity: every stage, through the C ABI, against the fp64 CPU oracle on
the same seeded inputs."""
import numpy as np
import pytest
import torch

import gen
import oracle
import paper_2512_01278_amd as pa
from tests.harness import (GpuRun, check_out, check_topk_exact, compare_with_oracle, to_f64, LSE_ABS)

pytestmark = pytest.mark.gpu


def small(seed, **kw):
    d = dict(name="small", seed=seed, B=3, Hq=8, Hkv=2, D=128, P=16, spec_k=2, q_dtype="bf16",
             kv_dtype="bf16", seq_lens=[3, 130, 517], budgets=[2, 40, 64])
    d.update(kw)
    return gen.make_custom(**d)


def round_trip(w, requests=None, what="", flags=0, fused_select=False):
    print(f"[case] {what or w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} D={w.D} P={w.P} k={w.spec_k} "
          f"{w.q_dtype}/{w.kv_dtype} L={w.seq_lens[:6].tolist()} seed={w.seed} flags={flags} fused={fused_select}", flush=True)
    run = GpuRun(w, flags=flags)
    run.run_all(fused_select=fused_select)
    rep = compare_with_oracle(w, run, requests, what or w.name)
    print(f"[ok] {what or w.name}: {rep}", flush=True)
    return run, rep


# ------------------------------------------------------------ config 1 ------
def test_config1_tiny_fp32():
    round_trip(gen.make_workload(1), what="config1")


# --------------------------------------------- small shapes, ragged tails ----
@pytest.mark.parametrize("seed,kw", [
    (101, dict()),
    (102, dict(q_dtype="f32", kv_dtype="f32", D=64)),
    (103, dict(kv_dtype="fp8_e4m3", Hq=16, Hkv=2, spec_k=4, seq_lens=[5, 255, 1000], budgets=[5, 16, 512])),
    (104, dict(P=64, spec_k=8, Hq=8, Hkv=2, seq_lens=[9, 64, 700], budgets=[9, 64, 100])),
    (105, dict(P=1, spec_k=0, Hq=4, Hkv=4, seq_lens=[1, 2, 129], budgets=[1, 1, 128])),
    (106, dict(D=64, Hq=16, Hkv=1, spec_k=3, seq_lens=[4, 256, 257], budgets=[300, 1, 257])),
    (107, dict(q_dtype="f32", kv_dtype="bf16", spec_k=15, Hq=4, Hkv=1, seq_lens=[16, 17, 400], budgets=[3, 3, 3])),
    (108, dict(B=1, Hq=32, Hkv=8, spec_k=4, seq_lens=[2100], budgets=[128], sink_tokens=4)),
    (109, dict(kv_dtype="fp8_e4m3", q_dtype="f32", D=64, P=4, seq_lens=[3, 4, 333], budgets=[1, 4, 33])),
    # the largest row counts of the matrix-core path: 64 rows (4 row blocks) from 16 queries x 4 heads and from
    # 4 queries x 16 heads, 48 rows (3 row blocks) with fp8 KV
    (116, dict(spec_k=15, Hq=8, Hkv=2, seq_lens=[16, 130, 1100], budgets=[16, 40, 64])),
    (117, dict(spec_k=3, Hq=16, Hkv=1, seq_lens=[4, 257, 600], budgets=[4, 64, 64])),
    (118, dict(kv_dtype="fp8_e4m3", spec_k=5, Hq=16, Hkv=2, seq_lens=[6, 255, 1000], budgets=[6, 16, 128])),
    # fp8 KV through the one-wavefront pass: 20 rows (2 row blocks) and 6 rows (1 row block)
    (119, dict(kv_dtype="fp8_e4m3", spec_k=4, Hq=8, Hkv=2, seq_lens=[33, 700, 2100], budgets=[8, 64, 128])),
    (120, dict(kv_dtype="fp8_e4m3", spec_k=2, Hq=4, Hkv=2, seq_lens=[7, 300, 1500], budgets=[7, 32, 64])),
])
def test_small_shapes(seed, kw):
    round_trip(small(seed, **kw))


def test_random_shapes_both_call_styles():
    """24 seeded random shapes of the matrix-core paths (1 to 64 query rows per KV head, bf16 and fp8 KV, pages of
    16 to 64 tokens, contexts from the queries' own tokens up to 30 K), as three calls and as the fused call."""
    rng = np.random.default_rng(20251201278)
    for it in range(24):
        G = int(rng.choice([1, 2, 4, 8, 16])); Hkv = int(rng.choice([1, 2, 4])); k = int(rng.integers(0, 9))
        if (k + 1) * G > 64:
            k = 64 // G - 1
        P = int(rng.choice([16, 32, 64])); B = int(rng.integers(1, 5))
        kvd = str(rng.choice(["bf16", "fp8_e4m3"]))
        pool = [int(rng.integers(1, 40)), int(rng.integers(40, 600)), int(rng.integers(600, 4000)),
                int(rng.integers(8000, 30000)) if it % 6 == 5 else int(rng.integers(100, 900))]
        lens = [max(k + 1, int(x)) for x in rng.choice(pool, size=B)]
        buds = [int(min(l, rng.choice([1, 7, 32, 100, 513, 700]))) for l in lens]
        w = gen.make_custom(name="random", seed=9100 + it, B=B, Hq=G * Hkv, Hkv=Hkv, D=128, P=P, spec_k=k, q_dtype="bf16",
                            kv_dtype=kvd, seq_lens=lens, budgets=buds, sink_tokens=int(rng.choice([0, 4])))
        for fused in (False, True):
            round_trip(w, what=f"random shape {it}", fused_select=fused)


# ------------------------ work division of the two verification passes ----
def test_many_tiny_requests_span_ranges():
    """300 requests of 5..70 tokens: more requests than lanes in the wave-wide search for a range's
    first request, ranges of a single tile, and (more ranges than tiles) empty ranges."""
    rng = np.random.default_rng(7)
    lens = rng.integers(5, 71, size=300).tolist()
    w = small(110, B=300, Hq=8, Hkv=2, spec_k=4, seq_lens=lens, budgets=[8] * 300)
    round_trip(w, what="300 tiny requests")


def test_batch_larger_than_one_planning_pass():
    """1100 requests: the unit prefix is built in two passes of 1024 and a range's first request is found
    through a prefix longer than one wavefront-wide search step."""
    rng = np.random.default_rng(9)
    lens = rng.integers(3, 40, size=1100).tolist()
    w = small(115, B=1100, Hq=4, Hkv=1, spec_k=2, seq_lens=lens, budgets=[4] * 1100)
    round_trip(w, what="1100 tiny requests")


@pytest.mark.parametrize("waves", [0, 1])
def test_plan_inside_the_pass_with_a_full_register_set(waves):
    """1000 requests, many of equal length: the single pass works out its own plan (lengths of all requests in
    16 registers per lane, ranks with ties by index); with one wavefront per compute unit there are fewer
    wavefronts than requests, so each ranks several."""
    rng = np.random.default_rng(19)
    lens = rng.integers(3, 12, size=1000).tolist()
    w = small(116, B=1000, Hq=4, Hkv=2, spec_k=2, seq_lens=lens, budgets=[4] * 1000)
    pa.pillar_set_option("verify_waves", waves)
    try:
        round_trip(w, what=f"1000 tiny requests, verify_waves={waves}")
    finally:
        pa.pillar_set_option("verify_waves", 0)


def test_few_wide_ranges_cross_pairs_and_page_windows():
    """One wavefront per compute unit: every range then covers several (request, head) pairs and
    more than the 64 pages a lane register holds, so segments, partial slots and page windows change
    inside a range."""
    lens = [3000, 1100, 4097, 2500]
    w = small(111, B=4, Hq=16, Hkv=4, spec_k=4, seq_lens=lens, budgets=[64] * 4)
    pa.pillar_set_option("verify_waves", 1)
    try:
        round_trip(w, what="wide ranges")
    finally:
        pa.pillar_set_option("verify_waves", 0)


def test_peaked_attention_wide_logit_range():
    """Sinks with ten times the key norm and strong pillars: row maxima jump by tens of bits between
    tiles (rescaling of the running sums), and most tokens end with probabilities around 2^-40, far
    down the exponent range of the 16-bit stash but inside it."""
    w = small(114, B=2, Hq=16, Hkv=4, spec_k=4, seq_lens=[1500, 3100], budgets=[64, 128],
              sink_tokens=4, sink_gain=10.0, pillar_gain=6.0)
    _, rep = round_trip(w, what="peaked")
    assert rep["scores"] < 1e-3


def test_two_pass_variant_with_fp32_probabilities():
    """PILLAR_FLAG_EXACT_SCORES reads K twice and never rounds a probability below fp32: same results, and
    the score statistic then agrees with the oracle to fp32 accuracy."""
    exact = pa.PILLAR_FLAG_EXACT_SCORES
    _, rep = round_trip(small(112, B=4, Hq=16, Hkv=4, spec_k=4, seq_lens=[3000, 40, 4097, 2500], budgets=[64] * 4),
                        what="two-pass", flags=exact)
    assert rep["scores"] < 5e-5
    round_trip(small(113, kv_dtype="fp8_e4m3", Hq=16, Hkv=2, spec_k=4, seq_lens=[5, 255, 1000], budgets=[5, 16, 512]),
               what="two-pass fp8", flags=exact)
    round_trip(gen.make_workload(4, batch=1), what="two-pass config4[:1]", flags=exact)


def test_generic_kernels_on_a_matrix_core_shape():
    """PILLAR_FLAG_GENERIC_KERNELS: the vector-ALU kernels on a shape the matrix-core kernels normally take, against
    the oracle, and against the matrix-core result (two implementations of one definition)."""
    w = small(119, B=3, Hq=16, Hkv=4, spec_k=4, seq_lens=[6, 300, 1100], budgets=[6, 40, 64])
    slow, _ = round_trip(w, what="generic kernels, bf16", flags=pa.PILLAR_FLAG_GENERIC_KERNELS)
    fast, _ = round_trip(w, what="matrix-core kernels, same input")
    assert (to_f64(slow.out) - to_f64(fast.out)).__abs__().max() <= 1.6e-2       # two bf16 roundings of one value
    assert np.abs(to_f64(slow.lse) - to_f64(fast.lse)).max() <= LSE_ABS


def _floor_workload():
    """One request, one KV head, every query row the same vector 8 e_0, keys x_t e_0: the base-2 logit of token t is
    1.02 x_t for every row.  Token 0 has x = 64, the others sweep [-6, 6] every 128 tokens: their probabilities run from 2^-71 to
    2^-59, across the 2^-62 at which the 16-bit stash drops a value, and across [1e-20, 1e-19]."""
    L = 32768
    w = small(170, B=1, Hq=4, Hkv=1, spec_k=4, seq_lens=[L], budgets=[64])
    one = gen.bf16_bits_from_f32(np.array([8.0], dtype=np.float32))[0]
    w.q[:] = 0
    w.q[..., 0] = one
    x = np.tile(np.linspace(-6.0, 6.0, 128), L // 128).astype(np.float32)    # every 128 tokens cover the whole range
    x[0] = 64.0
    xb = gen.bf16_bits_from_f32(x)
    for t in range(L):
        page, slot = int(w.block_table[0, t // w.P]), t % w.P
        w.k_pool[page, 0, slot, :] = 0
        w.k_pool[page, 0, slot, 0] = xb[t]
    return w


def test_probabilities_below_the_stash_floor():
    """Reading R19: the default path drops a row's exponential below 2^-62 of its running maximum, so a score may
    be short by up to 2^-62 in absolute terms (and only a score below 2^-62 can be); above that the relative bound
    holds alone.  With PILLAR_FLAG_EXACT_SCORES the relative bound holds down to its 1e-20 floor."""
    from tests.harness import check_scores, SCORE_FLUSH
    w = _floor_workload()
    want = oracle.verify_attn(w)[2]
    band = (want[0, 0] >= 1e-20) & (want[0, 0] <= 1e-19)
    assert band.sum() > 100, "the workload must put scores into [1e-20, 1e-19]"
    pa.pillar_set_option("verify_waves", 1)              # ranges of several tiles: the large maximum is carried along
    try:
        run = GpuRun(w)
        run.run_all()
    finally:
        pa.pillar_set_option("verify_waves", 0)
    got = run.scores.cpu().numpy().astype(np.float64)
    check_scores(got, want, w.seq_lens, [0], "stash floor, default path", abs_slack=SCORE_FLUSH)
    big = want[0, 0] >= 2.0 ** -61
    rel = np.abs(got[0, 0, :len(big)][big] - want[0, 0][big]) / want[0, 0][big]
    assert rel.max() <= 1e-3, f"scores above the floor: rel error {rel.max():.3e}"
    dropped = (got[0, 0, :band.size] == 0) & band
    print(f"[floor] {int(band.sum())} scores in [1e-20, 1e-19], {int(dropped.sum())} of them dropped to 0", flush=True)
    assert dropped.any(), "the case must reach the floor it is about"
    exact = GpuRun(w, flags=pa.PILLAR_FLAG_EXACT_SCORES)
    exact.run_all()
    check_scores(exact.scores.cpu().numpy().astype(np.float64), want, w.seq_lens, [0], "stash floor, exact scores")


@pytest.mark.parametrize("flags", [0, pa.PILLAR_FLAG_EXACT_SCORES, pa.PILLAR_FLAG_GENERIC_KERNELS])
def test_context_shorter_than_its_queries(flags):
    """seq_lens[b] < k+1 is outside the documented range; the documented behaviour is harmless: a query that sees no
    token gets zeros and lse = -inf and adds nothing to the statistic, and nothing becomes NaN."""
    w = small(171, B=4, Hq=16, Hkv=4, spec_k=4, seq_lens=[2, 1, 300, 4], budgets=[2, 1, 40, 4], allow_short=True)
    run = GpuRun(w, flags=flags)
    run.run_all()
    want_out, want_lse, want_scores = oracle.verify_attn(w)
    check_out(to_f64(run.out), want_out, w.kv_dtype, "short contexts: out")
    lse = to_f64(run.lse)
    assert np.array_equal(np.isneginf(lse), np.isneginf(want_lse))
    fin = np.isfinite(want_lse)
    assert np.abs(lse[fin] - want_lse[fin]).max() <= LSE_ABS
    from tests.harness import check_scores, check_topk_exact
    check_scores(run.scores.cpu().numpy().astype(np.float64), want_scores, w.seq_lens, range(w.B), "short contexts")
    check_topk_exact(run.indices.cpu().numpy(), run.counts.cpu().numpy(), run.scores.cpu().numpy()[:, :, :w.max_seq_len],
                     w.seq_lens, w.budgets, range(w.B), "short contexts")


# ------------------------------------------ the measured configs, reduced ----
@pytest.mark.parametrize("cfg,batch", [(2, 2), (3, 4), (4, 1), (5, 2)])
def test_config_reduced_batch(cfg, batch):
    round_trip(gen.make_workload(cfg, batch=batch), what=f"config{cfg}[:{batch}]")


# ------------------ full size, every request, through the calls bench.py times ----
@pytest.mark.timeout(1100)
@pytest.mark.parametrize("cfg,fused", [(2, True), (2, False), (3, True), (4, True), (5, True)])
def test_config_full_size_every_request(cfg, fused):
    """The whole batch of a measured configuration, launched as bench.py launches it (pillar_verify_select +
    pillar_sparse_decode; for config 2 also as three calls), every request compared element by element with the
    oracle: out, lse, scores, selection (bit-exact on the GPU's scores, tie band on the oracle's), draft."""
    w = gen.make_workload(cfg)
    run, rep = round_trip(w, what=f"config{cfg} full size, fused={fused}", fused_select=fused)
    scores = run.scores.cpu().numpy()
    for b in range(w.B):
        L = int(w.seq_lens[b])
        tot = scores[b, :, :L].astype(np.float64).sum(-1)
        assert np.all(np.abs(tot - 1.0) < 1e-4), f"request {b}: scores sum to {tot}"
    assert np.array_equal(run.counts.cpu().numpy(), np.minimum(w.budgets, w.seq_lens))


# --------------------------- verification and selection in one call ----------
def _same_as_two_calls(w, what, with_scores=True, flags=0):
    """pillar_verify_select against pillar_verify_attn + pillar_select_topk on the same inputs: every
    output bit for bit, and the whole round against the oracle."""
    two = GpuRun(w, flags=flags)
    two.run_all()
    one = GpuRun(w, flags=flags)
    one.verify_select(with_scores=with_scores)
    one.decode()
    torch.cuda.synchronize()
    assert torch.equal(one.out.view(torch.int16), two.out.view(torch.int16)), f"{what}: out differs"
    assert torch.equal(one.lse, two.lse), f"{what}: lse differs"
    assert torch.equal(one.counts, two.counts) and torch.equal(one.indices, two.indices), f"{what}: selection differs"
    assert torch.equal(one.d_out.view(torch.int16), two.d_out.view(torch.int16)), f"{what}: draft differs"
    if with_scores:
        for b in range(w.B):
            L = int(w.seq_lens[b])
            assert torch.equal(one.scores[b, :, :L], two.scores[b, :, :L]), f"{what}: scores differ, request {b}"
        rep = compare_with_oracle(w, one, None, what)
        print(f"[ok] {what}: {rep}", flush=True)


def test_verify_select_equals_the_two_calls():
    _same_as_two_calls(small(120, B=4, Hq=16, Hkv=4, spec_k=4, seq_lens=[5, 700, 2049, 33], budgets=[8, 64, 128, 40]), "fused select")
    _same_as_two_calls(small(121, kv_dtype="fp8_e4m3", Hq=16, Hkv=2, spec_k=4, seq_lens=[5, 255, 1000], budgets=[5, 16, 512]),
                       "fused select fp8")
    _same_as_two_calls(small(122, P=64, spec_k=8, Hq=8, Hkv=2, seq_lens=[9, 64, 700], budgets=[9, 64, 100]), "fused select 36 rows")
    _same_as_two_calls(small(123, B=2, Hq=8, Hkv=2, spec_k=2, seq_lens=[9000, 300], budgets=[300, 300]), "fused select, 16 keys per thread")
    _same_as_two_calls(small(124, B=3, Hq=8, Hkv=2, spec_k=2, seq_lens=[3, 130, 517], budgets=[2, 40, 64]), "fused select, no scores",
                       with_scores=False)
    # shapes the matrix-core path does not take go through the two calls inside the library
    _same_as_two_calls(small(125, q_dtype="f32", kv_dtype="f32", D=64), "fused select, generic path")
    _same_as_two_calls(small(126, q_dtype="f32", kv_dtype="f32", D=64), "fused select, generic path, no scores", with_scores=False)


def test_verify_select_with_the_two_pass_variant():
    _same_as_two_calls(small(127, B=3, Hq=16, Hkv=4, spec_k=4, seq_lens=[40, 700, 2049], budgets=[8, 64, 128]),
                       "select, fp32 probabilities", flags=pa.PILLAR_FLAG_EXACT_SCORES)


def test_verify_select_reduced_configs():
    # config 4's rows (28 K tokens) are longer than the finish kernel keeps on chip: two steps inside the library
    for cfg, batch in [(3, 4), (5, 2), (4, 1)]:
        _same_as_two_calls(gen.make_workload(cfg, batch=batch), f"fused select config{cfg}[:{batch}]")


# -------------------------------------------- index lists from other sources ----
def test_window_and_tail_lists_match_the_oracle_and_feed_the_draft():
    """Static sink + window lists and the post-verification tail: integer-exact against the oracle,
    and the draft kernel on those lists against the oracle's sparse attention."""
    rng = np.random.default_rng(11)
    lens = [3, 40, 517, 2049, 64]
    w = small(130, B=5, Hq=16, Hkv=4, spec_k=2, seq_lens=lens, budgets=[8, 12, 64, 128, 64])
    run = GpuRun(w)
    pa.pillar_window_indices(run.dw.kv.seq_lens, run.dw.budgets, w.Hkv, 4, run.max_budget, run.indices, run.counts)
    torch.cuda.synchronize()
    want_idx, want_cnt = oracle.window_indices(w.seq_lens, w.budgets, w.Hkv, 4, max_budget=run.max_budget)
    assert np.array_equal(run.counts.cpu().numpy(), want_cnt)
    assert np.array_equal(run.indices.cpu().numpy(), want_idx)
    # the tail: pretend the last tokens of each request were generated after the lists were made
    n_new = np.array([1, 2, 0, 2, 70], dtype=np.int32)
    first_new = (w.seq_lens - np.minimum(n_new, w.seq_lens)).astype(np.int32)
    pa.pillar_extend_indices(run.indices, run.counts, torch.from_numpy(first_new).to(run.dev), torch.from_numpy(n_new).to(run.dev))
    torch.cuda.synchronize()
    ext_idx, ext_cnt = oracle.extend_indices(want_idx, want_cnt, first_new, n_new)
    got_idx, got_cnt = run.indices.cpu().numpy(), run.counts.cpu().numpy()
    assert np.array_equal(got_cnt, ext_cnt)
    for b in range(w.B):
        assert np.array_equal(got_idx[b, :, :ext_cnt[b]], ext_idx[b, :, :ext_cnt[b]]), f"request {b}"
    run.decode()
    torch.cuda.synchronize()
    want_out, want_lse = oracle.sparse_decode(w, ext_idx, ext_cnt)
    check_out(to_f64(run.d_out), want_out, w.kv_dtype, "draft on window + tail lists")
    assert np.abs(run.d_lse.cpu().numpy() - want_lse).max() < LSE_ABS


# ------------------------------------------- per-request speculative lengths ----
def _hetero_case(w, spec, what, with_select):
    run = GpuRun(w)
    spec_dev = torch.from_numpy(spec.astype(np.int32)).to(run.dev)
    if with_select:
        pa.pillar_verify_hetero(run.dw.kv, run.dw.q, w.spec_k, spec_dev, run.out, run.lse, run.scores, run.workspace,
                                budgets=run.dw.budgets, max_budget=run.max_budget, indices=run.indices, counts=run.counts)
    else:
        pa.pillar_verify_hetero(run.dw.kv, run.dw.q, w.spec_k, spec_dev, run.out, run.lse, run.scores, run.workspace)
        run.topk()
    torch.cuda.synchronize()
    want_out, want_lse, want_scores = oracle.verify_attn(w, spec_lens=spec)
    got_out, got_lse = to_f64(run.out), run.lse.cpu().numpy().astype(np.float64)
    for b in range(w.B):
        nq = int(spec[b]) + 1
        check_out(got_out[b, :nq], want_out[b, :nq], w.kv_dtype, f"{what}: out of request {b}")
        assert np.abs(got_lse[b, :nq] - want_lse[b, :nq]).max() < LSE_ABS, f"{what}: lse of request {b}"
        assert np.isnan(got_out[b, nq:]).all(), f"{what}: unused query slots of request {b} were written"
    from tests.harness import check_scores, check_topk_against_oracle_scores
    worst = check_scores(run.scores.cpu().numpy(), want_scores, w.seq_lens, range(w.B), what)
    check_topk_against_oracle_scores(run.indices.cpu().numpy(), run.counts.cpu().numpy(), want_scores, w.seq_lens, w.budgets,
                                     range(w.B), what)
    print(f"[ok] {what}: scores {worst:.2e}", flush=True)


def test_requests_with_different_speculative_lengths():
    w = small(160, B=5, Hq=16, Hkv=4, spec_k=4, seq_lens=[5, 700, 2049, 33, 1500], budgets=[4, 64, 128, 16, 64])
    _hetero_case(w, np.array([4, 0, 2, 3, 1]), "hetero k", with_select=False)
    _hetero_case(w, np.array([0, 4, 1, 0, 3]), "hetero k, fused selection", with_select=True)
    w8 = small(161, kv_dtype="fp8_e4m3", Hq=16, Hkv=2, spec_k=4, seq_lens=[5, 255, 1000], budgets=[5, 16, 128])
    _hetero_case(w8, np.array([2, 4, 0]), "hetero k, fp8, 40 rows", with_select=True)
    with pytest.raises(pa.PillarError) as e:      # the generic kernels do not know per-request lengths
        wf = small(162, q_dtype="f32", kv_dtype="f32", D=64)
        r = GpuRun(wf)
        pa.pillar_verify_hetero(r.dw.kv, r.dw.q, wf.spec_k, torch.zeros(wf.B, dtype=torch.int32, device=r.dev), r.out, r.lse,
                                r.scores, r.workspace)
    assert e.value.status == pa.binding.PILLAR_EUNSUPPORTED


# ------------------------------------------------------------- KV append ------
@pytest.mark.parametrize("kv_dtype,q_dtype,D", [("bf16", "bf16", 128), ("f32", "f32", 64)])
def test_append_kv_then_verify(kv_dtype, q_dtype, D):
    """Cut the rows of the k+1 newest tokens out of the pools on the GPU (poison them), append them
    through the entry point: the pools are back bit for bit (as the oracle's append makes them), and the
    whole round on them matches the oracle."""
    w = small(150, B=4, Hq=8, Hkv=2, D=D, spec_k=3, q_dtype=q_dtype, kv_dtype=kv_dtype, seq_lens=[4, 130, 517, 64],
              budgets=[4, 40, 64, 64])
    n = w.n_q
    run = GpuRun(w)
    k_new = np.zeros((w.B, n, w.Hkv, w.D), dtype=w.k_pool.dtype)
    v_new = np.zeros_like(k_new)
    k_cut, v_cut = w.k_pool.copy(), w.v_pool.copy()
    poison = np.array(0x7FC1 if kv_dtype == "bf16" else 0x7FC00001).astype(w.k_pool.dtype)
    for b in range(w.B):
        L = int(w.seq_lens[b])
        for i in range(n):
            pos = L - n + i
            page, slot = int(w.block_table[b, pos // w.P]), pos % w.P
            k_new[b, i], v_new[b, i] = w.k_pool[page, :, slot, :], w.v_pool[page, :, slot, :]
            k_cut[page, :, slot, :] = poison
            v_cut[page, :, slot, :] = poison
    want_k, want_v = oracle.append_kv(w, k_cut, v_cut, k_new, v_new)
    bits = lambda a: a.view(np.uint16 if kv_dtype == "bf16" else np.uint32)      # unused slots hold NaN patterns
    assert np.array_equal(bits(want_k), bits(w.k_pool)) and np.array_equal(bits(want_v), bits(w.v_pool))
    kv = run.dw.kv
    kv.k_pool.view(torch.int16 if kv_dtype == "bf16" else torch.int32).copy_(torch.from_numpy(k_cut.view(np.int16 if kv_dtype == "bf16" else np.int32)))
    kv.v_pool.view(torch.int16 if kv_dtype == "bf16" else torch.int32).copy_(torch.from_numpy(v_cut.view(np.int16 if kv_dtype == "bf16" else np.int32)))
    to_dev = lambda x: torch.from_numpy(x.view(np.int16 if kv_dtype == "bf16" else np.int32)).to(run.dev)
    pa.pillar_append_kv(kv, to_dev(k_new), to_dev(v_new))
    torch.cuda.synchronize()
    as_int = torch.int16 if kv_dtype == "bf16" else torch.int32
    assert torch.equal(kv.k_pool.view(as_int).cpu(), torch.from_numpy(w.k_pool.view(np.int16 if kv_dtype == "bf16" else np.int32)))
    assert torch.equal(kv.v_pool.view(as_int).cpu(), torch.from_numpy(w.v_pool.view(np.int16 if kv_dtype == "bf16" else np.int32)))
    run.run_all()
    rep = compare_with_oracle(w, run, None, "round after append")
    print(f"[ok] append {kv_dtype}: {rep}", flush=True)


def test_append_kv_refuses_fp8_pools():
    w = small(151, kv_dtype="fp8_e4m3", Hq=16, Hkv=2, spec_k=2, seq_lens=[5, 255, 100], budgets=[5, 16, 16])
    run = GpuRun(w)
    fake = torch.zeros((w.B, 3, w.Hkv, w.D), dtype=torch.uint8, device=run.dev)
    with pytest.raises(pa.PillarError) as e:
        pa.pillar_append_kv(run.dw.kv, fake, fake)
    assert e.value.status == pa.binding.PILLAR_EUNSUPPORTED


# ------------------------------------------------------ stream capture ------
def test_step_replays_from_a_captured_graph():
    """The entry points only enqueue kernels on the caller's stream: a whole step captured into a graph and
    replayed gives, every time, exactly what the eager calls give (outputs are wiped between replays)."""
    w = small(140, B=4, Hq=16, Hkv=4, spec_k=4, seq_lens=[40, 700, 2049, 333], budgets=[8, 64, 128, 32])
    eager = GpuRun(w)
    eager.run_all(fused_select=True)
    run = GpuRun(w)
    run.run_all(fused_select=True)              # first calls outside the capture (one-time function attributes)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run.verify_select()
            run.decode()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (run.out, run.lse, run.scores, run.d_out, run.d_lse):
            t.fill_(float("nan"))
        run.indices.fill_(-7)
        run.counts.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(run.out.view(torch.int16), eager.out.view(torch.int16)), f"replay {rep}: out"
        assert torch.equal(run.lse, eager.lse), f"replay {rep}: lse"
        assert torch.equal(run.indices, eager.indices) and torch.equal(run.counts, eager.counts), f"replay {rep}: selection"
        assert torch.equal(run.d_out.view(torch.int16), eager.d_out.view(torch.int16)), f"replay {rep}: draft"
        for b in range(w.B):
            L = int(w.seq_lens[b])
            assert torch.equal(run.scores[b, :, :L], eager.scores[b, :, :L]), f"replay {rep}: scores of request {b}"


# ----------------------------------------------------------- edge cases ------
def test_outputs_are_bit_identical_from_run_to_run():
    w = small(201, seq_lens=[40, 300, 1500], budgets=[8, 30, 100])
    run = GpuRun(w)
    run.run_all()
    first = [t.clone() for t in (run.out, run.lse, run.scores, run.indices, run.counts, run.d_out, run.d_lse)]
    run.run_all()
    for a, b in zip(first, (run.out, run.lse, run.scores, run.indices, run.counts, run.d_out, run.d_lse)):
        assert torch.equal(a.view(torch.uint8).flatten(), b.view(torch.uint8).flatten())


def test_optional_outputs_may_be_null():
    w = small(202)
    run = GpuRun(w)
    run.verify(with_scores=False, with_lse=False)
    torch.cuda.synchronize()
    assert torch.isnan(run.scores).all() and torch.isnan(run.lse).all()
    want, _, _ = oracle.verify_attn(w)
    check_out(to_f64(run.out), want, w.kv_dtype, "out without scores")


def test_sparse_with_every_index_equals_verify_with_k0():
    w = small(203, spec_k=0, seq_lens=[1, 77, 600], budgets=[1, 77, 600])
    w.q_draft = w.q[:, 0].copy()
    run = GpuRun(w)
    run.run_all()
    assert run.counts.cpu().tolist() == [1, 77, 600]
    assert run.indices[2, 0].cpu().tolist() == list(range(600))
    a, b = to_f64(run.out[:, 0]), to_f64(run.d_out)
    assert np.abs(a - b).max() <= 1.6e-2            # two bf16 roundings of the same value
    assert np.abs(to_f64(run.lse[:, 0]) - to_f64(run.d_lse)).max() <= LSE_ABS
    compare_with_oracle(w, run)


def test_strided_pool_layout_and_wide_block_table():
    # pool stored [page][slot][head][dim]; the block table has spare columns
    w = small(204, extra_table_cols=3)
    run = GpuRun(w)
    kv = run.dw.kv
    kv.k_pool = kv.k_pool.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    kv.v_pool = kv.v_pool.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert kv.k_pool.stride(1) == w.D and kv.k_pool.stride(2) == w.Hkv * w.D
    run.run_all()
    compare_with_oracle(w, run)


def test_empty_selection_and_zero_budget():
    w = small(205, budgets=[0, 5, 0])
    run = GpuRun(w)
    run.run_all()
    assert run.counts.cpu().tolist() == [0, 5, 0]
    assert (run.indices[0] == -1).all() and (run.indices[2] == -1).all()
    assert (run.d_out[0] == 0).all() and torch.isinf(run.d_lse[0]).all() and (run.d_lse[0] < 0).all()
    compare_with_oracle(w, run, requests=[1])


def test_topk_exact_ties_synthetic_scores():
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(7)
    B, Hkv, L = 3, 2, 5000
    s = (rng.integers(0, 6, size=(B, Hkv, L)) / 8.0).astype(np.float32)        # only six distinct values
    s[2] = rng.random((Hkv, L)).astype(np.float32) ** 12                        # tiny values, wide exponent range
    lens = np.array([5000, 4097, 1023], dtype=np.int32)
    bud = np.array([700, 4097, 1], dtype=np.int32)
    st = torch.from_numpy(s).to(dev)
    idx = torch.full((B, Hkv, 4097), -9, dtype=torch.int32, device=dev)
    cnt = torch.zeros(B, dtype=torch.int32, device=dev)
    pa.pillar_select_topk(st, torch.from_numpy(lens).to(dev), torch.from_numpy(bud).to(dev), 5000, 4097, idx, cnt)
    torch.cuda.synchronize()
    check_topk_exact(idx.cpu().numpy(), cnt.cpu().numpy(), s, lens, bud, [0, 1, 2], "ties")


def test_decode_accepts_unsorted_and_repeated_free_lists():
    w = small(206, seq_lens=[50, 300, 900], budgets=[10, 100, 300])
    run = GpuRun(w)
    run.verify(); run.topk()
    torch.cuda.synchronize()
    idx = run.indices.cpu().numpy().copy()
    cnt = run.counts.cpu().numpy()
    rng = np.random.default_rng(1)
    for b in range(w.B):
        for g in range(w.Hkv):
            idx[b, g, :cnt[b]] = rng.permutation(idx[b, g, :cnt[b]])
    ti = torch.from_numpy(idx).to(run.dev)
    run.decode(indices=ti)
    torch.cuda.synchronize()
    want, want_l = oracle.sparse_decode(w, idx, cnt)
    check_out(to_f64(run.d_out), want, w.kv_dtype, "shuffled list")
