"""A unified draft / verify batch (paper Section 4.2) through pillar_mixed_step, against the oracle's per-request
composition, and against the same work done as two calls."""
import numpy as np
import pytest
import torch

import gen
import oracle
import paper_2512_01278_amd as pa
from paper_2512_01278_amd.runner import GpuRun
from tests.harness import (LSE_ABS, check_out, check_scores, check_topk_against_oracle_scores, check_topk_exact, to_f64)

pytestmark = pytest.mark.gpu


def _prepare(w):
    """Lists of a previous verification for every request, then sentinels in every output."""
    run = GpuRun(w)
    run.verify_select()
    torch.cuda.synchronize()
    old_idx, old_cnt = run.indices.clone(), run.counts.clone()
    for t in (run.out, run.lse, run.scores, run.d_out, run.d_lse):
        t.fill_(float("nan"))
    return run, old_idx, old_cnt


def _mixed(run, ver, dra):
    dev = run.dev
    v = torch.tensor(ver, dtype=torch.int32, device=dev) if len(ver) else None
    d = torch.tensor(dra, dtype=torch.int32, device=dev) if len(dra) else None
    w = run.w
    pa.pillar_mixed_step(run.dw.kv, v, d, run.dw.q, w.spec_k, run.out, run.lse, run.scores, run.dw.budgets, run.max_budget,
                         run.indices, run.counts, run.dw.q_draft, run.d_out, run.d_lse, run.workspace)


def _check_against_oracle(w, run, ver, dra, old_idx, old_cnt, what):
    ref = oracle.mixed_step(w, ver, dra, old_idx.cpu().numpy(), old_cnt.cpu().numpy())
    out, lse, scores = to_f64(run.out), to_f64(run.lse), to_f64(run.scores)
    idx, cnt = run.indices.cpu().numpy(), run.counts.cpu().numpy()
    d_out, d_lse = to_f64(run.d_out), to_f64(run.d_lse)
    if ver:
        check_out(out[ver], ref["out"][ver], w.kv_dtype, what + ": verification out")
        assert np.abs(lse[ver] - ref["lse"][ver]).max() <= LSE_ABS
        check_scores(scores, ref["scores"], w.seq_lens, ver, what)
        check_topk_exact(idx, cnt, run.scores.cpu().numpy()[:, :, :w.max_seq_len], w.seq_lens, w.budgets, ver, what)
        check_topk_against_oracle_scores(idx, cnt, ref["scores"], w.seq_lens, w.budgets, ver, what)
    if dra:
        check_out(d_out[dra], ref["draft_out"][dra], w.kv_dtype, what + ": draft out")
        assert np.abs(d_lse[dra] - ref["draft_lse"][dra]).max() <= LSE_ABS
    # a request keeps what its phase does not produce
    for b in range(w.B):
        if b not in ver:
            assert np.isnan(out[b]).all() and np.isnan(lse[b]).all() and np.isnan(scores[b]).all(), f"{what}: request {b} was verified"
            assert np.array_equal(idx[b], old_idx[b].cpu().numpy()) and cnt[b] == int(old_cnt[b]), f"{what}: lists of request {b} changed"
        if b not in dra:
            assert np.isnan(d_out[b]).all() and np.isnan(d_lse[b]).all(), f"{what}: request {b} was drafted"


def _case(w, ver, dra, what, draft_bits=True):
    print(f"[case] {what}: B={w.B} L={w.seq_lens.tolist()[:8]} verify={ver} draft={dra}", flush=True)
    run, old_idx, old_cnt = _prepare(w)
    _mixed(run, ver, dra)
    torch.cuda.synchronize()
    _check_against_oracle(w, run, ver, dra, old_idx, old_cnt, what)
    # the same work as two calls (verification of the one list, then the draft of the other): the same bits
    two, oi, oc = _prepare(w)
    _mixed(two, ver, [])
    _mixed(two, [], dra)
    torch.cuda.synchronize()
    for name in ("out", "lse", "scores", "indices", "counts", "d_out", "d_lse"):
        a, b = getattr(run, name), getattr(two, name)
        if name.startswith("d_") and not draft_bits:
            # more than 32 query rows: the draft workgroups of the fused grid have two wavefronts, those of the draft
            # kernel four, so the partial sums of a list are grouped differently (both were compared with the oracle)
            live = torch.as_tensor(sorted(dra), device=a.device, dtype=torch.long)
            assert torch.allclose(a[live].float(), b[live].float(), rtol=2e-2, atol=2e-2), f"{what}: {name} differs from the two calls"
            continue
        assert torch.equal(a.view(torch.uint8).flatten(), b.view(torch.uint8).flatten()), f"{what}: {name} differs from the two calls"
    print(f"[ok] {what}", flush=True)


def test_mixed_batch_small():
    w = gen.make_custom(name="mixed", seed=401, B=6, Hq=16, Hkv=4, D=128, P=16, spec_k=4, q_dtype="bf16", kv_dtype="bf16",
                        seq_lens=[700, 40, 2049, 5, 1300, 333], budgets=[64, 8, 128, 4, 96, 32], sink_tokens=4)
    _case(w, [1, 4], [0, 2, 3, 5], "mixed batch")
    _case(w, [5, 0, 2], [3], "mixed batch, lists in any order, one request idle")
    _case(w, [0, 1, 2, 3, 4, 5], [], "everything verifies")
    _case(w, [], [0, 1, 2, 3, 4, 5], "everything drafts")


def test_mixed_batch_long_lists_and_wide_groups():
    # lists longer than one 512-row span leave partials that the draft's merge kernel combines
    w = gen.make_custom(name="mixed-long", seed=402, B=4, Hq=16, Hkv=4, D=128, P=16, spec_k=2, q_dtype="bf16", kv_dtype="bf16",
                        seq_lens=[3000, 700, 2049, 1500], budgets=[1500, 300, 900, 100], sink_tokens=4)
    _case(w, [2], [0, 1, 3], "mixed batch, split lists")
    # 40 query rows per KV head (fp8 KV): the verification runs two wavefronts per range, and so do the draft workgroups of the same grid
    w8 = gen.make_custom(name="mixed-fp8", seed=403, B=4, Hq=16, Hkv=2, D=128, P=16, spec_k=4, q_dtype="bf16",
                         kv_dtype="fp8_e4m3", seq_lens=[255, 1000, 40, 600], budgets=[16, 128, 8, 64])
    _case(w8, [1, 2], [0, 3], "mixed batch, fp8, 40 rows", draft_bits=False)


def test_mixed_batch_config3_reduced():
    w = gen.make_workload(3, batch=10)
    _case(w, [0, 5], [1, 2, 3, 4, 6, 7, 8, 9], "config3[:10], every fifth request verifies")


def test_mixed_step_refuses_other_modes():
    w = gen.make_custom(name="mixed-f32", seed=404, B=2, Hq=8, Hkv=2, D=64, P=16, spec_k=2, q_dtype="f32", kv_dtype="f32",
                        seq_lens=[40, 300], budgets=[8, 16])
    run = GpuRun(w)
    with pytest.raises(pa.PillarError) as e:
        _mixed(run, [0], [1])
    assert e.value.status == pa.binding.PILLAR_EUNSUPPORTED
