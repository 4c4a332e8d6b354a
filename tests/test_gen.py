"""The seeded generator: determinism, layout, and the structure it promises."""
import numpy as np

import gen


def test_same_seed_same_tensors_and_config_shapes():
    a, b = gen.make_workload(1), gen.make_workload(1)
    for f in ("q", "q_draft", "k_pool", "v_pool", "block_table", "seq_lens", "budgets"):
        assert np.array_equal(getattr(a, f), getattr(b, f), equal_nan=True), f
    assert a.seq_lens.tolist() == [300, 512] and a.num_pages == 51 and a.k_pool.shape == (51, 1, 16, 64)
    assert a.n_q == 4 and a.G == 4 and a.budgets.tolist() == [64, 64]


def test_block_table_uses_distinct_pages_and_poison_marks_the_rest():
    w = gen.make_custom(name="t", seed=3, B=3, Hq=2, Hkv=2, D=8, P=4, spec_k=1, q_dtype="bf16",
                        kv_dtype="bf16", seq_lens=[5, 8, 2], budgets=[1, 1, 1], pool_factor=2.0)
    used = w.block_table[w.block_table >= 0]
    assert len(set(used.tolist())) == len(used) == 2 + 2 + 1
    nan = lambda x: (x & 0x7FFF) > 0x7F80
    for p in range(w.num_pages):
        if p not in used:
            assert nan(w.k_pool[p]).all() and nan(w.v_pool[p]).all()
    last = w.block_table[0, 1]                      # request 0: 5 tokens, slot 0 of its 2nd page valid
    assert not nan(w.k_pool[last, :, 0]).any() and nan(w.k_pool[last, :, 1:]).all()


def test_fp8_pool_decodes_close_to_a_normal_and_scales_are_per_page_head():
    w = gen.make_custom(name="t", seed=4, B=1, Hq=8, Hkv=2, D=32, P=16, spec_k=0, q_dtype="bf16",
                        kv_dtype="fp8_e4m3", seq_lens=[64], budgets=[4], exact_pool=True, pillar_frac=0)
    assert w.k_scale.shape == (4, 2) and w.k_pool.dtype == np.uint8
    assert (w.k_pool & 0x7F).max() == 0x7E           # each tile's amax maps to 448
    assert np.all(w.k_scale > 0) and np.all(w.k_scale < 0.02)


def test_budget_rule_of_config3_and_required_bytes():
    w = gen.make_workload(3, batch=2)
    assert np.all(w.budgets % 64 == 0) and np.all(w.budgets >= 0.05 * w.seq_lens) and np.all(w.budgets < 0.05 * w.seq_lens + 64)
    tok = int(w.seq_lens.sum())
    assert w.verify_bytes() == tok * 8 * (2 * 128 * 2 + 4) + 2 * 2 * 5 * 32 * 128 * 2
    assert w.draft_bytes() == int(w.budgets.sum()) * 8 * (512 + 4) + 2 * 2 * 32 * 128 * 2
