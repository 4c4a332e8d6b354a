"""The C ABI without a GPU: the library loads, exports what the header
declares, and rejects bad arguments on the host before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2512_01278_amd import binding as pb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # non-null, 256-aligned, never dereferenced on the host


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pb.LIB_PATH):
        from paper_2512_01278_amd.build import build
        build(verbose=False)
    return pb.load()


def good_kv(**kw):
    s = pb.pillar_kv_t()
    s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, s.page_size = 4, 32, 8, 128, 16
    s.q_dtype, s.kv_dtype, s.sm_scale = pb.PILLAR_BF16, pb.PILLAR_BF16, 0.088
    s.k_pool = s.v_pool = s.block_table = s.seq_lens = FAKE
    s.stride_page, s.stride_head, s.stride_slot = 8 * 16 * 128, 16 * 128, 128
    s.num_pages, s.block_table_stride, s.max_seq_len = 1000, 64, 1024
    for k, v in kw.items():
        setattr(s, k, v)
    return s


def test_header_functions_are_all_exported(lib):
    names = set()
    for header in ("pillar.h", "pillar_bench.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(pillar_[a-z_]+)\s*\(", text))
    assert names == set(pb.EXPORTS), names ^ set(pb.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layout_matches_the_header():
    assert C.sizeof(pb.pillar_kv_t) == 120 and pb.pillar_kv_t.k_pool.offset == 32
    assert pb.pillar_kv_t.block_table.offset == 96 and pb.pillar_kv_t.max_seq_len.offset == 112
    assert C.sizeof(pb.pillar_kernel_time) == 64


def test_version_and_status_strings(lib):
    assert lib.pillar_version() >= 100
    seen = {lib.pillar_status_string(c) for c in (0, -1, -2, -3, -4, -5)}
    assert len(seen) == 6 and b"unknown" in lib.pillar_status_string(-99)


def verify(lib, s, q=FAKE, k=4, out=FAKE, scores=FAKE, stride=1024, ws=FAKE, wsz=1 << 40):
    return lib.pillar_verify_attn(C.byref(s), q, k, out, None, scores, stride, ws, wsz, None)


def test_workspace_query(lib):
    s = good_kv()
    n = lib.pillar_workspace_bytes(C.byref(s), 4, 256)
    assert n > 0 and n % 256 == 0
    assert lib.pillar_workspace_bytes(C.byref(good_kv(batch=0)), 4, 256) == 0
    assert lib.pillar_workspace_bytes(None, 4, 256) == 0
    assert lib.pillar_workspace_bytes(C.byref(s), 16, 256) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(batch=0), pb.PILLAR_EINVAL), (dict(num_kv_heads=5), pb.PILLAR_EINVAL),
    (dict(k_pool=None), pb.PILLAR_EINVAL), (dict(seq_lens=None), pb.PILLAR_EINVAL),
    (dict(kv_dtype=pb.PILLAR_FP8_E4M3), pb.PILLAR_EINVAL),           # fp8 without scales
    (dict(sm_scale=0.0), pb.PILLAR_EINVAL), (dict(stride_slot=64), pb.PILLAR_EINVAL),
    (dict(max_seq_len=64 * 16 + 1), pb.PILLAR_EINVAL),
    (dict(head_dim=96, stride_slot=128), pb.PILLAR_EUNSUPPORTED), (dict(page_size=24), pb.PILLAR_EUNSUPPORTED),
    (dict(q_dtype=pb.PILLAR_FP8_E4M3), pb.PILLAR_EUNSUPPORTED), (dict(kv_dtype=7), pb.PILLAR_EUNSUPPORTED),
    (dict(num_q_heads=8 * 32), pb.PILLAR_EUNSUPPORTED),
    (dict(flags=4), pb.PILLAR_EINVAL), (dict(flags=-1), pb.PILLAR_EINVAL),
])
def test_bad_cache_descriptions_are_rejected(lib, kw, code):
    s = good_kv(**kw)
    assert verify(lib, s) == code
    assert lib.pillar_sparse_decode(C.byref(s), FAKE, FAKE, FAKE, 256, FAKE, None, FAKE, 1 << 40, None) == code


def test_bad_call_arguments_are_rejected(lib):
    s = good_kv()
    assert verify(lib, s, q=None) == pb.PILLAR_EINVAL
    assert verify(lib, s, out=None) == pb.PILLAR_EINVAL
    assert verify(lib, s, k=-1) == pb.PILLAR_EINVAL
    assert verify(lib, s, k=16) == pb.PILLAR_EUNSUPPORTED
    assert verify(lib, good_kv(num_q_heads=64), k=8) == pb.PILLAR_EUNSUPPORTED     # 9*8 rows > 64
    assert verify(lib, s, stride=1000) == pb.PILLAR_EINVAL
    assert verify(lib, s, ws=None) == pb.PILLAR_EWORKSPACE
    assert verify(lib, s, ws=FAKE + 8) == pb.PILLAR_EWORKSPACE
    assert verify(lib, s, wsz=128) == pb.PILLAR_EWORKSPACE
    assert lib.pillar_verify_attn(None, FAKE, 4, FAKE, None, None, 0, FAKE, 1 << 40, None) == pb.PILLAR_EINVAL
    tk = lambda **k: lib.pillar_select_topk(k.get("scores", FAKE), k.get("stride", 1024), FAKE, k.get("budgets", FAKE),
                                            k.get("batch", 4), 8, 1024, k.get("mb", 256), FAKE, k.get("counts", FAKE),
                                            None, 0, None)
    assert tk(scores=None) == pb.PILLAR_EINVAL and tk(budgets=None) == pb.PILLAR_EINVAL
    assert tk(counts=None) == pb.PILLAR_EINVAL and tk(batch=0) == pb.PILLAR_EINVAL
    assert tk(mb=0) == pb.PILLAR_EINVAL and tk(stride=512) == pb.PILLAR_EINVAL
    vs = lambda **k: lib.pillar_verify_select(C.byref(s), k.get("q", FAKE), 4, FAKE, None, None, 0, k.get("budgets", FAKE),
                                              k.get("mb", 256), k.get("idx", FAKE), k.get("cnt", FAKE), k.get("ws", FAKE),
                                              k.get("wsz", 1 << 40), None)
    assert vs(q=None) == pb.PILLAR_EINVAL and vs(budgets=None) == pb.PILLAR_EINVAL and vs(idx=None) == pb.PILLAR_EINVAL
    assert vs(cnt=None) == pb.PILLAR_EINVAL and vs(mb=0) == pb.PILLAR_EINVAL
    assert vs(ws=None) == pb.PILLAR_EWORKSPACE and vs(wsz=128) == pb.PILLAR_EWORKSPACE
    vh = lambda **k: lib.pillar_verify_hetero(C.byref(k.get("kv", s)), FAKE, 4, k.get("spec", FAKE), FAKE, None, None, 0,
                                              k.get("budgets", None), k.get("mb", 0), k.get("idx", None), k.get("cnt", None),
                                              FAKE, 1 << 40, None)
    assert vh(spec=None) == pb.PILLAR_EINVAL
    assert vh(budgets=FAKE) == pb.PILLAR_EINVAL                      # selection wanted, but not all of its arguments
    assert vh(budgets=FAKE, idx=FAKE, cnt=FAKE, mb=0) == pb.PILLAR_EINVAL
    assert vh(kv=good_kv(q_dtype=pb.PILLAR_F32, kv_dtype=pb.PILLAR_F32)) == pb.PILLAR_EUNSUPPORTED   # generic kernels only
    assert vh(kv=good_kv(flags=pb.PILLAR_FLAG_EXACT_SCORES)) == pb.PILLAR_EUNSUPPORTED
    assert vh(kv=good_kv(flags=pb.PILLAR_FLAG_GENERIC_KERNELS)) == pb.PILLAR_EUNSUPPORTED
    assert lib.pillar_append_kv(C.byref(s), None, FAKE, 3, None) == pb.PILLAR_EINVAL
    assert lib.pillar_append_kv(C.byref(s), FAKE, FAKE, 0, None) == pb.PILLAR_EINVAL
    assert lib.pillar_append_kv(C.byref(good_kv(kv_dtype=pb.PILLAR_FP8_E4M3, k_scale=FAKE, v_scale=FAKE)), FAKE, FAKE, 3, None) \
        == pb.PILLAR_EUNSUPPORTED
    assert lib.pillar_window_indices(None, FAKE, 4, 8, 4, 64, FAKE, FAKE, None) == pb.PILLAR_EINVAL
    assert lib.pillar_window_indices(FAKE, FAKE, 4, 8, -1, 64, FAKE, FAKE, None) == pb.PILLAR_EINVAL
    assert lib.pillar_extend_indices(FAKE, FAKE, None, FAKE, 4, 8, 64, None) == pb.PILLAR_EINVAL
    assert lib.pillar_extend_indices(FAKE, FAKE, FAKE, FAKE, 4, 8, 0, None) == pb.PILLAR_EINVAL
    sd = lambda **k: lib.pillar_sparse_decode(C.byref(s), k.get("q", FAKE), k.get("idx", FAKE), k.get("cnt", FAKE),
                                              k.get("mb", 256), k.get("out", FAKE), None, FAKE, 1 << 40, None)
    assert sd(q=None) == pb.PILLAR_EINVAL and sd(idx=None) == pb.PILLAR_EINVAL
    assert sd(cnt=None) == pb.PILLAR_EINVAL and sd(out=None) == pb.PILLAR_EINVAL and sd(mb=0) == pb.PILLAR_EINVAL


def test_mixed_step_arguments(lib):
    s = good_kv()
    def ms(kv=s, vids=FAKE, nv=2, dids=FAKE, nd=2, qv=FAKE, outv=FAKE, budgets=FAKE, mb=256, idx=FAKE, cnt=FAKE, qd=FAKE, outd=FAKE,
           ws=FAKE, wsz=1 << 40):
        return lib.pillar_mixed_step(C.byref(kv), vids, nv, dids, nd, qv, 4, outv, None, None, 0, budgets, mb, idx, cnt, qd, outd, None,
                                     ws, wsz, None)
    assert ms(nv=-1) == pb.PILLAR_EINVAL and ms(nd=5) == pb.PILLAR_EINVAL          # more than the batch holds
    assert ms(vids=None) == pb.PILLAR_EINVAL and ms(dids=None) == pb.PILLAR_EINVAL
    assert ms(qv=None) == pb.PILLAR_EINVAL and ms(outd=None) == pb.PILLAR_EINVAL
    assert ms(budgets=None) == pb.PILLAR_EINVAL and ms(mb=0) == pb.PILLAR_EINVAL and ms(cnt=None) == pb.PILLAR_EINVAL
    assert ms(ws=None) == pb.PILLAR_EWORKSPACE and ms(wsz=128) == pb.PILLAR_EWORKSPACE
    assert ms(kv=good_kv(flags=pb.PILLAR_FLAG_EXACT_SCORES)) == pb.PILLAR_EUNSUPPORTED
    assert ms(kv=good_kv(q_dtype=pb.PILLAR_F32, kv_dtype=pb.PILLAR_F32)) == pb.PILLAR_EUNSUPPORTED
    assert ms(nv=0, nd=0, vids=None, dids=None, qv=None, outv=None, qd=None, outd=None) == pb.PILLAR_OK     # nothing to do


def test_static_decode_rejects_what_its_scratch_cannot_hold(lib):
    sds = lambda s, mb=256, q=FAKE: lib.pillar_sparse_decode_static(C.byref(s), q, FAKE, FAKE, mb, FAKE, None, None)
    assert sds(good_kv(), q=None) == pb.PILLAR_EINVAL and sds(good_kv(), mb=0) == pb.PILLAR_EINVAL
    assert sds(good_kv(batch=0)) == pb.PILLAR_EINVAL
    # 2048 requests x 8 heads x 8 splits x 4 rows x 512 B of partial results = 268 MB: beyond the 32 MiB array
    assert sds(good_kv(batch=2048, max_seq_len=1024), mb=1024) == pb.PILLAR_ETOOLARGE
    assert b"32 MiB" in lib.pillar_status_string(pb.PILLAR_ETOOLARGE)


def test_option_names_and_ranges(lib):
    lib.pillar_set_option.restype = C.c_int
    lib.pillar_set_option.argtypes = [C.c_char_p, C.c_int64]
    ok = [(b"verify_waves", 4), (b"verify_waves", 0), (b"decode_rows", 64), (b"decode_rows", 0)]
    for name, value in ok:
        assert lib.pillar_set_option(name, value) == 0, (name, value)
    bad = [(b"verify_waves", 9), (b"verify_mode", 1), (b"decode_rows", 48), (b"decode_rows", 8192),
           (b"verify_waves", -1), (b"no_such_knob", 1), (None, 1)]
    for name, value in bad:
        assert lib.pillar_set_option(name, value) == -1, (name, value)


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    monkeypatch.setattr(pb, "_lib", None)
    monkeypatch.setattr(pb, "LIB_PATH", "/nonexistent/libpillar.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        pb.load()
