// C ABI of the PillarAttn hot path: argument validation on the host, then
// dispatch to the kernel files.  Nothing here allocates device memory or
// synchronises (the optional profiler aside).
#include <hip/hip_runtime.h>

#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "launch.hpp"
#include "pillar.h"
#include "pillar_bench.h"

namespace pillar {

// ---------------------------------------------------------------- profiler --
// Event pairs come from a pool created by pillar_profile_enable: the entry points only record.
namespace {
struct Pending {
  const char* name;
  hipEvent_t start, stop;
};
constexpr size_t kEventPairs = 8192;
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_free;     // unused pairs
bool g_pool_made = false;
std::vector<Pending> g_pending;
std::map<std::string, std::pair<int64_t, double>> g_totals;

void drain_locked() {
  for (auto& p : g_pending) {
    float ms = 0.f;
    if (hipEventSynchronize(p.stop) == hipSuccess && hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
      auto& e = g_totals[p.name];
      e.first += 1;
      e.second += ms;
    }
    g_free.emplace_back(p.start, p.stop);
  }
  g_pending.clear();
}
}  // namespace

KernelTimer::KernelTimer(const char* name, hipStream_t stream) : name_(name), stream_(stream) {
  if (!g_prof_on) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (g_free.empty()) return;                  // pool used up: this launch goes unrecorded
  start_ = g_free.back().first;
  stop_ = g_free.back().second;
  g_free.pop_back();
  (void)hipEventRecord(start_, stream_);
}

KernelTimer::~KernelTimer() {
  if (!start_) return;
  (void)hipEventRecord(stop_, stream_);
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_pending.push_back({name_, start_, stop_});
}

// -------------------------------------------------------------- validation --
namespace {

bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

int check_kv(const pillar_kv_t* kv) {
  if (!kv) return PILLAR_EINVAL;
  if (kv->batch < 1 || kv->num_q_heads < 1 || kv->num_kv_heads < 1 || kv->head_dim < 1 || kv->page_size < 1 ||
      kv->num_pages < 1 || kv->block_table_stride < 1 || kv->max_seq_len < 1)
    return PILLAR_EINVAL;
  if (kv->num_q_heads % kv->num_kv_heads != 0) return PILLAR_EINVAL;
  if (!kv->k_pool || !kv->v_pool || !kv->block_table || !kv->seq_lens) return PILLAR_EINVAL;
  if (kv->q_dtype != PILLAR_F32 && kv->q_dtype != PILLAR_BF16) return PILLAR_EUNSUPPORTED;
  if (kv->kv_dtype != PILLAR_F32 && kv->kv_dtype != PILLAR_BF16 && kv->kv_dtype != PILLAR_FP8_E4M3)
    return PILLAR_EUNSUPPORTED;
  if (kv->kv_dtype == PILLAR_FP8_E4M3 && (!kv->k_scale || !kv->v_scale)) return PILLAR_EINVAL;
  if (!(kv->sm_scale > 0.f) || !(kv->sm_scale < 1e30f)) return PILLAR_EINVAL;
  if (kv->stride_slot < kv->head_dim || kv->stride_head < 1 || kv->stride_page < 1) return PILLAR_EINVAL;
  if (static_cast<int64_t>(kv->max_seq_len) > static_cast<int64_t>(kv->block_table_stride) * kv->page_size)
    return PILLAR_EINVAL;
  if (kv->head_dim != 64 && kv->head_dim != 128) return PILLAR_EUNSUPPORTED;
  if (!pow2(kv->page_size) || kv->page_size > 256) return PILLAR_EUNSUPPORTED;
  if (kv->num_q_heads / kv->num_kv_heads > 16) return PILLAR_EUNSUPPORTED;
  if (kv->flags & ~(PILLAR_FLAG_EXACT_SCORES | PILLAR_FLAG_GENERIC_KERNELS)) return PILLAR_EINVAL;
  return PILLAR_OK;
}

int check_spec(const pillar_kv_t* kv, int spec_len_k) {
  if (spec_len_k < 0) return PILLAR_EINVAL;
  if (spec_len_k > 15) return PILLAR_EUNSUPPORTED;
  if ((spec_len_k + 1) * (kv->num_q_heads / kv->num_kv_heads) > kMaxRows) return PILLAR_EUNSUPPORTED;
  return PILLAR_OK;
}

KvView make_view(const pillar_kv_t* kv) {
  KvView v;
  v.k_pool = kv->k_pool;
  v.v_pool = kv->v_pool;
  v.k_scale = kv->k_scale;
  v.v_scale = kv->v_scale;
  v.block_table = kv->block_table;
  v.seq_lens = kv->seq_lens;
  v.req_ids = nullptr;
  v.stride_page = kv->stride_page;
  v.stride_head = kv->stride_head;
  v.stride_slot = kv->stride_slot;
  v.batch = kv->batch;
  v.num_q_heads = kv->num_q_heads;
  v.num_kv_heads = kv->num_kv_heads;
  v.head_dim = kv->head_dim;
  v.page_size = kv->page_size;
  v.page_shift = __builtin_ctz(static_cast<unsigned>(kv->page_size));
  v.block_table_stride = kv->block_table_stride;
  v.max_seq_len = kv->max_seq_len;
  v.sm_scale = kv->sm_scale;
  return v;
}

int check_workspace(const void* ws, size_t have, size_t need) {
  if (need == 0) return PILLAR_OK;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || have < need) return PILLAR_EWORKSPACE;
  return PILLAR_OK;
}

size_t verify_workspace(const KvView& v, int n_q) {
  const size_t a = verify_generic_workspace(v, n_q);
  size_t b = 0;
  if (v.head_dim == 128 && v.page_size >= 16) {
    b = verify_range_workspace(v, n_q);
  }
  return a > b ? a : b;
}

}  // namespace

Options& options() {
  static Options o;
  return o;
}

}  // namespace pillar

using namespace pillar;

namespace {

// scores for an internal two-step fallback of pillar_verify_select live behind the stage workspaces
size_t scratch_score_stride(const KvView& v) { return (static_cast<size_t>(v.max_seq_len) + 3) / 4 * 4; }
size_t scratch_scores_bytes(const KvView& v) {
  return static_cast<size_t>(v.batch) * v.num_kv_heads * scratch_score_stride(v) * sizeof(float);
}

size_t draft_region_offset(const KvView& v, int n_q) {
  return align_up(align_up(verify_workspace(v, n_q), 256) + scratch_scores_bytes(v), 256);
}

// req_ids / n_req (optional): the call covers only these requests (device list of request indices); draft (optional): one
// draft step of other requests to run in the same grid where the kernels allow it, else right after.
int verify_common(const pillar_kv_t* kv, const void* q, int32_t spec_len_k, const int32_t* spec_lens, void* out, float* lse,
                  float* scores, int64_t score_stride, const SelectOut* select, void* workspace, size_t workspace_bytes,
                  void* hip_stream, const int32_t* req_ids = nullptr, int32_t n_req = 0, const DecodeArgs* draft = nullptr) {
  int rc = check_kv(kv);
  if (rc != PILLAR_OK) return rc;
  rc = check_spec(kv, spec_len_k);
  if (rc != PILLAR_OK) return rc;
  if (!q || !out) return PILLAR_EINVAL;
  if (scores && score_stride < kv->max_seq_len) return PILLAR_EINVAL;
  VerifyArgs a;
  a.kv = make_view(kv);
  if (req_ids) {
    a.kv.req_ids = req_ids;
    a.kv.batch = n_req;
  }
  a.q = q;
  a.out = out;
  a.lse = lse;
  a.scores = scores;
  a.score_stride = score_stride;
  a.n_q = spec_len_k + 1;
  a.q_dtype = kv->q_dtype;
  a.kv_dtype = kv->kv_dtype;
  a.workspace = workspace;
  a.select = select;
  a.spec_lens = spec_lens;
  a.exact_scores = (kv->flags & PILLAR_FLAG_EXACT_SCORES) != 0;
  const bool generic = (kv->flags & PILLAR_FLAG_GENERIC_KERNELS) != 0;
  // per-request speculative lengths exist in the matrix-core single-pass kernels only
  if (spec_lens && (generic || !verify_range_supported(a))) return PILLAR_EUNSUPPORTED;
  const size_t stage_ws = verify_workspace(a.kv, a.n_q);
  rc = check_workspace(workspace, workspace_bytes, stage_ws + (select ? scratch_scores_bytes(a.kv) : 0));
  if (rc != PILLAR_OK) return rc;
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (select) {                                  // long rows pass the statistic between workgroups through memory
    a.scratch_scores = reinterpret_cast<float*>(static_cast<char*>(workspace) + align_up(stage_ws, 256));
    a.scratch_stride = static_cast<int64_t>(scratch_score_stride(a.kv));
  }
  if (select && !(!generic && verify_select_fused(a))) {
    // two steps: the statistic goes through memory (the caller's buffer, or scratch behind the stage workspace)
    if (req_ids) return PILLAR_EUNSUPPORTED;      // (the stand-alone Top-K kernel knows no request lists)
    a.select = nullptr;
    if (!a.scores) {
      a.scores = reinterpret_cast<float*>(static_cast<char*>(workspace) + align_up(stage_ws, 256));
      a.score_stride = static_cast<int64_t>(scratch_score_stride(a.kv));
    }
    const hipError_t e1 = (!generic && verify_range_supported(a)) ? launch_verify_range(a, st) : launch_verify_generic(a, st);
    if (e1 != hipSuccess) return PILLAR_EHIP;
    TopkArgs t;
    t.scores = a.scores;
    t.score_stride = a.score_stride;
    t.seq_lens = a.kv.seq_lens;
    t.budgets = select->budgets;
    t.batch = a.kv.batch;
    t.num_kv_heads = a.kv.num_kv_heads;
    t.max_seq_len = a.kv.max_seq_len;
    t.max_budget = select->max_budget;
    t.indices = select->indices;
    t.counts = select->counts;
    return launch_topk(t, st) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
  }
  hipError_t e;
  if (!generic && verify_range_supported(a)) {
    if (draft && verify_fuses_draft(a)) return launch_verify_range(a, st, draft) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
    e = launch_verify_range(a, st);
  } else {
    e = launch_verify_generic(a, st);
  }
  if (e != hipSuccess) return PILLAR_EHIP;
  if (draft) e = launch_decode_mfma(*draft, st);
  return e == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
}

}  // namespace

extern "C" {

int pillar_version(void) { return 100; }

const char* pillar_status_string(int status) {
  switch (status) {
    case PILLAR_OK: return "ok";
    case PILLAR_EINVAL: return "invalid argument (null pointer, non-positive size or inconsistent shapes)";
    case PILLAR_EUNSUPPORTED: return "shape or dtype outside the supported set";
    case PILLAR_EWORKSPACE: return "workspace null, not 256-byte aligned, or too small";
    case PILLAR_EHIP: return "HIP runtime error at launch";
    case PILLAR_ETOOLARGE: return "the problem needs more scratch than the library's own 32 MiB array holds: use the entry point that takes a workspace";
    default: return "unknown status";
  }
}

size_t pillar_workspace_bytes(const pillar_kv_t* kv, int32_t spec_len_k, int32_t max_budget) {
  if (check_kv(kv) != PILLAR_OK || check_spec(kv, spec_len_k) != PILLAR_OK || max_budget < 0) return 0;
  const KvView v = make_view(kv);
  // [verification | scores of pillar_verify_select's two-step fallback | draft partials]: the draft region is its
  // own so that a unified batch (pillar_mixed_step) can run both at once
  const size_t need = draft_region_offset(v, spec_len_k + 1) + ((v.head_dim == 128) ? decode_mfma_workspace(v, max_budget) : 0);
  return need < 256 ? 256 : need;
}

int pillar_verify_attn(const pillar_kv_t* kv, const void* q, int32_t spec_len_k, void* out, float* lse,
                       float* scores, int64_t score_stride, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  return verify_common(kv, q, spec_len_k, nullptr, out, lse, scores, score_stride, nullptr, workspace, workspace_bytes, hip_stream);
}

int pillar_verify_select(const pillar_kv_t* kv, const void* q, int32_t spec_len_k, void* out, float* lse,
                         float* scores, int64_t score_stride, const int32_t* budgets, int32_t max_budget,
                         int32_t* indices, int32_t* counts, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  if (!budgets || !indices || !counts || max_budget < 1) return PILLAR_EINVAL;
  SelectOut sel;
  sel.budgets = budgets;
  sel.max_budget = max_budget;
  sel.indices = indices;
  sel.counts = counts;
  return verify_common(kv, q, spec_len_k, nullptr, out, lse, scores, score_stride, &sel, workspace, workspace_bytes, hip_stream);
}

int pillar_verify_hetero(const pillar_kv_t* kv, const void* q, int32_t spec_len_max, const int32_t* spec_lens, void* out,
                         float* lse, float* scores, int64_t score_stride, const int32_t* budgets, int32_t max_budget,
                         int32_t* indices, int32_t* counts, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!spec_lens) return PILLAR_EINVAL;
  const bool want_select = budgets || indices || counts;
  if (want_select && (!budgets || !indices || !counts || max_budget < 1)) return PILLAR_EINVAL;
  SelectOut sel;
  sel.budgets = budgets;
  sel.max_budget = max_budget;
  sel.indices = indices;
  sel.counts = counts;
  return verify_common(kv, q, spec_len_max, spec_lens, out, lse, scores, score_stride, want_select ? &sel : nullptr, workspace,
                       workspace_bytes, hip_stream);
}

int pillar_select_topk(const float* scores, int64_t score_stride, const int32_t* seq_lens, const int32_t* budgets,
                       int32_t batch, int32_t num_kv_heads, int32_t max_seq_len, int32_t max_budget,
                       int32_t* indices, int32_t* counts, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  if (!scores || !seq_lens || !budgets || !indices || !counts) return PILLAR_EINVAL;
  if (batch < 1 || num_kv_heads < 1 || max_seq_len < 1 || max_budget < 1) return PILLAR_EINVAL;
  if (score_stride < max_seq_len) return PILLAR_EINVAL;
  TopkArgs a;
  a.scores = scores;
  a.score_stride = score_stride;
  a.seq_lens = seq_lens;
  a.budgets = budgets;
  a.batch = batch;
  a.num_kv_heads = num_kv_heads;
  a.max_seq_len = max_seq_len;
  a.max_budget = max_budget;
  a.indices = indices;
  a.counts = counts;
  const hipError_t e = launch_topk(a, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
}

int pillar_sparse_decode(const pillar_kv_t* kv, const void* q, const int32_t* indices, const int32_t* counts,
                         int32_t max_budget, void* out, float* lse, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  int rc = check_kv(kv);
  if (rc != PILLAR_OK) return rc;
  if (!q || !indices || !counts || !out) return PILLAR_EINVAL;
  if (max_budget < 1) return PILLAR_EINVAL;
  DecodeArgs a;
  a.kv = make_view(kv);
  a.q = q;
  a.indices = indices;
  a.counts = counts;
  a.max_budget = max_budget;
  a.out = out;
  a.lse = lse;
  a.q_dtype = kv->q_dtype;
  a.kv_dtype = kv->kv_dtype;
  a.workspace = workspace;
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (!(kv->flags & PILLAR_FLAG_GENERIC_KERNELS) && decode_mfma_supported(a)) {
    rc = check_workspace(workspace, workspace_bytes, decode_mfma_workspace(a.kv, max_budget));
    if (rc != PILLAR_OK) return rc;
    return launch_decode_mfma(a, st) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
  }
  return launch_decode_generic(a, st) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
}

int pillar_mixed_step(const pillar_kv_t* kv, const int32_t* verify_ids, int32_t n_verify, const int32_t* draft_ids,
                      int32_t n_draft, const void* q_verify, int32_t spec_len_k, void* out_verify, float* lse_verify,
                      float* scores, int64_t score_stride, const int32_t* budgets, int32_t max_budget, int32_t* indices,
                      int32_t* counts, const void* q_draft, void* out_draft, float* lse_draft, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  int rc = check_kv(kv);
  if (rc != PILLAR_OK) return rc;
  rc = check_spec(kv, spec_len_k);
  if (rc != PILLAR_OK) return rc;
  if (n_verify < 0 || n_draft < 0 || n_verify > kv->batch || n_draft > kv->batch) return PILLAR_EINVAL;
  if ((n_verify > 0 && (!verify_ids || !q_verify || !out_verify)) || (n_draft > 0 && (!draft_ids || !q_draft || !out_draft)))
    return PILLAR_EINVAL;
  if (!budgets || !indices || !counts || max_budget < 1) return PILLAR_EINVAL;
  if (kv->flags != 0) return PILLAR_EUNSUPPORTED;            // matrix-core kernels, default statistic only
  const KvView full = make_view(kv);
  const size_t dec_off = draft_region_offset(full, spec_len_k + 1);
  rc = check_workspace(workspace, workspace_bytes, dec_off + decode_mfma_workspace(full, max_budget));
  if (rc != PILLAR_OK) return rc;
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  DecodeArgs d;
  d.kv = full;
  d.kv.req_ids = draft_ids;
  d.kv.batch = n_draft;
  d.q = q_draft;
  d.indices = indices;
  d.counts = counts;
  d.max_budget = max_budget;
  d.out = out_draft;
  d.lse = lse_draft;
  d.q_dtype = kv->q_dtype;
  d.kv_dtype = kv->kv_dtype;
  d.workspace = static_cast<char*>(workspace) + dec_off;
  if (n_draft > 0 && !decode_mfma_supported(d)) return PILLAR_EUNSUPPORTED;
  if (n_verify == 0) {
    if (n_draft == 0) return PILLAR_OK;
    return launch_decode_mfma(d, st) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
  }
  {
    VerifyArgs probe;                            // the shapes the matrix-core verification takes
    probe.kv = full;
    probe.q = q_verify;
    probe.out = out_verify;
    probe.lse = lse_verify;
    probe.scores = scores;
    probe.score_stride = score_stride;
    probe.n_q = spec_len_k + 1;
    probe.q_dtype = kv->q_dtype;
    probe.kv_dtype = kv->kv_dtype;
    probe.workspace = workspace;
    if (!verify_range_supported(probe)) return PILLAR_EUNSUPPORTED;
  }
  SelectOut sel;
  sel.budgets = budgets;
  sel.max_budget = max_budget;
  sel.indices = indices;
  sel.counts = counts;
  return verify_common(kv, q_verify, spec_len_k, nullptr, out_verify, lse_verify, scores, score_stride, &sel, workspace,
                       workspace_bytes, hip_stream, verify_ids, n_verify, n_draft > 0 ? &d : nullptr);
}

int pillar_sparse_decode_static(const pillar_kv_t* kv, const void* q, const int32_t* indices, const int32_t* counts,
                                int32_t max_budget, void* out, float* lse, void* hip_stream) {
  int rc = check_kv(kv);
  if (rc != PILLAR_OK) return rc;
  if (!q || !indices || !counts || !out) return PILLAR_EINVAL;
  if (max_budget < 1) return PILLAR_EINVAL;
  DecodeArgs a;
  a.kv = make_view(kv);
  a.q = q;
  a.indices = indices;
  a.counts = counts;
  a.max_budget = max_budget;
  a.out = out;
  a.lse = lse;
  a.q_dtype = kv->q_dtype;
  a.kv_dtype = kv->kv_dtype;
  a.workspace = nullptr;
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (!(kv->flags & PILLAR_FLAG_GENERIC_KERNELS) && decode_mfma_supported(a)) {
    if (decode_mfma_workspace(a.kv, max_budget) > decode_static_scratch_bytes()) return PILLAR_ETOOLARGE;
    return launch_decode_mfma_static(a, st) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
  }
  return launch_decode_generic(a, st) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;     // needs no scratch at all
}

int pillar_append_kv(const pillar_kv_t* kv, const void* k_new, const void* v_new, int32_t n_new, void* hip_stream) {
  const int rc = check_kv(kv);
  if (rc != PILLAR_OK) return rc;
  if (!k_new || !v_new || n_new < 1) return PILLAR_EINVAL;
  if (kv->kv_dtype == PILLAR_FP8_E4M3) return PILLAR_EUNSUPPORTED;      // the page scales would have to be recomputed
  const int esz = kv->kv_dtype == PILLAR_F32 ? 4 : 2;
  const KvView v = make_view(kv);
  // 16-byte pieces: rows and strides must be multiples of 16 bytes, bases aligned
  if ((v.head_dim * esz) % 16 || (v.stride_page * esz) % 16 || (v.stride_head * esz) % 16 || (v.stride_slot * esz) % 16)
    return PILLAR_EUNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(v.k_pool) | reinterpret_cast<uintptr_t>(v.v_pool) | reinterpret_cast<uintptr_t>(k_new) |
       reinterpret_cast<uintptr_t>(v_new)) & 15u)
    return PILLAR_EUNSUPPORTED;
  return launch_append_kv(v, k_new, v_new, n_new, esz, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
}

int pillar_window_indices(const int32_t* seq_lens, const int32_t* budgets, int32_t batch, int32_t num_kv_heads,
                          int32_t sink_tokens, int32_t max_budget, int32_t* indices, int32_t* counts, void* hip_stream) {
  if (!seq_lens || !budgets || !indices || !counts) return PILLAR_EINVAL;
  if (batch < 1 || num_kv_heads < 1 || max_budget < 1 || sink_tokens < 0) return PILLAR_EINVAL;
  return launch_window_indices(seq_lens, budgets, batch, num_kv_heads, sink_tokens, max_budget, indices, counts,
                               static_cast<hipStream_t>(hip_stream)) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
}

int pillar_extend_indices(int32_t* indices, int32_t* counts, const int32_t* first_new, const int32_t* n_new,
                          int32_t batch, int32_t num_kv_heads, int32_t max_budget, void* hip_stream) {
  if (!indices || !counts || !first_new || !n_new) return PILLAR_EINVAL;
  if (batch < 1 || num_kv_heads < 1 || max_budget < 1) return PILLAR_EINVAL;
  return launch_extend_indices(indices, counts, first_new, n_new, batch, num_kv_heads, max_budget,
                               static_cast<hipStream_t>(hip_stream)) == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
}

int pillar_set_option(const char* name, int64_t value) {
  if (!name || value < 0) return PILLAR_EINVAL;
  Options& o = options();
  const std::string k(name);
  if (k == "verify_waves") {
    if (value > 8) return PILLAR_EINVAL;
    o.verify_waves = static_cast<int>(value);
  } else if (k == "decode_rows") {
    if (value % 32 != 0 || value > 4096) return PILLAR_EINVAL;
    o.decode_rows = static_cast<int>(value);
  } else {
    return PILLAR_EINVAL;
  }
  return PILLAR_OK;
}


void pillar_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (on && !g_pool_made) {
    g_pool_made = true;
    for (size_t i = 0; i < kEventPairs; ++i) {
      hipEvent_t a = nullptr, b = nullptr;
      if (hipEventCreate(&a) != hipSuccess) break;
      if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); break; }
      g_free.emplace_back(a, b);
    }
  }
  g_prof_on = on != 0;
}

void pillar_profile_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  drain_locked();
  g_totals.clear();
}

int pillar_profile_read(pillar_kernel_time* entries, int cap) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  drain_locked();
  int n = 0;
  for (const auto& kvp : g_totals) {
    if (entries && n < cap) {
      std::memset(&entries[n], 0, sizeof(entries[n]));
      std::strncpy(entries[n].name, kvp.first.c_str(), sizeof(entries[n].name) - 1);
      entries[n].launches = kvp.second.first;
      entries[n].total_ms = kvp.second.second;
    }
    ++n;
  }
  return n;
}

}  // extern "C"
