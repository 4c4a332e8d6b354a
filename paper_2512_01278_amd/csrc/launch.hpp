// Host-side interfaces between the C ABI (pillar_api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "common.hpp"

namespace pillar {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Brackets one kernel launch with HIP events when profiling is switched on.
struct KernelTimer {
  KernelTimer(const char* name, hipStream_t stream);
  ~KernelTimer();
  const char* name_;
  hipStream_t stream_;
  hipEvent_t start_ = nullptr, stop_ = nullptr;
};

// where a fused verification + selection leaves the critical tokens
struct SelectOut {
  const int32_t* budgets;
  int32_t max_budget;
  int32_t* indices;
  int32_t* counts;
};

struct VerifyArgs {
  KvView kv;
  const void* q;
  void* out;
  float* lse;            // may be null
  float* scores;         // may be null
  int64_t score_stride;
  int32_t n_q;           // k+1
  int32_t q_dtype, kv_dtype;
  void* workspace;
  const SelectOut* select = nullptr;   // non-null: also select the Top-K of every (request, KV head)
  bool exact_scores = false;           // PILLAR_FLAG_EXACT_SCORES: K read twice, fp32 probabilities
  const int32_t* spec_lens = nullptr;  // non-null: device [B], request b speculates spec_lens[b] <= n_q - 1 tokens
  float* scratch_scores = nullptr;     // with select: room for the statistic ([slots][Hkv][scratch_stride]) if scores is null
  int64_t scratch_stride = 0;
};

struct DecodeArgs {
  KvView kv;
  const void* q;
  const int32_t* indices;
  const int32_t* counts;
  int32_t max_budget;
  void* out;
  float* lse;            // may be null
  int32_t q_dtype, kv_dtype;
  void* workspace;
};

// split partials of the draft step (decode_mfma.hip carves them out of the workspace)
struct DecWs {
  float* part_m;   // [B][Hkv][nsplit][16]  log2 domain
  float* part_l;   // [B][Hkv][nsplit][16]
  float* part_o;   // [B][Hkv][nsplit][G][128]
};

struct TopkArgs {
  const float* scores;
  int64_t score_stride;
  const int32_t* seq_lens;
  const int32_t* budgets;
  int32_t batch, num_kv_heads, max_seq_len, max_budget;
  int32_t* indices;
  int32_t* counts;
};

// generic (any supported shape, fp32 arithmetic on the vector ALUs)
size_t verify_generic_workspace(const KvView& kv, int n_q);
hipError_t launch_verify_generic(const VerifyArgs& a, hipStream_t s);
hipError_t launch_decode_generic(const DecodeArgs& a, hipStream_t s);
hipError_t launch_topk(const TopkArgs& a, hipStream_t s);
hipError_t launch_append_kv(const KvView& kv, const void* k_new, const void* v_new, int n_new, int esz, hipStream_t s);
hipError_t launch_window_indices(const int32_t* seq_lens, const int32_t* budgets, int batch, int num_kv_heads, int sink_tokens,
                                 int max_budget, int32_t* indices, int32_t* counts, hipStream_t s);
hipError_t launch_extend_indices(int32_t* indices, int32_t* counts, const int32_t* first_new, const int32_t* n_new, int batch,
                                 int num_kv_heads, int max_budget, hipStream_t s);

// matrix-core paths (bf16 queries, bf16 / fp8 KV, head_dim 128, pages >= 16)
bool verify_range_supported(const VerifyArgs& a);
size_t verify_range_workspace(const KvView& kv, int n_q);
// `fused_draft` (optional): one draft step of other requests that shares the grid of the streaming pass; only
// where verify_fuses_draft(a) holds.  The caller still owes nothing: the draft's merge launch is included.
hipError_t launch_verify_range(const VerifyArgs& a, hipStream_t s, const DecodeArgs* fused_draft = nullptr);
bool verify_fuses_draft(const VerifyArgs& a);
bool verify_select_fused(const VerifyArgs& a);          // a.select can be served by the finish kernel itself
bool decode_mfma_supported(const DecodeArgs& a);
size_t decode_mfma_workspace(const KvView& kv, int max_budget);
hipError_t launch_decode_mfma(const DecodeArgs& a, hipStream_t s);
int decode_span_rows(const KvView& kv, int max_budget);   // rows of an index list one workgroup takes
DecWs decode_carve(const KvView& kv, int max_budget, void* workspace);
hipError_t launch_decode_merge(const DecodeArgs& a, hipStream_t s);          // combines the spans of lists longer than one
size_t decode_static_scratch_bytes();                     // size of the library's own scratch array
hipError_t launch_decode_mfma_static(const DecodeArgs& a, hipStream_t s);   // same kernels, partials in that array

// process-wide tuning knobs (pillar_set_option); 0 = default
struct Options {
  int verify_waves = 0;   // wavefronts per compute unit of the two verification passes
  int decode_rows = 0;    // rows of the index list per workgroup of the draft kernel
};
Options& options();

}  // namespace pillar
