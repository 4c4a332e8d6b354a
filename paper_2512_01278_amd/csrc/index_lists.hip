// Index lists that do not come from attention scores, for the same sparse
// draft kernel (paper Section 4.2: with page size 1 any token set is a list).
//
//   window   the static "attention sinks + recent window" pattern of the
//            sliding-window drafts the paper compares against (Sections 1, 3.3, 5.2):
//            the first `sink_tokens` positions and the most recent ones;
//   extend   tokens generated after the last verification have no score yet,
//            but a draft step must see them: their positions are appended to
//            every head's list.
// And the write that precedes a verification: the K/V rows of the newest
// tokens go into their pages (append, then attend).
#include "launch.hpp"

namespace pillar {
namespace {

constexpr int kThreads = 256;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kThreads) void window_indices(const int32_t* seq_lens, const int32_t* budgets, int num_kv_heads,
                                                           int sink_tokens, int max_budget, int32_t* indices, int32_t* counts) {
  const int b = blockIdx.y, g = blockIdx.x;
  const int L = seq_lens[b];
  const int K = max(0, min(min(budgets[b], L), max_budget));
  const int ns = min(sink_tokens, K);
  int32_t* out = indices + (static_cast<int64_t>(b) * num_kv_heads + g) * max_budget;
  if (g == 0 && threadIdx.x == 0) counts[b] = K;
  for (int j = threadIdx.x; j < max_budget; j += kThreads) out[j] = j < ns ? j : (j < K ? L - K + j : -1);
}

// one workgroup per request: it reads the old count before anybody overwrites it
__global__ __launch_bounds__(kThreads) void extend_indices(int32_t* indices, int32_t* counts, const int32_t* first_new,
                                                           const int32_t* n_new, int num_kv_heads, int max_budget) {
  const int b = blockIdx.x;
  const int c = min(max(counts[b], 0), max_budget);
  const int n = max(0, min(n_new[b], max_budget - c));
  const int first = first_new[b];
  __syncthreads();
  for (int e = threadIdx.x; e < num_kv_heads * n; e += kThreads) {
    const int g = e / n, j = e - g * n;
    indices[(static_cast<int64_t>(b) * num_kv_heads + g) * max_budget + c + j] = first + j;
  }
  if (threadIdx.x == 0) counts[b] = c + n;
}

// one workgroup per (request, new token): its Hkv rows of K and of V, 16 bytes per thread and step
__global__ __launch_bounds__(kThreads) void append_kv(KvView kv, const uint8_t* k_new, const uint8_t* v_new, int n_new, int esz) {
  const int b = blockIdx.y, i = blockIdx.x;
  const int pos = kv.seq_lens[b] - n_new + i;
  if (pos < 0) return;
  const int page = kv.block_table[static_cast<int64_t>(b) * kv.block_table_stride + (pos >> kv.page_shift)];
  const int slot = pos & (kv.page_size - 1);
  const int row_bytes = kv.head_dim * esz;                       // a multiple of 16
  const int chunks = row_bytes / 16;
  uint8_t* kp = static_cast<uint8_t*>(const_cast<void*>(kv.k_pool));
  uint8_t* vp = static_cast<uint8_t*>(const_cast<void*>(kv.v_pool));
  for (int e = threadIdx.x; e < kv.num_kv_heads * chunks; e += kThreads) {
    const int g = e / chunks, c = e - g * chunks;
    const int64_t src = ((static_cast<int64_t>(b) * n_new + i) * kv.num_kv_heads + g) * row_bytes + 16 * c;
    const int64_t dst = (static_cast<int64_t>(page) * kv.stride_page + static_cast<int64_t>(g) * kv.stride_head +
                         static_cast<int64_t>(slot) * kv.stride_slot) * esz + 16 * c;
    *reinterpret_cast<u32x4*>(kp + dst) = *reinterpret_cast<const u32x4*>(k_new + src);
    *reinterpret_cast<u32x4*>(vp + dst) = *reinterpret_cast<const u32x4*>(v_new + src);
  }
}

}  // namespace

hipError_t launch_append_kv(const KvView& kv, const void* k_new, const void* v_new, int n_new, int esz, hipStream_t s) {
  KernelTimer t("append_kv", s);
  hipLaunchKernelGGL(append_kv, dim3(n_new, kv.batch), dim3(kThreads), 0, s, kv, static_cast<const uint8_t*>(k_new),
                     static_cast<const uint8_t*>(v_new), n_new, esz);
  return hipGetLastError();
}

hipError_t launch_window_indices(const int32_t* seq_lens, const int32_t* budgets, int batch, int num_kv_heads, int sink_tokens,
                                 int max_budget, int32_t* indices, int32_t* counts, hipStream_t s) {
  KernelTimer t("window_indices", s);
  hipLaunchKernelGGL(window_indices, dim3(num_kv_heads, batch), dim3(kThreads), 0, s, seq_lens, budgets, num_kv_heads, sink_tokens,
                     max_budget, indices, counts);
  return hipGetLastError();
}

hipError_t launch_extend_indices(int32_t* indices, int32_t* counts, const int32_t* first_new, const int32_t* n_new, int batch,
                                 int num_kv_heads, int max_budget, hipStream_t s) {
  KernelTimer t("extend_indices", s);
  hipLaunchKernelGGL(extend_indices, dim3(batch), dim3(kThreads), 0, s, indices, counts, first_new, n_new, num_kv_heads, max_budget);
  return hipGetLastError();
}

}  // namespace pillar
