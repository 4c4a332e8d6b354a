// Sparse draft attention, generic path (any supported shape and dtype, fp32
// arithmetic on the vector ALUs).
//
// Paper Sections 1 and 4.2: a draft step loads and attends to the critical
// tokens only; with the KV-Cache addressed row by row ("page size 1") this is
// the same pipeline as full attention, driven by an index list.
//
// One workgroup per (request, KV head) walks the index list in tiles of kTile
// rows with a running (max, sum, output): the textbook online softmax.
#include "launch.hpp"

namespace pillar {
namespace {

constexpr int kTile = 128;
constexpr int kThreads = 256;
constexpr int kMaxG = 16;
constexpr int kMaxD = 128;
constexpr int kAccPerThread = kMaxG * kMaxD / kThreads;   // 8

template <int QDT, int KVDT>
__global__ __launch_bounds__(kThreads) void decode_generic(DecodeArgs a) {
  __shared__ float qs[kMaxG * kMaxD];
  __shared__ float s[kMaxG * kTile];
  __shared__ float row_m[kMaxG], row_l[kMaxG], row_alpha[kMaxG];
  __shared__ int32_t tok[kTile];
  __shared__ int32_t tok_page[kTile];

  const KvView& kv = a.kv;
  const int b = blockIdx.y, g = blockIdx.x;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int D = kv.head_dim;
  const int n = min(max(a.counts[b], 0), a.max_budget);
  const int32_t* list = a.indices + (static_cast<int64_t>(b) * kv.num_kv_heads + g) * a.max_budget;

  for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
    const int r = idx / D, d = idx - r * D;
    qs[idx] = Storage<QDT>::load(a.q, (static_cast<int64_t>(b) * kv.num_q_heads + g * G + r) * D + d);
  }
  if (threadIdx.x < kMaxG) { row_m[threadIdx.x] = -INFINITY; row_l[threadIdx.x] = 0.f; }
  float acc[kAccPerThread];
#pragma unroll
  for (int j = 0; j < kAccPerThread; ++j) acc[j] = 0.f;
  __syncthreads();

  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  for (int j0 = 0; j0 < n; j0 += kTile) {
    const int nj = min(kTile, n - j0);
    for (int jj = threadIdx.x; jj < kTile; jj += kThreads) tok[jj] = jj < nj ? list[j0 + jj] : 0;
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * kTile; idx += kThreads) {
      const int r = idx / kTile, jj = idx - r * kTile;
      float v = -INFINITY;
      if (jj < nj) {
        int page;
        const int64_t off = row_offset(kv, b, g, tok[jj], &page);
        if (r == 0) tok_page[jj] = page;
        const float* qr = qs + r * D;
        float dot = 0.f;
        for (int d = 0; d < D; ++d) dot = fmaf(qr[d], Storage<KVDT>::load(kv.k_pool, off + d), dot);
        if (KVDT == PILLAR_FP8_E4M3) dot *= kv.k_scale[static_cast<int64_t>(page) * kv.num_kv_heads + g];
        v = dot * kv.sm_scale;
      }
      s[idx] = v;
    }
    __syncthreads();
    for (int r = wave; r < G; r += kThreads / kWave) {
      float* sr = s + r * kTile;
      float m = -INFINITY;
      for (int jj = lane; jj < kTile; jj += kWave) m = fmaxf(m, sr[jj]);
      m = fmaxf(wave_max(m), row_m[r]);                 // nj >= 1, so m is finite
      float l = 0.f;
      for (int jj = lane; jj < kTile; jj += kWave) {
        const float p = __expf(sr[jj] - m);             // exp(-inf) = 0 for the padding
        sr[jj] = p;
        l += p;
      }
      l = wave_sum(l);
      if (lane == 0) {
        const float alpha = (row_m[r] == -INFINITY) ? 0.f : __expf(row_m[r] - m);
        row_alpha[r] = alpha;
        row_l[r] = row_l[r] * alpha + l;
        row_m[r] = m;
      }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kAccPerThread; ++j) {
      const int idx = threadIdx.x + j * kThreads;
      if (idx < G * D) {
        const int r = idx / D, d = idx - r * D;
        const float* pr = s + r * kTile;
        float o = acc[j] * row_alpha[r];
        for (int jj = 0; jj < nj; ++jj) {
          const int t = tok[jj];
          const int page = tok_page[jj];
          const int64_t off = static_cast<int64_t>(page) * kv.stride_page + static_cast<int64_t>(g) * kv.stride_head +
                              static_cast<int64_t>(t & (kv.page_size - 1)) * kv.stride_slot;
          float v = Storage<KVDT>::load(kv.v_pool, off + d);
          if (KVDT == PILLAR_FP8_E4M3) v *= kv.v_scale[static_cast<int64_t>(page) * kv.num_kv_heads + g];
          o = fmaf(pr[jj], v, o);
        }
        acc[j] = o;
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < kAccPerThread; ++j) {
    const int idx = threadIdx.x + j * kThreads;
    if (idx < G * D) {
      const int r = idx / D, d = idx - r * D;
      const int64_t row = static_cast<int64_t>(b) * kv.num_q_heads + g * G + r;
      const float l = row_l[r];
      Storage<QDT>::store(a.out, row * D + d, n > 0 ? acc[j] / l : 0.f);
      if (d == 0 && a.lse) a.lse[row] = n > 0 ? row_m[r] + __logf(l) : -INFINITY;
    }
  }
}

}  // namespace

hipError_t launch_decode_generic(const DecodeArgs& a, hipStream_t s) {
  const dim3 grid(a.kv.num_kv_heads, a.kv.batch);
  KernelTimer t("decode_generic", s);
#define PILLAR_CASE(Q, K)                                                            \
  if (a.q_dtype == Q && a.kv_dtype == K) {                                           \
    hipLaunchKernelGGL((decode_generic<Q, K>), grid, dim3(kThreads), 0, s, a);       \
    return hipGetLastError();                                                        \
  }
  PILLAR_CASE(PILLAR_F32, PILLAR_F32)
  PILLAR_CASE(PILLAR_F32, PILLAR_BF16)
  PILLAR_CASE(PILLAR_F32, PILLAR_FP8_E4M3)
  PILLAR_CASE(PILLAR_BF16, PILLAR_F32)
  PILLAR_CASE(PILLAR_BF16, PILLAR_BF16)
  PILLAR_CASE(PILLAR_BF16, PILLAR_FP8_E4M3)
#undef PILLAR_CASE
  return hipErrorInvalidValue;
}

}  // namespace pillar
