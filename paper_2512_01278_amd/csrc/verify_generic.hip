// Verification attention, generic path: any supported shape and dtype, fp32
// arithmetic on the vector ALUs.  Correct everywhere, fast nowhere: it serves
// the shapes the MFMA path does not cover (fp32 tensors, head_dim 64) and is
// the in-library cross-check of that path.
//
// Paper Section 4.1: the k+1 verification rows attend to the whole KV-Cache;
// the softmax probabilities, averaged over those rows and the query heads of
// one GQA group, are the score statistic that Top-K later reads.
//
// Three launches:
//   split   one workgroup per (request, KV head, chunk of kChunk tokens):
//           logits of all R=(k+1)*G rows against the chunk, chunk-local
//           softmax, partial output -> workspace
//   merge   one workgroup per (request, KV head): combines the partials by
//           their log-sum-exp, writes out and lse
//   scores  same grid as split: logits again, now against the final lse:
//           exp(s - lse) is the exact softmax probability; mean over rows
#include "launch.hpp"

namespace pillar {
namespace {

constexpr int kChunk = 128;     // tokens per workgroup
constexpr int kThreads = 256;

struct GenericWs {
  float* part_m;   // [B][Hkv][NC][R]
  float* part_l;   // [B][Hkv][NC][R]
  float* part_o;   // [B][Hkv][NC][R][D]
  float* lse;      // [B][Hkv][R]  natural log
  int nc;
};

__host__ __device__ inline int num_chunks(int max_seq_len) { return (max_seq_len + kChunk - 1) / kChunk; }

// Logits of rows r<R against tokens t0..t0+kChunk-1 of (b, g) into s[r][tt]
// (sm_scale applied, -inf where masked or beyond the sequence).  q rows are
// staged in qs[R][D] first.
template <int QDT, int KVDT>
__device__ void logits_tile(const KvView& kv, const void* q, int n_q, int b, int g, int t0, int L,
                            float* qs, float* s) {
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int D = kv.head_dim;
  for (int idx = threadIdx.x; idx < R * D; idx += kThreads) {
    const int r = idx / D, d = idx - r * D;
    const int i = r / G, hg = r - i * G;
    const int64_t off = ((static_cast<int64_t>(b) * n_q + i) * kv.num_q_heads + g * G + hg) * D + d;
    qs[idx] = Storage<QDT>::load(q, off);
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < R * kChunk; idx += kThreads) {
    const int r = idx / kChunk, tt = idx - r * kChunk;
    const int i = r / G;
    const int t = t0 + tt;
    float v = -INFINITY;
    if (t < L && t <= L - n_q + i) {
      int page;
      const int64_t off = row_offset(kv, b, g, t, &page);
      float acc = 0.f;
      const float* qr = qs + r * D;
      for (int d = 0; d < D; ++d) acc = fmaf(qr[d], Storage<KVDT>::load(kv.k_pool, off + d), acc);
      if (KVDT == PILLAR_FP8_E4M3) acc *= kv.k_scale[static_cast<int64_t>(page) * kv.num_kv_heads + g];
      v = acc * kv.sm_scale;
    }
    s[idx] = v;
  }
  __syncthreads();
}

template <int QDT, int KVDT>
__global__ __launch_bounds__(kThreads) void verify_split_generic(KvView kv, const void* q, int n_q, GenericWs ws) {
  extern __shared__ float smem[];
  const int b = blockIdx.z, g = blockIdx.y, c = blockIdx.x;
  const int L = kv.seq_lens[b];
  const int t0 = c * kChunk;
  if (t0 >= L) return;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int D = kv.head_dim;
  float* qs = smem;                  // [R][D]
  float* s = smem + R * D;           // [R][kChunk]
  logits_tile<QDT, KVDT>(kv, q, n_q, b, g, t0, L, qs, s);

  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t slot = (static_cast<int64_t>(b) * kv.num_kv_heads + g) * ws.nc + c;
  for (int r = wave; r < R; r += kThreads / kWave) {
    float* sr = s + r * kChunk;
    float m = -INFINITY;
    for (int tt = lane; tt < kChunk; tt += kWave) m = fmaxf(m, sr[tt]);
    m = wave_max(m);
    float l = 0.f;
    for (int tt = lane; tt < kChunk; tt += kWave) {
      const float p = (m == -INFINITY) ? 0.f : __expf(sr[tt] - m);
      sr[tt] = p;
      l += p;
    }
    l = wave_sum(l);
    if (lane == 0) {
      ws.part_m[slot * R + r] = m;
      ws.part_l[slot * R + r] = l;
    }
  }
  __syncthreads();
  const int nt = min(kChunk, L - t0);
  for (int idx = threadIdx.x; idx < R * D; idx += kThreads) {
    const int r = idx / D, d = idx - r * D;
    const float* pr = s + r * kChunk;
    float acc = 0.f;
    for (int tt = 0; tt < nt; ++tt) {
      int page;
      const int64_t off = row_offset(kv, b, g, t0 + tt, &page);
      float v = Storage<KVDT>::load(kv.v_pool, off + d);
      if (KVDT == PILLAR_FP8_E4M3) v *= kv.v_scale[static_cast<int64_t>(page) * kv.num_kv_heads + g];
      acc = fmaf(pr[tt], v, acc);
    }
    ws.part_o[(slot * R + r) * D + d] = acc;
  }
}

template <int QDT>
__global__ __launch_bounds__(kThreads) void verify_merge_generic(KvView kv, int n_q, GenericWs ws, void* out,
                                                                  float* lse_out) {
  const int b = blockIdx.y, g = blockIdx.x;
  const int L = kv.seq_lens[b];
  const int nc = (L + kChunk - 1) / kChunk;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int D = kv.head_dim;
  const int64_t base = (static_cast<int64_t>(b) * kv.num_kv_heads + g) * ws.nc;
  for (int idx = threadIdx.x; idx < R * D; idx += kThreads) {
    const int r = idx / D, d = idx - r * D;
    float m = -INFINITY;
    for (int c = 0; c < nc; ++c) m = fmaxf(m, ws.part_m[(base + c) * R + r]);
    float l = 0.f, o = 0.f;
    for (int c = 0; c < nc; ++c) {
      const float mc = ws.part_m[(base + c) * R + r];
      const float w = (mc == -INFINITY) ? 0.f : __expf(mc - m);
      l = fmaf(ws.part_l[(base + c) * R + r], w, l);
      o = fmaf(ws.part_o[((base + c) * R + r) * D + d], w, o);
    }
    const int i = r / G, hg = r - i * G;
    const int64_t row = (static_cast<int64_t>(b) * n_q + i) * kv.num_q_heads + g * G + hg;
    const bool live = l > 0.f;                 // false for a row that sees no token at all: zeros, lse = -inf
    Storage<QDT>::store(out, row * D + d, live ? o / l : 0.f);
    if (d == 0) {
      const float v = m + __logf(l);
      ws.lse[(static_cast<int64_t>(b) * kv.num_kv_heads + g) * R + r] = live ? v : INFINITY;   // +inf: no weight in the statistic
      if (lse_out) lse_out[row] = live ? v : -INFINITY;
    }
  }
}

template <int QDT, int KVDT>
__global__ __launch_bounds__(kThreads) void verify_scores_generic(KvView kv, const void* q, int n_q, GenericWs ws,
                                                                   float* scores, int64_t score_stride) {
  extern __shared__ float smem[];
  const int b = blockIdx.z, g = blockIdx.y, c = blockIdx.x;
  const int L = kv.seq_lens[b];
  const int t0 = c * kChunk;
  if (t0 >= L) return;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int D = kv.head_dim;
  float* qs = smem;
  float* s = smem + R * D;
  logits_tile<QDT, KVDT>(kv, q, n_q, b, g, t0, L, qs, s);
  const float* lse = ws.lse + (static_cast<int64_t>(b) * kv.num_kv_heads + g) * R;
  const float inv_r = 1.0f / static_cast<float>(R);
  for (int tt = threadIdx.x; tt < kChunk; tt += kThreads) {
    if (t0 + tt >= L) continue;
    float acc = 0.f;
    for (int r = 0; r < R; ++r) {
      const float v = s[r * kChunk + tt];
      acc += (v == -INFINITY) ? 0.f : __expf(v - lse[r]);
    }
    scores[(static_cast<int64_t>(b) * kv.num_kv_heads + g) * score_stride + t0 + tt] = acc * inv_r;
  }
}

GenericWs carve(const KvView& kv, int n_q, void* workspace) {
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const size_t R = static_cast<size_t>(n_q) * G;
  const size_t nc = num_chunks(kv.max_seq_len);
  const size_t pairs = static_cast<size_t>(kv.batch) * kv.num_kv_heads;
  char* p = static_cast<char*>(workspace);
  GenericWs w;
  w.nc = static_cast<int>(nc);
  w.part_m = reinterpret_cast<float*>(p); p += align_up(pairs * nc * R * 4, 256);
  w.part_l = reinterpret_cast<float*>(p); p += align_up(pairs * nc * R * 4, 256);
  w.part_o = reinterpret_cast<float*>(p); p += align_up(pairs * nc * R * kv.head_dim * 4, 256);
  w.lse = reinterpret_cast<float*>(p);
  return w;
}

template <int QDT, int KVDT>
hipError_t run(const VerifyArgs& a, hipStream_t st) {
  const KvView& kv = a.kv;
  const GenericWs ws = carve(kv, a.n_q, a.workspace);
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = a.n_q * G;
  const size_t smem = (static_cast<size_t>(R) * kv.head_dim + static_cast<size_t>(R) * kChunk) * sizeof(float);
  const dim3 grid(ws.nc, kv.num_kv_heads, kv.batch);
  {
    KernelTimer t("verify_split_generic", st);
    hipLaunchKernelGGL((verify_split_generic<QDT, KVDT>), grid, dim3(kThreads), smem, st, kv, a.q, a.n_q, ws);
  }
  {
    KernelTimer t("verify_merge_generic", st);
    hipLaunchKernelGGL((verify_merge_generic<QDT>), dim3(kv.num_kv_heads, kv.batch), dim3(kThreads), 0, st, kv,
                       a.n_q, ws, a.out, a.lse);
  }
  if (a.scores) {
    KernelTimer t("verify_scores_generic", st);
    hipLaunchKernelGGL((verify_scores_generic<QDT, KVDT>), grid, dim3(kThreads), smem, st, kv, a.q, a.n_q, ws,
                       a.scores, a.score_stride);
  }
  return hipGetLastError();
}

}  // namespace

size_t verify_generic_workspace(const KvView& kv, int n_q) {
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const size_t R = static_cast<size_t>(n_q) * G;
  const size_t nc = num_chunks(kv.max_seq_len);
  const size_t pairs = static_cast<size_t>(kv.batch) * kv.num_kv_heads;
  return 2 * align_up(pairs * nc * R * 4, 256) + align_up(pairs * nc * R * kv.head_dim * 4, 256) +
         align_up(pairs * R * 4, 256);
}

hipError_t launch_verify_generic(const VerifyArgs& a, hipStream_t s) {
#define PILLAR_CASE(Q, K) \
  if (a.q_dtype == Q && a.kv_dtype == K) return run<Q, K>(a, s);
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
