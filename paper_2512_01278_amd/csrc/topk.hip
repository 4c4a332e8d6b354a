// Critical-token selection: Top-K of the averaged verification scores per
// (request, KV head) -- paper Section 4.1.
//
// Exact radix select.  A float's bit pattern, mapped to an unsigned key whose
// integer order is the float order, is resolved 8 bits at a time from the top:
// each pass histograms one digit of the keys that still match the prefix found
// so far and picks the digit that contains the K-th largest key.  After four
// passes the prefix IS the K-th largest key T.  One ordered sweep then emits,
// in ascending position, every key > T and the first (K - #greater) keys == T:
// equal scores go to the lower position, and the list comes out sorted by
// position, which is what the draft kernel's gather likes.
//
// One workgroup of 1024 threads per (request, KV head); the score row (at most
// 128 KiB) is read from L2 on every pass.  Bit-exact and deterministic: the
// only atomics are integer histogram increments.
#include "launch.hpp"
#include "topk_core.hpp"

namespace pillar {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWave;


__global__ __launch_bounds__(kThreads) void topk_radix(TopkArgs a) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix, sh_remaining;
  __shared__ uint32_t wave_tot[2][kWaves];
  __shared__ uint32_t sh_base_sel, sh_base_eq;

  const int b = blockIdx.y, g = blockIdx.x;
  const int L = a.seq_lens[b];
  const int K = max(0, min(min(a.budgets[b], L), a.max_budget));
  int32_t* out = a.indices + (static_cast<int64_t>(b) * a.num_kv_heads + g) * a.max_budget;
  if (g == 0 && threadIdx.x == 0) a.counts[b] = K;
  for (int j = K + threadIdx.x; j < a.max_budget; j += kThreads) out[j] = -1;
  if (K == 0) return;
  const float* row = a.scores + (static_cast<int64_t>(b) * a.num_kv_heads + g) * a.score_stride;

  uint32_t prefix = 0, remaining = K;      // uniform across the workgroup
  if (K < L) {
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      const uint32_t mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
      if (threadIdx.x < 256) hist[threadIdx.x] = 0;
      __syncthreads();
      for (int t = threadIdx.x; t < L; t += kThreads) {
        const uint32_t key = order_key(row[t]);
        if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xffu], 1u);
      }
      __syncthreads();
      if (threadIdx.x < kWave) {
        // lane l owns digits 255-4l .. 252-4l; walk the digits downwards
        const int lane = threadIdx.x;
        uint32_t c[4], tot = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { c[j] = hist[255 - 4 * lane - j]; tot += c[j]; }
        uint32_t incl = tot;               // inclusive scan over lanes
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
          const uint32_t v = __shfl_up(incl, o, kWave);
          if (lane >= o) incl += v;
        }
        uint32_t above = incl - tot;       // keys in strictly higher digits than this lane's
        if (above < remaining && incl >= remaining) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (above < remaining && above + c[j] >= remaining) {
              sh_prefix = prefix | (static_cast<uint32_t>(255 - 4 * lane - j) << shift);
              sh_remaining = remaining - above;
              above = remaining;           // stop: only one digit can match
            } else {
              above += c[j];
            }
          }
        }
      }
      __syncthreads();
      prefix = sh_prefix;
      remaining = sh_remaining;
      __syncthreads();
    }
  } else {
    prefix = 0;                            // take everything: every key >= 0
    remaining = 0;
  }
  const uint32_t T = prefix;
  const bool take_all = !(K < L);
  // remaining = how many keys equal to T are taken (lowest positions first)

  if (threadIdx.x == 0) { sh_base_sel = 0; sh_base_eq = 0; }
  __syncthreads();
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  for (int t0 = 0; t0 < L; t0 += kThreads) {
    const int t = t0 + threadIdx.x;
    uint32_t key = 0;
    bool gt = false, eq = false;
    if (t < L) {
      key = order_key(row[t]);
      gt = take_all || key > T;
      eq = !take_all && key == T;
    }
    // rank among equals, in position order
    const uint64_t eq_mask = __ballot(eq);
    const uint32_t eq_before = __popcll(eq_mask & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[0][wave] = __popcll(eq_mask);
    __syncthreads();
    uint32_t eq_off = sh_base_eq;
    for (int w = 0; w < wave; ++w) eq_off += wave_tot[0][w];
    const bool sel = gt || (eq && eq_off + eq_before < remaining);
    const uint64_t sel_mask = __ballot(sel);
    const uint32_t sel_before = __popcll(sel_mask & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[1][wave] = __popcll(sel_mask);
    __syncthreads();
    uint32_t sel_off = sh_base_sel;
    for (int w = 0; w < wave; ++w) sel_off += wave_tot[1][w];
    if (sel) out[sel_off + sel_before] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
      uint32_t e = 0, s = 0;
      for (int w = 0; w < kWaves; ++w) { e += wave_tot[0][w]; s += wave_tot[1][w]; }
      sh_base_eq += e;
      sh_base_sel += s;
    }
    __syncthreads();
  }
}


// Register-resident variant for rows of at most kThreads * KPT scores: every thread keeps KPT
// consecutive keys, so the row is read once and the ordered emission is one scan (topk_core.hpp).
template <int KPT>
__global__ __launch_bounds__(kThreads) void topk_select(TopkArgs a) {
  __shared__ SelectLds<kThreads, 1> lds;
  const int b = blockIdx.y, g = blockIdx.x;
  const int L = a.seq_lens[b];
  const int K = max(0, min(min(a.budgets[b], L), a.max_budget));
  int32_t* out = a.indices + (static_cast<int64_t>(b) * a.num_kv_heads + g) * a.max_budget;
  if (g == 0 && threadIdx.x == 0) a.counts[b] = K;
  for (int j = K + threadIdx.x; j < a.max_budget; j += kThreads) out[j] = -1;
  if (K == 0) return;
  const float* row = a.scores + (static_cast<int64_t>(b) * a.num_kv_heads + g) * a.score_stride;

  // thread t holds positions t*KPT .. t*KPT+KPT-1
  const int t0 = threadIdx.x * KPT;
  uint32_t key[1][KPT];
  if ((a.score_stride & 3) == 0 && (reinterpret_cast<uintptr_t>(a.scores) & 15u) == 0) {
#pragma unroll
    for (int j = 0; j < KPT; j += 4) {
      float4 v = {0.f, 0.f, 0.f, 0.f};
      if (t0 + j + 3 < L) {
        v = *reinterpret_cast<const float4*>(row + t0 + j);
      } else {
        if (t0 + j < L) v.x = row[t0 + j];
        if (t0 + j + 1 < L) v.y = row[t0 + j + 1];
        if (t0 + j + 2 < L) v.z = row[t0 + j + 2];
      }
      key[0][j] = order_key(v.x); key[0][j + 1] = order_key(v.y); key[0][j + 2] = order_key(v.z); key[0][j + 3] = order_key(v.w);
    }
  } else {
#pragma unroll
    for (int j = 0; j < KPT; ++j) key[0][j] = order_key(t0 + j < L ? row[t0 + j] : 0.f);
  }
  select_topk_in_registers<kThreads, KPT, 1>(key, L, K, out, lds);
}

}  // namespace

hipError_t launch_topk(const TopkArgs& a, hipStream_t s) {
  const dim3 grid(a.num_kv_heads, a.batch), block(kThreads);
  if (a.max_seq_len <= kThreads * 8) {
    KernelTimer t("topk_select", s);
    hipLaunchKernelGGL(topk_select<8>, grid, block, 0, s, a);
  } else if (a.max_seq_len <= kThreads * 16) {
    KernelTimer t("topk_select", s);
    hipLaunchKernelGGL(topk_select<16>, grid, block, 0, s, a);
  } else if (a.max_seq_len <= kThreads * 32) {
    KernelTimer t("topk_select", s);
    hipLaunchKernelGGL(topk_select<32>, grid, block, 0, s, a);
  } else {
    KernelTimer t("topk_radix", s);
    hipLaunchKernelGGL(topk_radix, grid, block, 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace pillar
