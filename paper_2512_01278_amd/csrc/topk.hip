// Critical-token selection: Top-K of the verification scores per
// (request, KV head) -- paper Section 4.1, "the sparsity pattern can be
// directly identified by ... applying Top-K on the dumped attention scores".
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

namespace pillar {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWave;

__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

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


// Inclusive prefix sum over the 64 lanes of a wavefront on the vector ALU: shifts by 1, 2, 4, 8
// inside each row of 16 lanes, then the last lane of row 0/2 is broadcast into row 1/3 and the last
// lane of the lower half into the upper half (lanes shifted in from outside read 0).
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v) {
  int x = static_cast<int>(v);
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, false);   // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, false);   // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, false);   // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, false);   // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
  return static_cast<uint32_t>(x);
}

// Register-resident variant for rows of at most kThreads * KPT scores: every thread keeps KPT
// consecutive keys, so the row is read once and the ordered emission is one scan.  The key is
// resolved in three passes of 12, 12 and 8 bits: the wide first digit (sign, exponent and three
// mantissa bits) spreads attention scores, which share a few exponents, over many more bins than an
// 8-bit digit does, and that is what keeps the LDS histogram increments from serialising.
template <int KPT>
__global__ __launch_bounds__(kThreads) void topk_select(TopkArgs a) {
  __shared__ uint32_t hist[4096];
  __shared__ uint32_t wave_sum[2][kWaves];
  __shared__ uint32_t sh_prefix, sh_remaining;

  const int b = blockIdx.y, g = blockIdx.x;
  const int L = a.seq_lens[b];
  const int K = max(0, min(min(a.budgets[b], L), a.max_budget));
  int32_t* out = a.indices + (static_cast<int64_t>(b) * a.num_kv_heads + g) * a.max_budget;
  if (g == 0 && threadIdx.x == 0) a.counts[b] = K;
  for (int j = K + threadIdx.x; j < a.max_budget; j += kThreads) out[j] = -1;
  if (K == 0) return;
  const float* row = a.scores + (static_cast<int64_t>(b) * a.num_kv_heads + g) * a.score_stride;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;

  // thread t holds positions t*KPT .. t*KPT+KPT-1; positions beyond L get the smallest key and are never taken
  const int t0 = threadIdx.x * KPT;
  uint32_t key[KPT];
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
      key[j] = order_key(v.x); key[j + 1] = order_key(v.y); key[j + 2] = order_key(v.z); key[j + 3] = order_key(v.w);
    }
  } else {
#pragma unroll
    for (int j = 0; j < KPT; ++j) key[j] = order_key(t0 + j < L ? row[t0 + j] : 0.f);
  }

  uint32_t prefix = 0, remaining = K;      // uniform across the workgroup
  const bool take_all = !(K < L);
  if (!take_all) {
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = pass == 0 ? 20 : pass == 1 ? 8 : 0;
      const int bins = pass == 2 ? 256 : 4096;
      const uint32_t digit_mask = bins - 1;
      const uint32_t mask = pass == 0 ? 0u : pass == 1 ? 0xfff00000u : 0xffffff00u;
      for (int i = threadIdx.x; i < bins; i += kThreads) hist[i] = 0;
      __syncthreads();
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const bool act = t0 + j < L && (key[j] & mask) == prefix;
        const uint32_t bin = (key[j] >> shift) & digit_mask;
        // a wavefront whose active lanes all hit one bin (constant or zero scores) adds once
        const uint64_t m = __ballot(act);
        if (m == 0) continue;
        const int leader = __ffsll(static_cast<long long>(m)) - 1;
        const uint32_t leader_bin = __shfl(bin, leader, kWave);
        if (__all(!act || bin == leader_bin)) {
          if (lane == leader) atomicAdd(&hist[leader_bin], static_cast<uint32_t>(__popcll(m)));
        } else if (act) {
          atomicAdd(&hist[bin], 1u);
        }
      }
      __syncthreads();
      // thread t owns the bins (bins-1) - per*t - j, j < per, walking the digits downwards
      const int per = bins / kThreads;       // 4, or 0 for the 256-bin pass (then the first 256 threads own one)
      uint32_t c[4] = {0u, 0u, 0u, 0u}, tot = 0;
      if (per > 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { c[j] = hist[bins - 1 - 4 * threadIdx.x - j]; tot += c[j]; }
      } else if (threadIdx.x < 256) {
        c[0] = hist[255 - threadIdx.x];
        tot = c[0];
      }
      uint32_t incl = wave_inclusive_sum(tot);   // inclusive scan over the workgroup: lanes, then wavefronts
      if (lane == kWave - 1) wave_sum[0][wave] = incl;
      __syncthreads();
      uint32_t before = 0;
      for (int w = 0; w < wave; ++w) before += wave_sum[0][w];
      incl += before;
      uint32_t above = incl - tot;           // keys in strictly higher digits than this thread's
      if (above < remaining && incl >= remaining) {
        const int nown = per > 0 ? 4 : 1;
        for (int j = 0; j < nown; ++j) {
          if (above < remaining && above + c[j] >= remaining) {
            const uint32_t digit = per > 0 ? static_cast<uint32_t>(bins - 1 - 4 * threadIdx.x - j) : static_cast<uint32_t>(255 - threadIdx.x);
            sh_prefix = prefix | (digit << shift);
            sh_remaining = remaining - above;
            above = remaining;               // stop: only one digit can match
          } else {
            above += c[j];
          }
        }
      }
      __syncthreads();
      prefix = sh_prefix;
      remaining = sh_remaining;
      __syncthreads();
    }
  } else {
    remaining = 0;
  }
  const uint32_t T = prefix;
  // remaining = how many keys equal to T are taken (lowest positions first)

  uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const bool in = t0 + j < L;
    n_gt += (in && (take_all || key[j] > T)) ? 1u : 0u;
    n_eq += (in && !take_all && key[j] == T) ? 1u : 0u;
  }
  // exclusive scans of both counts over the workgroup, in position order
  uint32_t s_gt = wave_inclusive_sum(n_gt), s_eq = wave_inclusive_sum(n_eq);
  if (lane == kWave - 1) { wave_sum[0][wave] = s_gt; wave_sum[1][wave] = s_eq; }
  __syncthreads();
  uint32_t b_gt = 0, b_eq = 0;
  for (int w = 0; w < wave; ++w) { b_gt += wave_sum[0][w]; b_eq += wave_sum[1][w]; }
  uint32_t gt_before = b_gt + s_gt - n_gt, eq_before = b_eq + s_eq - n_eq;
  // output slot of a selected key = (# greater before it) + (# equal-and-taken before it)
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const bool in = t0 + j < L;
    const bool gt = in && (take_all || key[j] > T);
    const bool eq = in && !take_all && key[j] == T;
    if (gt || (eq && eq_before < remaining)) out[gt_before + min(eq_before, remaining)] = t0 + j;
    gt_before += gt ? 1u : 0u;
    eq_before += eq ? 1u : 0u;
  }
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
