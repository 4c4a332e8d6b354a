// Exact selection of the K largest of up to kSelectThreads * KPT keys held in registers by one
// 1024-thread workgroup (paper Section 4.1: Top-K on the averaged scores).  Shared by the stand-alone
// Top-K kernel and by the verification finish kernel that selects straight from on-chip scores.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"

namespace pillar {
namespace {

constexpr int kSelectThreads = 1024;
constexpr int kSelectWaves = kSelectThreads / kWave;

// float -> unsigned key whose integer order is the float order
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
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

// LDS the selection needs (one instance per workgroup).
struct SelectLds {
  uint32_t hist[4096];
  uint32_t wave_sum[2][kSelectWaves];
  uint32_t prefix, remaining;
};

// Thread t holds the keys of positions t*KPT .. t*KPT+KPT-1 (`t0` = t*KPT); positions >= L are ignored.
// Writes the K selected positions in ascending order to out[0..K).  Three histogram passes of 12, 12 and
// 8 bits find the K-th largest key: the wide first digit (sign, exponent and three mantissa bits) spreads
// attention scores, which share a few exponents, over many more bins than an 8-bit digit does, and that is
// what keeps the LDS histogram increments from serialising.  Every thread of the workgroup must call this.
template <int KPT>
__device__ __forceinline__ void select_topk_in_registers(const uint32_t (&key)[KPT], int t0, int L, int K, int32_t* out,
                                                         SelectLds& lds) {
  uint32_t* hist = lds.hist;
  uint32_t (*wave_sum)[kSelectWaves] = lds.wave_sum;
  uint32_t& sh_prefix = lds.prefix;
  uint32_t& sh_remaining = lds.remaining;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  uint32_t prefix = 0, remaining = K;      // uniform across the workgroup
  const bool take_all = !(K < L);
  if (!take_all) {
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = pass == 0 ? 20 : pass == 1 ? 8 : 0;
      const int bins = pass == 2 ? 256 : 4096;
      const uint32_t digit_mask = bins - 1;
      const uint32_t mask = pass == 0 ? 0u : pass == 1 ? 0xfff00000u : 0xffffff00u;
      for (int i = threadIdx.x; i < bins; i += kSelectThreads) hist[i] = 0;
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
      const int per = bins / kSelectThreads;       // 4, or 0 for the 256-bin pass (then the first 256 threads own one)
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
}  // namespace pillar
