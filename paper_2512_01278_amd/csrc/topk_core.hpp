// Exact selection of the K largest keys held in registers by one workgroup (paper Section 4.1: Top-K on
// the averaged scores).  Shared by the stand-alone Top-K kernel and by the verification finish kernel,
// which selects straight from on-chip scores.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"

namespace pillar {
namespace {

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

// minimum / maximum over the 64 lanes of a wavefront, uniform result: the same DPP ladder as the prefix sum (lanes
// without a source keep the identity), the total ends up in the last lane
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  int x = static_cast<int>(v);
  const int id = -1;                               // 0xffffffff
  auto mn = [](int a, int b) { return static_cast<int>(min(static_cast<uint32_t>(a), static_cast<uint32_t>(b))); };
  x = mn(x, __builtin_amdgcn_update_dpp(id, x, 0x111, 0xF, 0xF, false));
  x = mn(x, __builtin_amdgcn_update_dpp(id, x, 0x112, 0xF, 0xF, false));
  x = mn(x, __builtin_amdgcn_update_dpp(id, x, 0x114, 0xF, 0xF, false));
  x = mn(x, __builtin_amdgcn_update_dpp(id, x, 0x118, 0xF, 0xF, false));
  x = mn(x, __builtin_amdgcn_update_dpp(id, x, 0x142, 0xA, 0xF, false));
  x = mn(x, __builtin_amdgcn_update_dpp(id, x, 0x143, 0xC, 0xF, false));
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(x, kWave - 1));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  int x = static_cast<int>(v);
  auto mx = [](int a, int b) { return static_cast<int>(max(static_cast<uint32_t>(a), static_cast<uint32_t>(b))); };
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, false));
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, false));
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, false));
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, false));
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false));
  x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false));
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(x, kWave - 1));
}

// LDS the selection needs (one instance per workgroup of THREADS threads holding CH chunks of keys).
template <int THREADS, int CH> struct SelectLds {
  uint32_t hist[4096];
  uint32_t wave_sum[2][CH][THREADS / kWave];
  uint32_t prefix[3], remaining[3];        // one slot per pass: no barrier between reading one and writing the next
};

// The workgroup holds CH * THREADS * KPC keys: key[c][j] of thread t belongs to position
// c * (THREADS * KPC) + t * KPC + j; positions >= L are ignored.  Writes the K selected positions in
// ascending order to out[0..K).  Three histogram passes of 12, 12 and 8 bits find the K-th largest key:
// the wide first digit (sign, exponent and three mantissa bits) spreads attention scores, which share a
// few exponents, over many more bins than an 8-bit digit does, and that is what keeps the LDS histogram
// increments from serialising.  Equal keys go to the lower position.  Every thread of the workgroup must
// call this.
template <int THREADS, int KPC, int CH>
__device__ __forceinline__ void select_topk_in_registers(const uint32_t (&key)[CH][KPC], int L, int K, int32_t* out,
                                                         SelectLds<THREADS, CH>& lds) {
  constexpr int kWaves = THREADS / kWave;
  constexpr int kChunk = THREADS * KPC;
  static_assert(4096 % THREADS == 0 && THREADS >= 256, "bins are dealt out evenly");
  uint32_t* hist = lds.hist;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int t0 = static_cast<int>(threadIdx.x) * KPC;
  uint32_t prefix = 0, remaining = K;      // uniform across the workgroup
  const bool take_all = !(K < L);
  const int nch = (L + kChunk - 1) / kChunk;   // chunks that hold any position of this row (uniform): the others are skipped
  if (!take_all) {
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = pass == 0 ? 20 : pass == 1 ? 8 : 0;
      const int bins = pass == 2 ? 256 : 4096;
      const uint32_t digit_mask = bins - 1;
      const uint32_t mask = pass == 0 ? 0u : pass == 1 ? 0xfff00000u : 0xffffff00u;
      if (pass == 0) {                           // later passes find the bins zeroed by their last readers
        for (int i = threadIdx.x; i < 4096; i += THREADS) hist[i] = 0;
        __syncthreads();
      }
      // A wavefront whose active keys all fall into one bin (constant or zero scores, or the few keys left in a late
      // pass) adds their number once instead of queueing up on one LDS address; otherwise every key adds itself.
      uint32_t lo = 0xffffffffu, hi = 0u, mine = 0u;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        if (c >= nch) continue;
#pragma unroll
        for (int j = 0; j < KPC; ++j) {
          const bool act = c * kChunk + t0 + j < L && (key[c][j] & mask) == prefix;
          const uint32_t bin = (key[c][j] >> shift) & digit_mask;
          lo = act ? min(lo, bin) : lo;
          hi = act ? max(hi, bin) : hi;
          mine += act ? 1u : 0u;
        }
      }
      const uint32_t wave_lo = wave_min_u32(lo), wave_hi = wave_max_u32(hi);
      if (wave_lo >= wave_hi) {                  // one bin, or no active key at all (lo = ~0 > hi = 0)
        const uint32_t total = wave_inclusive_sum(mine);
        if (lane == kWave - 1 && total > 0) atomicAdd(&hist[wave_lo], total);
      } else {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          if (c >= nch) continue;
#pragma unroll
          for (int j = 0; j < KPC; ++j) {
            const bool act = c * kChunk + t0 + j < L && (key[c][j] & mask) == prefix;
            if (act) atomicAdd(&hist[(key[c][j] >> shift) & digit_mask], 1u);
          }
        }
      }
      __syncthreads();
      // thread t owns the bins (bins-1) - per*t - j, j < per, walking the digits downwards; it reads them
      // and leaves them zero for the next pass
      constexpr int kPerWide = 4096 / THREADS;     // 4 or 8 bins per thread in the two 12-bit passes
      const int per = pass == 2 ? (threadIdx.x < 256 ? 1 : 0) : kPerWide;
      uint32_t cnt[kPerWide], tot = 0;
#pragma unroll
      for (int j = 0; j < kPerWide; ++j) {
        cnt[j] = 0u;
        if (j < per) {
          uint32_t& slot = hist[bins - 1 - per * static_cast<int>(threadIdx.x) - j];
          cnt[j] = slot;
          slot = 0u;
        }
        tot += cnt[j];
      }
      uint32_t incl = wave_inclusive_sum(tot);   // inclusive scan over the workgroup: lanes, then wavefronts
      if (lane == kWave - 1) lds.wave_sum[pass & 1][0][wave] = incl;
      __syncthreads();
      uint32_t before = 0;
#pragma unroll 1
      for (int w = 0; w < wave; ++w) before += lds.wave_sum[pass & 1][0][w];
      incl += before;
      uint32_t above = incl - tot;           // keys in strictly higher digits than this thread's
      if (above < remaining && incl >= remaining) {
#pragma unroll
        for (int j = 0; j < kPerWide; ++j) {
          if (j < per) {
            if (above < remaining && above + cnt[j] >= remaining) {
              const uint32_t digit = static_cast<uint32_t>(bins - 1 - per * static_cast<int>(threadIdx.x) - j);
              lds.prefix[pass] = prefix | (digit << shift);
              lds.remaining[pass] = remaining - above;
              above = remaining;               // stop: only one digit can match
            } else {
              above += cnt[j];
            }
          }
        }
      }
      __syncthreads();
      prefix = lds.prefix[pass];
      remaining = lds.remaining[pass];
    }
  } else {
    remaining = 0;
  }
  const uint32_t T = prefix;
  // remaining = how many keys equal to T are taken (lowest positions first)

  // per chunk: how many of this thread's keys lie above T, and how many equal it
  uint32_t n_gt[CH], n_eq[CH], s_gt[CH], s_eq[CH];
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    n_gt[c] = n_eq[c] = s_gt[c] = s_eq[c] = 0;
    if (c >= nch) continue;
#pragma unroll
    for (int j = 0; j < KPC; ++j) {
      const bool in = c * kChunk + t0 + j < L;
      n_gt[c] += (in && (take_all || key[c][j] > T)) ? 1u : 0u;
      n_eq[c] += (in && !take_all && key[c][j] == T) ? 1u : 0u;
    }
    // exclusive scans of both counts over the workgroup, in position order (positions grow with the
    // chunk first, then with the thread)
    s_gt[c] = wave_inclusive_sum(n_gt[c]);
    s_eq[c] = wave_inclusive_sum(n_eq[c]);
    if (lane == kWave - 1) { lds.wave_sum[0][c][wave] = s_gt[c]; lds.wave_sum[1][c][wave] = s_eq[c]; }
  }
  __syncthreads();
  uint32_t base_gt = 0, base_eq = 0;           // keys of earlier chunks
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    if (c >= nch) continue;
    uint32_t b_gt = 0, b_eq = 0, t_gt = 0, t_eq = 0;
#pragma unroll 1
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t a = lds.wave_sum[0][c][w], e = lds.wave_sum[1][c][w];
      if (w < wave) { b_gt += a; b_eq += e; }
      t_gt += a;
      t_eq += e;
    }
    uint32_t gt_before = base_gt + b_gt + s_gt[c] - n_gt[c], eq_before = base_eq + b_eq + s_eq[c] - n_eq[c];
    // output slot of a selected key = (# greater before it) + (# equal-and-taken before it)
#pragma unroll
    for (int j = 0; j < KPC; ++j) {
      const int pos = c * kChunk + t0 + j;
      const bool in = pos < L;
      const bool gt = in && (take_all || key[c][j] > T);
      const bool eq = in && !take_all && key[c][j] == T;
      if (gt || (eq && eq_before < remaining)) out[gt_before + min(eq_before, remaining)] = pos;
      gt_before += gt ? 1u : 0u;
      eq_before += eq ? 1u : 0u;
    }
    base_gt += t_gt;
    base_eq += t_eq;
  }
}

}  // namespace
}  // namespace pillar
