// The tile engine shared by the MFMA verification and draft kernels (gfx950).
//
// One wavefront owns a tile of 32 token rows of one KV head: it loads the K
// and V rows from the paged pool with 16-byte, row-coalesced loads, parks
// them in its private 16 KiB of LDS, and feeds v_mfma_f32_16x16x32_bf16:
//
//   S^T[token, row] = K[token, :] . Q[row, :]      A = K   (16 tokens x 32 dims)
//                                                  B = Q^T (32 dims  x 16 rows)
//   O^T[dim,  row] += V[token, dim] * P[row, token] A = V^T (16 dims  x 32 tokens)
//                                                  B = P^T (32 tokens x 16 rows)
//
// "row" is one of the R = (k+1)*G query rows that share the KV head (paper
// Section 4.1: the k+1 verification queries, times the query heads of one
// group); a draft step has R = G.  Tokens sit on the MFMA's M side, so every
// lane owns ONE query row (its column n = lane % 16) and the online-softmax
// state of that row: the row maximum and sum need no cross-row traffic, and
// the accumulator layout of S^T (lane group g = lane / 16 holds tokens 4g..4g+3)
// is already the B-operand layout of P^T once the contraction index is
// permuted, which costs nothing because V^T is read with the same permutation.
//
// LDS layout of a tile: 32 padded rows (see kKRow / kVRow) so that the
// column-wise MFMA operand reads (K) and the transposing reads (V) spread over
// all banks.
#pragma once

#include "common.hpp"

namespace pillar {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTileTokens = 32;
constexpr int kHeadDim = 128;
// LDS rows are padded instead of swizzled: every access of a lane is then
// "per-lane base + compile-time offset", one address register per access kind.
//   K rows, 272 B apart: the 16 lanes of an MFMA operand read (16 rows, one
//   16-byte chunk each) fall 4 banks apart -> all 64 banks, no conflict.
//   V rows, 288 B apart: the 16 lanes of a transposing read (4 rows x 32 B)
//   fall 8 banks apart per row, and the next lane group 32 banks further.
constexpr int kKRow = 272;
constexpr int kVRow = 288;
constexpr int kKTileBytes = kTileTokens * kKRow;         // 8704
constexpr int kVTileBytes = kTileTokens * kVRow;         // 9216
constexpr int kWaveLds = kKTileBytes + kVTileBytes;      // K tile + V tile of one wavefront

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// byte address of 16-byte chunk `c` of row `r` in a K tile / a V tile
__device__ __forceinline__ int k_lds_addr(int r, int c) { return r * kKRow + (c << 4); }
__device__ __forceinline__ int v_lds_addr(int r, int c) { return r * kVRow + (c << 4); }

__device__ __forceinline__ float xor16(float v) { return __shfl_xor(v, 16, 64); }
__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32, 64); }

// Maximum / sum over the four lanes l, l^16, l^32, l^48 (the four token groups of one query row),
// left in all four.  v_permlane16_swap / v_permlane32_swap exchange 16- and 32-lane rows between two
// registers on the vector ALU: with both operands holding v, one result holds each lane's own row
// pair partner-first and the other own-first, so a commutative combine of the two results is the
// pairwise combine -- no trip through the LDS crossbar as with a shuffle.
__device__ __forceinline__ float max_over_groups(float v) {
  typedef unsigned u2 __attribute__((ext_vector_type(2)));
  u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float sum_over_groups(float v) {
  typedef unsigned u2 __attribute__((ext_vector_type(2)));
  u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(r.x) + __uint_as_float(r.y);
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r.x) + __uint_as_float(r.y);
}

// sum over the 16 lanes of a DPP row (all 16 lanes receive the total)
__device__ __forceinline__ float row16_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
  return v;
}

// Registers of one 32-token tile in flight from HBM.
//   bf16: 8 loads of 16 B for K and 8 for V per lane; load u covers token rows
//         4u..4u+3, 16 lanes per 256-byte row.
//   fp8 : 4 loads each; load u covers rows 8u..8u+7, 8 lanes per 128-byte row.
template <bool FP8> struct TileRegs {
  static constexpr int kLoads = FP8 ? 4 : 8;
  u32x4 k[kLoads];
  u32x4 v[kLoads];
};

// two packed fp8 e4m3 -> two packed bf16 (exact: e4m3 is a subset of bf16)
__device__ __forceinline__ uint32_t fp8x2_to_bf16x2(uint32_t src, bool hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  const f32x2 f = hi ? __builtin_amdgcn_cvt_pk_f32_fp8(src, true) : __builtin_amdgcn_cvt_pk_f32_fp8(src, false);
  // both values are exactly representable in bf16: truncation is exact
  return (__float_as_uint(f.x) >> 16) | (__float_as_uint(f.y) & 0xffff0000u);
}

// sixteen fp8 -> two 16-byte chunks of bf16
__device__ __forceinline__ void widen_fp8x16(const u32x4& src, u32x4& lo, u32x4& hi) {
  lo.x = fp8x2_to_bf16x2(src.x, false); lo.y = fp8x2_to_bf16x2(src.x, true);
  lo.z = fp8x2_to_bf16x2(src.y, false); lo.w = fp8x2_to_bf16x2(src.y, true);
  hi.x = fp8x2_to_bf16x2(src.z, false); hi.y = fp8x2_to_bf16x2(src.z, true);
  hi.z = fp8x2_to_bf16x2(src.w, false); hi.w = fp8x2_to_bf16x2(src.w, true);
}

// Parks the K (IS_V = false) or V rows of a tile in LDS as bf16 rows (fp8 rows
// are widened here, exactly).
template <bool FP8, bool IS_V>
__device__ __forceinline__ void rows_to_lds(const u32x4 (&regs)[TileRegs<FP8>::kLoads], uint8_t* tile, int lane) {
  if constexpr (!FP8) {
    const int c = lane & 15;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = 4 * u + (lane >> 4);
      *reinterpret_cast<u32x4*>(tile + (IS_V ? v_lds_addr(r, c) : k_lds_addr(r, c))) = regs[u];
    }
  } else {
    const int c = (lane & 7) * 2;          // 16 fp8 = two 16-byte bf16 chunks
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = 8 * u + (lane >> 3);
      u32x4 lo, hi;
      widen_fp8x16(regs[u], lo, hi);
      *reinterpret_cast<u32x4*>(tile + (IS_V ? v_lds_addr(r, c) : k_lds_addr(r, c))) = lo;
      *reinterpret_cast<u32x4*>(tile + (IS_V ? v_lds_addr(r, c + 1) : k_lds_addr(r, c + 1))) = hi;
    }
  }
}

template <bool FP8>
__device__ __forceinline__ void tile_to_lds(const TileRegs<FP8>& t, uint8_t* ktile, uint8_t* vtile, int lane) {
  rows_to_lds<FP8, false>(t.k, ktile, lane);
  rows_to_lds<FP8, true>(t.v, vtile, lane);
}

// S^T of the tile: acc[sub][rb] (sub = 16-token half, rb = 16-row block of Q).
// qf[rb][s] holds, for lane (n, g), Q[16rb+n][32s+8g .. 32s+8g+7].
template <int RB>
__device__ __forceinline__ void tile_qk(const uint8_t* ktile, const bf16x8 (&qf)[RB][4], f32x4 (&acc)[2][RB], int lane) {
  const int n = lane & 15, g = lane >> 4;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[sub][rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const u32x4 raw = *reinterpret_cast<const u32x4*>(ktile + k_lds_addr(16 * sub + n, 4 * s + g));
      const bf16x8 a = as_bf16x8(raw);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) acc[sub][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[rb][s], acc[sub][rb], 0, 0, 0);
    }
  }
}

// O^T += V^T P^T for the tile.  p[rb] is lane (n, g)'s B operand: elements
// 0..3 = P[row n][token 4g+0..3], elements 4..7 = P[row n][token 16+4g+0..3].
// The V^T operand comes from ds_read_b64_tr_b16: within each group of 16
// lanes, lane 4k+a supplies the address of 4 dims (16db+4a..+3) of token k of
// the group, and lane m receives dim 16db+m of the four tokens.  The
// accumulator o[rb][db] element i of lane (n, g) is O[row n][16db + 4g + i].
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;

template <int RB>
__device__ __forceinline__ void tile_pv(const uint8_t* vtile, const bf16x8 (&p)[RB], f32x4 (&o)[RB][8], int lane) {
  const int j = lane & 15, g = lane >> 4;
  const int k = j >> 2, a = j & 3;
  const int row0 = 4 * g + k, row1 = 16 + 4 * g + k;
#pragma unroll
  for (int db = 0; db < 8; ++db) {
    const int c = 2 * db + (a >> 1);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vtile + v_lds_addr(row0, c) + (a & 1) * 8));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vtile + v_lds_addr(row1, c) + (a & 1) * 8));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    const bf16x8 av = __builtin_bit_cast(bf16x8, both);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) o[rb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, p[rb], o[rb][db], 0, 0, 0);
    if (RB > 1 && (db & 1)) __builtin_amdgcn_sched_barrier(0);     // keeps the operand reads from piling up in registers
  }
}

// eight fp32 -> packed bf16 B operand (round to nearest even)
__device__ __forceinline__ bf16x8 pack_p(const f32x4& a, const f32x4& b) {
  bf16x8 r;
  r[0] = static_cast<__bf16>(a.x); r[1] = static_cast<__bf16>(a.y); r[2] = static_cast<__bf16>(a.z); r[3] = static_cast<__bf16>(a.w);
  r[4] = static_cast<__bf16>(b.x); r[5] = static_cast<__bf16>(b.y); r[6] = static_cast<__bf16>(b.z); r[7] = static_cast<__bf16>(b.w);
  return r;
}

}  // namespace pillar
