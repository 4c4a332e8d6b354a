// Pieces shared by the verification kernels that stream K/V tiles through registers into LDS.
#pragma once

#include "mfma_tile.hpp"

namespace pillar {
namespace {

// Per-lane constants of the row-coalesced tile loads.
template <bool FP8> struct LaneGeom {
  uint32_t lane_off;   // byte offset of this lane's row (within a 16-token group) and column
  uint32_t row_step;   // bytes between the rows two consecutive loads of a lane cover
  int row;             // this lane's row within the tile for load 0
};

template <bool FP8>
__device__ __forceinline__ LaneGeom<FP8> lane_geom(const KvView& kv, int lane) {
  constexpr int kLanesPerRow = FP8 ? 8 : 16;
  const int esz = FP8 ? 1 : 2;
  LaneGeom<FP8> g;
  g.row = lane / kLanesPerRow;
  g.lane_off = static_cast<uint32_t>(g.row * kv.stride_slot * esz + (lane % kLanesPerRow) * 16);
  g.row_step = static_cast<uint32_t>((64 / kLanesPerRow) * kv.stride_slot * esz);
  return g;
}

// Rows of the tile that lie beyond the sequence hold whatever the page holds;
// V must not bring NaN into the matrix product (0 * NaN), so they are zeroed.
template <bool FP8>
__device__ __forceinline__ void zero_tail_rows(u32x4 (&rv)[TileRegs<FP8>::kLoads], int tb, int L, const LaneGeom<FP8>& geo) {
  constexpr int kRowsPerLoad = FP8 ? 8 : 4;
#pragma unroll
  for (int u = 0; u < TileRegs<FP8>::kLoads; ++u)
    if (tb + kRowsPerLoad * u + geo.row >= L) rv[u] = u32x4{0u, 0u, 0u, 0u};
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack2(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v;
  v[0] = static_cast<__bf16>(a);
  v[1] = static_cast<__bf16>(b);
  return __builtin_bit_cast(uint32_t, v);
}

// S^T of the tile with the Q operand read from LDS: rows 0..R-1 in K-tile layout
// followed by one row of zeros that every padded row of the last block reads.
template <int RB>
__device__ __forceinline__ void tile_qk_ldsq(const uint8_t* ktile, const uint8_t* qtile, int R, f32x4 (&acc)[2][RB], int lane) {
  const int n = lane & 15, g = lane >> 4;
  int qrow[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) qrow[rb] = min(16 * rb + n, R);
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[sub][rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const bf16x8 a0 = as_bf16x8(*reinterpret_cast<const u32x4*>(ktile + k_lds_addr(n, 4 * s + g)));
    const bf16x8 a1 = as_bf16x8(*reinterpret_cast<const u32x4*>(ktile + k_lds_addr(16 + n, 4 * s + g)));
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const bf16x8 b = as_bf16x8(*reinterpret_cast<const u32x4*>(qtile + k_lds_addr(qrow[rb], 4 * s + g)));
      acc[0][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, acc[0][rb], 0, 0, 0);
      acc[1][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, acc[1][rb], 0, 0, 0);
    }
    if (RB > 1) __builtin_amdgcn_sched_barrier(0);     // keeps the operand reads from piling up in registers
  }
}

}  // namespace
}  // namespace pillar
