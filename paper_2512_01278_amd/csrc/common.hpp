// Shared device-side definitions of the PillarAttn kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pillar.h"

namespace pillar {

constexpr int kWave = 64;
constexpr int kMaxRows = 64;      // (k+1)*G rows of one KV head at most
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Device-side copy of the fields of pillar_kv_t the kernels read.
struct KvView {
  const void* k_pool;
  const void* v_pool;
  const float* k_scale;
  const float* v_scale;
  const int32_t* block_table;
  const int32_t* seq_lens;
  const int32_t* req_ids;      // null: slot i of this launch is request i; else request req_ids[i] (batch = number of slots)
  int64_t stride_page, stride_head, stride_slot;
  int32_t batch, num_q_heads, num_kv_heads, head_dim, page_size, page_shift;
  int32_t block_table_stride, max_seq_len;
  float sm_scale;
};

// A launch may cover a subset of the requests (a unified batch: some verify while the others draft).  Work is
// divided over the slots 0 .. batch-1 of the launch; everything a request owns (its row of the block table, its
// length, its queries, outputs, scores and index lists) is indexed by the request id of the slot.
__device__ __forceinline__ int request_of(const KvView& kv, int slot) { return kv.req_ids ? kv.req_ids[slot] : slot; }

// ---- storage formats -------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// round to nearest even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// OCP fp8 e4m3: sign, 4 exponent bits (bias 7), 3 mantissa bits; exponent 0 is
// subnormal (m * 2^-9); S.1111.111 is NaN; there are no infinities.
__device__ __forceinline__ float e4m3_to_f32(uint8_t c) {
  const uint32_t sign = static_cast<uint32_t>(c & 0x80u) << 24;
  const uint32_t mag = c & 0x7fu;
  float v;
  if (mag == 0x7fu) {
    v = __uint_as_float(0x7fc00000u);
  } else if (mag < 8u) {
    v = static_cast<float>(mag) * 0.001953125f;          // 2^-9
  } else {
    v = __uint_as_float((mag << 20) + (120u << 23));      // rebias 7 -> 127
  }
  return __uint_as_float(__float_as_uint(v) | sign);
}

template <int DT> struct Storage;
template <> struct Storage<PILLAR_F32> {
  using type = float;
  static __device__ __forceinline__ float load(const void* p, int64_t i) {
    return static_cast<const float*>(p)[i];
  }
  static __device__ __forceinline__ void store(void* p, int64_t i, float v) {
    static_cast<float*>(p)[i] = v;
  }
};
template <> struct Storage<PILLAR_BF16> {
  using type = uint16_t;
  static __device__ __forceinline__ float load(const void* p, int64_t i) {
    return bf16_to_f32(static_cast<const uint16_t*>(p)[i]);
  }
  static __device__ __forceinline__ void store(void* p, int64_t i, float v) {
    static_cast<uint16_t*>(p)[i] = f32_to_bf16(v);
  }
};
template <> struct Storage<PILLAR_FP8_E4M3> {
  using type = uint8_t;
  static __device__ __forceinline__ float load(const void* p, int64_t i) {
    return e4m3_to_f32(static_cast<const uint8_t*>(p)[i]);
  }
};

// ---- wave-level reductions ---------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// element offset of (token t of request b, KV head g) in a pool, and its page
__device__ __forceinline__ int64_t row_offset(const KvView& kv, int b, int g, int t, int* page_out) {
  const int page = kv.block_table[static_cast<int64_t>(b) * kv.block_table_stride + (t >> kv.page_shift)];
  const int slot = t & (kv.page_size - 1);
  *page_out = page;
  return static_cast<int64_t>(page) * kv.stride_page + static_cast<int64_t>(g) * kv.stride_head +
         static_cast<int64_t>(slot) * kv.stride_slot;
}

}  // namespace pillar
