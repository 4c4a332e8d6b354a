// The draft step of one (request, KV head, span of the index list) as a device function, shared by the draft
// kernel and by the kernel that runs a unified draft / verify batch in one grid (paper Sections 1 and 4.2).
#pragma once

#include "launch.hpp"
#include "mfma_tile.hpp"

namespace pillar {
namespace {

constexpr int kDecWaves = 4;                      // wavefronts per workgroup of the draft kernel
constexpr int kDecThreads = kDecWaves * kWave;

// Resolved rows of two tiles: lane j < 32 holds row j of one tile, lane 32 + j row j of another.
struct Rows {
  uint32_t off16;  // byte offset of the row in a pool, in units of 16 bytes (rows are 16-byte aligned)
  float ks, vs;    // fp8 only: dequantisation scales of that row
};

// token position -> page id -> row offset (and, for fp8, the scales of its page)
template <bool FP8>
__device__ __forceinline__ Rows resolve_rows(const KvView& kv, int b, int g, int tok) {
  const int esz = FP8 ? 1 : 2;
  Rows r;
  const int page = kv.block_table[static_cast<int64_t>(b) * kv.block_table_stride + (tok >> kv.page_shift)];
  const int64_t off = (static_cast<int64_t>(page) * kv.stride_page + static_cast<int64_t>(g) * kv.stride_head +
                       static_cast<int64_t>(tok & (kv.page_size - 1)) * kv.stride_slot) * esz;
  r.off16 = static_cast<uint32_t>(off >> 4);
  r.ks = r.vs = 1.f;
  if constexpr (FP8) {
    r.ks = kv.k_scale[static_cast<int64_t>(page) * kv.num_kv_heads + g];
    r.vs = kv.v_scale[static_cast<int64_t>(page) * kv.num_kv_heads + g];
  }
  return r;
}

// sends the row loads of the tile in half `half` (0: lanes 0..31, 1: lanes 32..63) of `r`
template <bool FP8>
__device__ __forceinline__ void issue_rows(const KvView& kv, const Rows& r, int half, TileRegs<FP8>& t, int lane) {
  constexpr int kRowsPerLoad = FP8 ? 8 : 4;
  constexpr int kLanesPerRow = FP8 ? 8 : 16;
  const int col = (lane % kLanesPerRow) * 16;
  const char* kp = static_cast<const char*>(kv.k_pool);
  const char* vp = static_cast<const char*>(kv.v_pool);
#pragma unroll
  for (int u = 0; u < TileRegs<FP8>::kLoads; ++u) {
    const int row = kRowsPerLoad * u + lane / kLanesPerRow;
    const uint64_t off = (static_cast<uint64_t>(__shfl(r.off16, 32 * half + row, 64)) << 4) + col;
    t.k[u] = *reinterpret_cast<const u32x4*>(kp + off);
    t.v[u] = *reinterpret_cast<const u32x4*>(vp + off);
  }
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  return f32_to_bf16(a) | (static_cast<uint32_t>(f32_to_bf16(b)) << 16);
}

// One (request slot, KV head, span) of the draft step by a workgroup of WAVES wavefronts.  s_tiles: per
// wavefront one tile buffer (the K rows, then, once S^T is done, the V rows of the same tile; at the end its
// (max, sum, O) for the combine).  Every thread of the workgroup must call this.
template <bool FP8, int WAVES>
__device__ __forceinline__ void decode_span_body(const DecodeArgs& a, const DecWs& ws, int span_rows, int nspan_max, int slot_b, int g,
                                                 int sp, uint8_t (*s_tiles)[kVTileBytes]) {
  const KvView& kv = a.kv;
  const int b = request_of(kv, slot_b);          // everything the request owns is indexed by its id
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int n = lane & 15, g4 = lane >> 4;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  uint8_t* s_tile = s_tiles[wave];
  const int32_t* list = a.indices + (static_cast<int64_t>(b) * kv.num_kv_heads + g) * a.max_budget;
  const int j_begin = sp * span_rows;
  // The index entries of the first four tiles of this wavefront (tiles wave, wave + WAVES, ...; register q holds
  // tile 2q in lanes 0..31 and tile 2q + 1 in lanes 32..63) leave together with the count: entries up to
  // max_budget exist, which of them count is decided when both are here.
  auto entry_of = [&](int round, int q) {
    const int tile = wave + WAVES * (4 * round + 2 * q + (lane >> 5));
    return j_begin + tile * kTileTokens + (lane & 31);
  };
  int tok[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) tok[q] = list[min(entry_of(0, q), a.max_budget - 1)];
  const int count = min(max(a.counts[b], 0), a.max_budget);
  uint16_t* out = static_cast<uint16_t*>(a.out);
  if (count == 0) {
    if (sp == 0) {
      for (int idx = threadIdx.x; idx < G * kHeadDim; idx += (WAVES * kWave))
        out[(static_cast<int64_t>(b) * kv.num_q_heads + g * G) * kHeadDim + idx] = 0;
      if (a.lse && threadIdx.x < G) a.lse[static_cast<int64_t>(b) * kv.num_q_heads + g * G + threadIdx.x] = -INFINITY;
    }
    return;
  }
  if (j_begin >= count) return;
  const int j_end = min(count, j_begin + span_rows);
  const int nspan = (count + span_rows - 1) / span_rows;
  const int ntiles = (j_end - j_begin + kTileTokens - 1) / kTileTokens;       // of the span
  const float c2 = kv.sm_scale * kLog2e;

  f32x4 o[1][8];
#pragma unroll
  for (int d = 0; d < 8; ++d) o[0][d] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;
  if (wave < ntiles) {
    // B operand: lane (n, g4) holds Q[row n][32s + 8 g4 .. +7]
    bf16x8 qf[1][4];
    const uint16_t* qrow = static_cast<const uint16_t*>(a.q) + (static_cast<int64_t>(b) * kv.num_q_heads + g * G + n) * kHeadDim;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (n < G) v = *reinterpret_cast<const u32x4*>(qrow + 32 * s + 8 * g4);
      qf[0][s] = as_bf16x8(v);
    }
    TileRegs<FP8> regs;
    bool first = true;
    for (int round = 0; wave + WAVES * 4 * round < ntiles; ++round) {
      if (round > 0) {
#pragma unroll
        for (int q = 0; q < 2; ++q) tok[q] = list[min(entry_of(round, q), a.max_budget - 1)];
      }
      // one chain for all four tiles: entries -> page ids -> row offsets.  Rows past the end of the list repeat
      // the first row of their tile (masked later); tiles past the end resolve token 0 and are never loaded.
      Rows rr[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int head = __shfl(tok[q], lane & 32, 64);
        const int e = entry_of(round, q);
        const bool tile_there = e - (lane & 31) < j_end;
        rr[q] = resolve_rows<FP8>(kv, b, g, e < j_end ? tok[q] : tile_there ? head : 0);
      }
      const int t_first = wave + WAVES * 4 * round;
      issue_rows<FP8>(kv, rr[0], 0, regs, lane);
      for (int k = 0; k < 4; ++k) {
        const int ti = t_first + WAVES * k;
        if (ti >= ntiles) break;
        const int jb = j_begin + ti * kTileTokens;
        const Rows& cur = (k & 2) ? rr[1] : rr[0];
        const int half = k & 1;
        const bool more = k < 3 && ti + WAVES < ntiles;
        rows_to_lds<FP8, false>(regs.k, s_tile, lane);
        f32x4 s[2][1];
        tile_qk<1>(s_tile, qf, s, lane);
        rows_to_lds<FP8, true>(regs.v, s_tile, lane);
        if (more) issue_rows<FP8>(kv, ((k + 1) & 2) ? rr[1] : rr[0], (k + 1) & 1, regs, lane);
        f32x4 vsc[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int slot = 16 * sub + 4 * g4 + i;
            float sc = c2;
            vsc[sub][i] = 1.f;
            if constexpr (FP8) {
              sc *= __shfl(cur.ks, 32 * half + slot, 64);
              vsc[sub][i] = __shfl(cur.vs, 32 * half + slot, 64);
            }
            float v = s[sub][0][i] * sc;
            if (jb + slot >= j_end) v = -INFINITY;
            s[sub][0][i] = v;
          }
        }
        float mx = fmaxf(fmaxf(fmaxf(s[0][0][0], s[0][0][1]), fmaxf(s[0][0][2], s[0][0][3])),
                         fmaxf(fmaxf(s[1][0][0], s[1][0][1]), fmaxf(s[1][0][2], s[1][0][3])));
        mx = max_over_groups(mx);
        const float m_new = fmaxf(m_run, mx);              // finite: every tile has a valid row
        const float alpha = exp2f(m_run - m_new);
        f32x4 p0, p1;
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          p0[i] = exp2f(s[0][0][i] - m_new);
          p1[i] = exp2f(s[1][0][i] - m_new);
          sum += p0[i] + p1[i];
        }
        l_run = l_run * alpha + sum;
        m_run = m_new;
        if (!first) {
#pragma unroll
          for (int d = 0; d < 8; ++d) o[0][d] *= alpha;
        }
        first = false;
        if constexpr (FP8) { p0 *= vsc[0]; p1 *= vsc[1]; }
        bf16x8 p[1];
        p[0] = pack_p(p0, p1);
        tile_pv<1>(s_tile, p, o, lane);
      }
    }
    l_run = sum_over_groups(l_run);
  }

  // combine the wavefronts of the workgroup: every one leaves (max, sum) per row and its O rows in its own tile
  // buffer (a wavefront that had no tile leaves max = -inf, sum = 0)
  float* part = reinterpret_cast<float*>(s_tile);          // [G][128] O, then [16] max, [16] sum
  if (n < G) {
#pragma unroll
    for (int db = 0; db < 8; ++db) *reinterpret_cast<f32x4*>(part + n * kHeadDim + 16 * db + 4 * g4) = o[0][db];
    if (g4 == 0) { part[16 * kHeadDim + n] = m_run; part[16 * kHeadDim + 16 + n] = l_run; }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * (kHeadDim / 4); idx += (WAVES * kWave)) {
    const int r = idx / (kHeadDim / 4), d4 = idx - r * (kHeadDim / 4);
    float m = -INFINITY;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) m = fmaxf(m, reinterpret_cast<const float*>(s_tiles[w])[16 * kHeadDim + r]);
    float l = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float* pw = reinterpret_cast<const float*>(s_tiles[w]);
      const float wgt = exp2f(pw[16 * kHeadDim + r] - m);        // m is finite: the first wavefront always has a tile
      l = fmaf(pw[16 * kHeadDim + 16 + r], wgt, l);
      acc += *reinterpret_cast<const f32x4*>(pw + r * kHeadDim + 4 * d4) * wgt;
    }
    const int64_t row = static_cast<int64_t>(b) * kv.num_q_heads + g * G + r;
    if (nspan == 1) {
      const float inv = 1.0f / l;
      u32x2 pk;
      pk.x = pack_bf16x2(acc.x * inv, acc.y * inv);
      pk.y = pack_bf16x2(acc.z * inv, acc.w * inv);
      *reinterpret_cast<u32x2*>(out + row * kHeadDim + 4 * d4) = pk;
      if (d4 == 0 && a.lse) a.lse[row] = (m + log2f(l)) * kLn2;
    } else {
      const int64_t slot = (static_cast<int64_t>(slot_b) * kv.num_kv_heads + g) * nspan_max + sp;
      if (d4 == 0) { ws.part_m[slot * 16 + r] = m; ws.part_l[slot * 16 + r] = l; }
      *reinterpret_cast<f32x4*>(ws.part_o + (slot * G + r) * kHeadDim + 4 * d4) = acc;
    }
  }
}

}  // namespace
}  // namespace pillar
