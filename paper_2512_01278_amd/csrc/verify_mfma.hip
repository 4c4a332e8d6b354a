// Verification attention on the matrix cores (bf16 queries, bf16 or fp8 KV,
// head_dim 128, pages of >= 16 tokens).
//
// Paper Section 4.1: the k+1 verification queries attend to the whole
// KV-Cache, and the softmax probabilities of that pass, averaged over the
// queries and the query heads of one GQA group, are what Top-K reads next.
// Section 1: the step is bound by loading the KV-Cache, so the kernel is
// organised around keeping HBM loads in flight; the arithmetic (R = (k+1)*G
// rows against every token: 20..80 flop per KV byte) goes to MFMA because the
// vector ALUs could not keep up with 8 TB/s.
//
// Work is cut into items of kChunk tokens of one (request, KV head) and handed
// out by an atomic ticket to a persistent grid (ragged contexts balance
// themselves).  Inside an item each of the four wavefronts streams its own
// 32-token tiles (mfma_tile.hpp) with the next tile's loads in flight while
// the current one is computed; no barrier is needed until the four partial
// (max, sum, O) are merged in LDS and written as the item's partial.
//
// Launches: plan (item table, counters) -> split (this) -> merge (partials ->
// out, lse) -> scores (QK^T again over K only, against the final lse).
#include "launch.hpp"
#include "mfma_tile.hpp"

namespace pillar {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kChunk = 512;                 // tokens per work item
constexpr int kLdsBytes = kWaves * kWaveLds;

struct FastWs {
  int32_t* ctrl;        // [0] split ticket, [1] scores ticket, [2] item count
  int32_t* item_base;   // [B+1] first item of request b (items of b: Hkv * chunks(b))
  int32_t* items;       // [max_items][2] = {b, g << 16 | chunk}
  float* part_m;        // [max_items][RB*16]  log2 domain
  float* part_l;        // [max_items][RB*16]
  float* part_o;        // [max_items][R][128]
  float* lse2;          // [B][Hkv][RB*16]     log2 domain, final
  int32_t max_items;
};

__host__ __device__ inline int chunks_of(int len) { return (len + kChunk - 1) / kChunk; }

// ---------------------------------------------------------------- plan ------
__global__ __launch_bounds__(1024) void verify_plan(KvView kv, FastWs ws) {
  __shared__ int32_t scan[1024];
  __shared__ int32_t carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int b0 = 0; b0 < kv.batch; b0 += 1024) {
    const int b = b0 + threadIdx.x;
    const int mine = b < kv.batch ? chunks_of(kv.seq_lens[b]) * kv.num_kv_heads : 0;
    scan[threadIdx.x] = mine;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int v = threadIdx.x >= o ? scan[threadIdx.x - o] : 0;
      __syncthreads();
      scan[threadIdx.x] += v;
      __syncthreads();
    }
    const int first = carry + scan[threadIdx.x] - mine;
    if (b < kv.batch) {
      ws.item_base[b] = first;
      const int nc = mine / kv.num_kv_heads;
      for (int j = 0; j < mine; ++j) {
        ws.items[2 * (first + j)] = b;
        ws.items[2 * (first + j) + 1] = ((j / nc) << 16) | (j % nc);
      }
    }
    __syncthreads();
    if (threadIdx.x == 1023) carry += scan[1023];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    ws.item_base[kv.batch] = carry;
    ws.ctrl[0] = 0;
    ws.ctrl[1] = 0;
    ws.ctrl[2] = carry;
  }
}

// ------------------------------------------------------- item helpers -------
struct Item {
  int b, g, c, L, t_begin, t_end, id;
};

__device__ __forceinline__ Item decode_item(const KvView& kv, const FastWs& ws, int id) {
  Item it;
  it.id = id;
  it.b = ws.items[2 * id];
  const int gc = ws.items[2 * id + 1];
  it.g = gc >> 16;
  it.c = gc & 0xffff;
  it.L = kv.seq_lens[it.b];
  it.t_begin = it.c * kChunk;
  it.t_end = min(it.L, it.t_begin + kChunk);
  return it;
}

template <int RB>
__device__ __forceinline__ void load_q_frags(const KvView& kv, const uint16_t* q, int n_q, int G, int R, const Item& it,
                                             bf16x8 (&qf)[RB][4], int lane) {
  const int n = lane & 15, g4 = lane >> 4;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int r = 16 * rb + n;
    const int i = r / G, hg = r - i * G;
    const uint16_t* row = q + ((static_cast<int64_t>(it.b) * n_q + i) * kv.num_q_heads + it.g * G + hg) * kHeadDim;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (r < R) v = *reinterpret_cast<const u32x4*>(row + 32 * s + 8 * g4);
      qf[rb][s] = as_bf16x8(v);
    }
  }
}

// Issues the loads of the 32-token tile that starts at token `tb`.  Rows past
// the end of the sequence re-read the last valid row (they are masked later).
// pg holds, in lane j, the page id of page (t_begin / P + j) of the request.
template <bool FP8>
__device__ __forceinline__ void issue_tile(const KvView& kv, const Item& it, int tb, int pg, TileRegs<FP8>& t, int lane) {
  constexpr int kRowsPerLoad = FP8 ? 8 : 4;
  constexpr int kLanesPerRow = FP8 ? 8 : 16;
  const int first_page = it.t_begin >> kv.page_shift;
  const int col = (lane % kLanesPerRow) * 16;       // byte offset inside the row
  const char* kp = static_cast<const char*>(kv.k_pool);
  const char* vp = static_cast<const char*>(kv.v_pool);
  const int esz = FP8 ? 1 : 2;
#pragma unroll
  for (int u = 0; u < TileRegs<FP8>::kLoads; ++u) {
    const int tok = min(tb + kRowsPerLoad * u + lane / kLanesPerRow, it.L - 1);
    const int page = __shfl(pg, (tok >> kv.page_shift) - first_page, 64);
    const int64_t off = (static_cast<int64_t>(page) * kv.stride_page + static_cast<int64_t>(it.g) * kv.stride_head +
                         static_cast<int64_t>(tok & (kv.page_size - 1)) * kv.stride_slot) * esz + col;
    t.k[u] = *reinterpret_cast<const u32x4*>(kp + off);
    t.v[u] = *reinterpret_cast<const u32x4*>(vp + off);
  }
}

__device__ __forceinline__ int load_page_ids(const KvView& kv, const Item& it, int lane) {
  const int first_page = it.t_begin >> kv.page_shift;
  const int last_page = (it.L - 1) >> kv.page_shift;
  const int p = min(first_page + lane, last_page);
  return kv.block_table[static_cast<int64_t>(it.b) * kv.block_table_stride + p];
}

// per-page dequantisation scales of the two 16-token halves of a tile
__device__ __forceinline__ void tile_scales(const KvView& kv, const Item& it, int tb, int pg, float (&ks)[2], float (&vs)[2]) {
  const int first_page = it.t_begin >> kv.page_shift;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const int tok = min(tb + 16 * sub, it.L - 1);
    const int page = __shfl(pg, (tok >> kv.page_shift) - first_page, 64);
    ks[sub] = kv.k_scale[static_cast<int64_t>(page) * kv.num_kv_heads + it.g];
    vs[sub] = kv.v_scale[static_cast<int64_t>(page) * kv.num_kv_heads + it.g];
  }
}

// ---------------------------------------------------------------- split -----
template <int RB, bool FP8>
__global__ __launch_bounds__(kThreads, 2) void verify_split_mfma(KvView kv, const uint16_t* q, int n_q, FastWs ws) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  __shared__ int s_item;
  __shared__ float s_m[kWaves][RB * 16], s_l[kWaves][RB * 16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, g4 = lane >> 4;
  uint8_t* ktile = smem + wave * kWaveLds;
  uint8_t* vtile = ktile + kKTileBytes;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const float c2 = kv.sm_scale * kLog2e;
  const int total = ws.ctrl[2];

  for (;;) {
    if (threadIdx.x == 0) s_item = atomicAdd(&ws.ctrl[0], 1);
    __syncthreads();
    const int id = s_item;
    __syncthreads();
    if (id >= total) break;
    const Item it = decode_item(kv, ws, id);
    const int ntiles = (it.t_end - it.t_begin + kTileTokens - 1) / kTileTokens;

    bf16x8 qf[RB][4];
    f32x4 o[RB][8];
    float m_run[RB], l_run[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      m_run[rb] = -INFINITY;
      l_run[rb] = 0.f;
#pragma unroll
      for (int d = 0; d < 8; ++d) o[rb][d] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    if (wave < ntiles) {
      load_q_frags<RB>(kv, q, n_q, G, R, it, qf, lane);
      const int pg = load_page_ids(kv, it, lane);
      TileRegs<FP8> regs;
      issue_tile<FP8>(kv, it, it.t_begin + wave * kTileTokens, pg, regs, lane);
      for (int ti = wave; ti < ntiles; ti += kWaves) {
        const int tb = it.t_begin + ti * kTileTokens;
        tile_to_lds<FP8>(regs, ktile, vtile, lane);
        float ks[2] = {1.f, 1.f}, vs[2] = {1.f, 1.f};
        if constexpr (FP8) tile_scales(kv, it, tb, pg, ks, vs);
        if (ti + kWaves < ntiles) issue_tile<FP8>(kv, it, tb + kWaves * kTileTokens, pg, regs, lane);

        f32x4 s[2][RB];
        tile_qk<RB>(ktile, qf, s, lane);
        // logits in the log2 domain; mask the tail and the causal triangle
        const bool edge = tb + kTileTokens > it.L - n_q;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
          const float sc = c2 * ks[sub];
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              float v = s[sub][rb][i] * sc;
              if (edge) {
                const int tok = tb + 16 * sub + 4 * g4 + i;
                const int r = 16 * rb + n;
                const int last = it.L - n_q + (r < R ? r / G : n_q - 1);   // padded rows: any finite row
                if (tok > last) v = -INFINITY;
              }
              s[sub][rb][i] = v;
            }
          }
        }
        bf16x8 p[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          float mx = fmaxf(fmaxf(fmaxf(s[0][rb][0], s[0][rb][1]), fmaxf(s[0][rb][2], s[0][rb][3])),
                           fmaxf(fmaxf(s[1][rb][0], s[1][rb][1]), fmaxf(s[1][rb][2], s[1][rb][3])));
          mx = fmaxf(mx, xor16(mx));
          mx = fmaxf(mx, xor32(mx));
          const float m_new = fmaxf(m_run[rb], mx);
          const float m_use = (m_new == -INFINITY) ? 0.f : m_new;     // row sees nothing yet
          const float alpha = exp2f(m_run[rb] - m_use);               // exp2(-inf) = 0 on the first tile
          f32x4 p0, p1;
          float sum = 0.f;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            p0[i] = exp2f(s[0][rb][i] - m_use);
            p1[i] = exp2f(s[1][rb][i] - m_use);
            sum += p0[i] + p1[i];
          }
          l_run[rb] = l_run[rb] * alpha + sum;
          m_run[rb] = m_new;
#pragma unroll
          for (int d = 0; d < 8; ++d) o[rb][d] *= alpha;
          if constexpr (FP8) { p0 *= vs[0]; p1 *= vs[1]; }
          p[rb] = pack_p(p0, p1);
        }
        tile_pv<RB>(vtile, p, o, lane);
      }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        l_run[rb] += xor16(l_run[rb]);
        l_run[rb] += xor32(l_run[rb]);
      }
    }

    // ---- merge the four wavefronts' partials ----
    if (g4 == 0) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        s_m[wave][16 * rb + n] = m_run[rb];
        s_l[wave][16 * rb + n] = l_run[rb];
      }
    }
    __syncthreads();
    float m_all[RB], l_all[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float m = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) m = fmaxf(m, s_m[w][16 * rb + n]);
      const float m_use = (m == -INFINITY) ? 0.f : m;
      float l = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) l += s_l[w][16 * rb + n] * exp2f(s_m[w][16 * rb + n] - m_use);
      m_all[rb] = m;
      l_all[rb] = l;
      const float mine = exp2f(m_run[rb] - m_use);
#pragma unroll
      for (int d = 0; d < 8; ++d) o[rb][d] *= mine;
    }
    // tree sum of O through LDS: waves 2,3 -> 0,1 ; wave 1 -> 0
    f32x4* xch = reinterpret_cast<f32x4*>(smem);
    constexpr int kPerWave = RB * 8 * 64;      // f32x4 slots
#pragma unroll
    for (int round = 0; round < 2; ++round) {
      const int senders_from = round == 0 ? 2 : 1;
      const int senders_to = round == 0 ? 4 : 2;
      __syncthreads();
      if (wave >= senders_from && wave < senders_to) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int d = 0; d < 8; ++d) xch[(wave - senders_from) * kPerWave + (rb * 8 + d) * 64 + lane] = o[rb][d];
      }
      __syncthreads();
      if (wave < senders_to - senders_from && wave < senders_from) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int d = 0; d < 8; ++d) o[rb][d] += xch[wave * kPerWave + (rb * 8 + d) * 64 + lane];
      }
    }
    if (wave == 0) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const int r = 16 * rb + n;
        if (g4 == 0) {
          ws.part_m[static_cast<int64_t>(id) * (RB * 16) + r] = m_all[rb];
          ws.part_l[static_cast<int64_t>(id) * (RB * 16) + r] = l_all[rb];
        }
        if (r < R) {
          float* dst = ws.part_o + (static_cast<int64_t>(id) * R + r) * kHeadDim;
#pragma unroll
          for (int db = 0; db < 8; ++db) *reinterpret_cast<f32x4*>(dst + 16 * db + 4 * g4) = o[rb][db];
        }
      }
    }
    __syncthreads();      // the tiles are reused by the next item
  }
}

// ---------------------------------------------------------------- merge -----
template <int RB>
__global__ __launch_bounds__(kThreads) void verify_merge_mfma(KvView kv, int n_q, FastWs ws, uint16_t* out, float* lse_out) {
  const int b = blockIdx.y, g = blockIdx.x;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int nc = chunks_of(kv.seq_lens[b]);
  const int first = ws.item_base[b] + g * nc;
  for (int idx = threadIdx.x; idx < R * (kHeadDim / 4); idx += kThreads) {
    const int r = idx / (kHeadDim / 4), d4 = idx - r * (kHeadDim / 4);
    float m = -INFINITY;
    for (int c = 0; c < nc; ++c) m = fmaxf(m, ws.part_m[static_cast<int64_t>(first + c) * (RB * 16) + r]);
    float l = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < nc; ++c) {
      const float w = exp2f(ws.part_m[static_cast<int64_t>(first + c) * (RB * 16) + r] - m);
      l = fmaf(ws.part_l[static_cast<int64_t>(first + c) * (RB * 16) + r], w, l);
      const f32x4 v = *reinterpret_cast<const f32x4*>(ws.part_o + (static_cast<int64_t>(first + c) * R + r) * kHeadDim + 4 * d4);
      acc += v * w;
    }
    const float inv = 1.0f / l;
    const int i = r / G, hg = r - i * G;
    const int64_t row = (static_cast<int64_t>(b) * n_q + i) * kv.num_q_heads + g * G + hg;
    u32x2 packed;
    packed.x = f32_to_bf16(acc.x * inv) | (static_cast<uint32_t>(f32_to_bf16(acc.y * inv)) << 16);
    packed.y = f32_to_bf16(acc.z * inv) | (static_cast<uint32_t>(f32_to_bf16(acc.w * inv)) << 16);
    *reinterpret_cast<u32x2*>(out + row * kHeadDim + 4 * d4) = packed;
    if (d4 == 0) {
      const float lse2 = m + log2f(l);
      ws.lse2[(static_cast<int64_t>(b) * kv.num_kv_heads + g) * (RB * 16) + r] = lse2;
      if (lse_out) lse_out[row] = lse2 * kLn2;
    }
  }
}

// --------------------------------------------------------------- scores -----
// K only: S^T again, p = exp2(s - lse2[row]) is the exact softmax probability;
// the mean over the R rows is a sum over the 16 lanes of an MFMA row block.
template <int RB, bool FP8>
__global__ __launch_bounds__(kThreads, 2) void verify_scores_mfma(KvView kv, const uint16_t* q, int n_q, FastWs ws,
                                                                  float* scores, int64_t score_stride) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  __shared__ int s_item;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, g4 = lane >> 4;
  uint8_t* ktile = smem + wave * kWaveLds;
  uint8_t* vtile = ktile + kKTileBytes;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const float c2 = kv.sm_scale * kLog2e;
  const float inv_r = 1.0f / static_cast<float>(R);
  const int total = ws.ctrl[2];
  for (;;) {
    if (threadIdx.x == 0) s_item = atomicAdd(&ws.ctrl[1], 1);
    __syncthreads();
    const int id = s_item;
    __syncthreads();
    if (id >= total) break;
    const Item it = decode_item(kv, ws, id);
    const int ntiles = (it.t_end - it.t_begin + kTileTokens - 1) / kTileTokens;
    if (wave >= ntiles) continue;
    bf16x8 qf[RB][4];
    load_q_frags<RB>(kv, q, n_q, G, R, it, qf, lane);
    float lse2[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      lse2[rb] = ws.lse2[(static_cast<int64_t>(it.b) * kv.num_kv_heads + it.g) * (RB * 16) + 16 * rb + n];
    const int pg = load_page_ids(kv, it, lane);
    float* dst = scores + (static_cast<int64_t>(it.b) * kv.num_kv_heads + it.g) * score_stride;
    TileRegs<FP8> regs;
    issue_tile<FP8>(kv, it, it.t_begin + wave * kTileTokens, pg, regs, lane);
    for (int ti = wave; ti < ntiles; ti += kWaves) {
      const int tb = it.t_begin + ti * kTileTokens;
      tile_to_lds<FP8>(regs, ktile, vtile, lane);
      float ks[2] = {1.f, 1.f}, vs[2] = {1.f, 1.f};
      if constexpr (FP8) tile_scales(kv, it, tb, pg, ks, vs);
      if (ti + kWaves < ntiles) issue_tile<FP8>(kv, it, tb + kWaves * kTileTokens, pg, regs, lane);
      f32x4 s[2][RB];
      tile_qk<RB>(ktile, qf, s, lane);
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const float sc = c2 * ks[sub];
        f32x4 tot = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          const int r = 16 * rb + n;
          const int last = it.L - n_q + r / G;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int tok = tb + 16 * sub + 4 * g4 + i;
            const float pv = exp2f(s[sub][rb][i] * sc - lse2[rb]);
            tot[i] += (r < R && tok <= last) ? pv : 0.f;
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) tot[i] = row16_sum(tot[i]) * inv_r;
        const int tok0 = tb + 16 * sub + 4 * g4;
        if (n == 0) {
          if (tok0 + 3 < it.L) {
            *reinterpret_cast<f32x4*>(dst + tok0) = tot;
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (tok0 + i < it.L) dst[tok0 + i] = tot[i];
          }
        }
      }
    }
  }
}

FastWs carve(const KvView& kv, int n_q, void* workspace, size_t* total_bytes) {
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const size_t R = static_cast<size_t>(n_q) * G;
  const size_t rpad = (R + 15) / 16 * 16;
  const size_t max_items = static_cast<size_t>(kv.batch) * kv.num_kv_heads * chunks_of(kv.max_seq_len);
  char* p = static_cast<char*>(workspace);
  size_t off = 0;
  FastWs w;
  auto take = [&](size_t bytes) { char* r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
  w.ctrl = reinterpret_cast<int32_t*>(take(64 * 4));
  w.item_base = reinterpret_cast<int32_t*>(take((static_cast<size_t>(kv.batch) + 1) * 4));
  w.items = reinterpret_cast<int32_t*>(take(max_items * 8));
  w.part_m = reinterpret_cast<float*>(take(max_items * rpad * 4));
  w.part_l = reinterpret_cast<float*>(take(max_items * rpad * 4));
  w.part_o = reinterpret_cast<float*>(take(max_items * R * kHeadDim * 4));
  w.lse2 = reinterpret_cast<float*>(take(static_cast<size_t>(kv.batch) * kv.num_kv_heads * rpad * 4));
  w.max_items = static_cast<int32_t>(max_items);
  if (total_bytes) *total_bytes = off;
  return w;
}

int g_num_cus = 0;
int persistent_grid() {
  if (g_num_cus == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    g_num_cus = cus;
  }
  return 2 * g_num_cus;
}

template <int RB, bool FP8>
hipError_t run(const VerifyArgs& a, hipStream_t st) {
  const KvView& kv = a.kv;
  const FastWs ws = carve(kv, a.n_q, a.workspace, nullptr);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&verify_split_mfma<RB, FP8>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&verify_scores_mfma<RB, FP8>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const uint16_t* q = static_cast<const uint16_t*>(a.q);
  const int grid = persistent_grid();
  {
    KernelTimer t("verify_plan", st);
    hipLaunchKernelGGL(verify_plan, dim3(1), dim3(1024), 0, st, kv, ws);
  }
  {
    KernelTimer t("verify_split_mfma", st);
    hipLaunchKernelGGL((verify_split_mfma<RB, FP8>), dim3(grid), dim3(kThreads), kLdsBytes, st, kv, q, a.n_q, ws);
  }
  {
    KernelTimer t("verify_merge_mfma", st);
    hipLaunchKernelGGL((verify_merge_mfma<RB>), dim3(kv.num_kv_heads, kv.batch), dim3(kThreads), 0, st, kv, a.n_q, ws,
                       static_cast<uint16_t*>(a.out), a.lse);
  }
  if (a.scores) {
    KernelTimer t("verify_scores_mfma", st);
    hipLaunchKernelGGL((verify_scores_mfma<RB, FP8>), dim3(grid), dim3(kThreads), kLdsBytes, st, kv, q, a.n_q, ws,
                       a.scores, a.score_stride);
  }
  return hipGetLastError();
}

}  // namespace

bool verify_mfma_supported(const VerifyArgs& a) {
  const KvView& kv = a.kv;
  if (a.q_dtype != PILLAR_BF16) return false;
  if (a.kv_dtype != PILLAR_BF16 && a.kv_dtype != PILLAR_FP8_E4M3) return false;
  if (kv.head_dim != kHeadDim || kv.page_size < 16) return false;
  const int64_t align = a.kv_dtype == PILLAR_BF16 ? 8 : 16;      // elements per 16 bytes
  if (kv.stride_page % align || kv.stride_head % align || kv.stride_slot % align) return false;
  if ((reinterpret_cast<uintptr_t>(kv.k_pool) | reinterpret_cast<uintptr_t>(kv.v_pool) | reinterpret_cast<uintptr_t>(a.q) |
       reinterpret_cast<uintptr_t>(a.out)) & 15u)
    return false;
  if (a.scores && ((reinterpret_cast<uintptr_t>(a.scores) & 15u) || (a.score_stride & 3))) return false;
  if (kChunk / kv.page_size > 64) return false;
  return true;
}

size_t verify_mfma_workspace(const KvView& kv, int n_q) {
  size_t total = 0;
  carve(kv, n_q, nullptr, &total);
  return total;
}

hipError_t launch_verify_mfma(const VerifyArgs& a, hipStream_t s) {
  const int G = a.kv.num_q_heads / a.kv.num_kv_heads;
  const int rb = (a.n_q * G + 15) / 16;
  const bool fp8 = a.kv_dtype == PILLAR_FP8_E4M3;
#define PILLAR_CASE(N)                                      \
  if (rb == N) return fp8 ? run<N, true>(a, s) : run<N, false>(a, s);
  PILLAR_CASE(1)
  PILLAR_CASE(2)
  PILLAR_CASE(3)
  PILLAR_CASE(4)
#undef PILLAR_CASE
  return hipErrorInvalidValue;
}

}  // namespace pillar
