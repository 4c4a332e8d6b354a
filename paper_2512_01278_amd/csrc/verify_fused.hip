// Verification attention with the score statistic, in one persistent kernel
// (bf16 queries, bf16 or fp8 KV, head_dim 128, pages of >= 16 tokens).
//
// Paper Section 4.1: the verification pass yields, besides its output, the
// softmax probabilities of the k+1 verification rows, averaged over rows and
// over the query heads of one GQA group; Top-K reads that statistic next.  A
// probability needs the row's log-sum-exp over the WHOLE context, which is
// only known once every token has been seen.  The paper caches logits and
// log-sum-exp and rematerialises; here the logits are recomputed instead,
// because re-reading K is nearly free on this chip when it happens soon after
// the first read: the Infinity Cache (256 MB, memory side) serves the second
// read at HBM-like bandwidth ON TOP of what HBM delivers (measured: streaming
// 2 GB while re-reading data touched 64 MB earlier costs about 10 % more time
// than streaming alone).  A logit dump would add 16..60 % HBM traffic.
//
// Each (request, KV head) is cut into slices of `slice_tokens` tokens, and a
// slice is the work of ONE wavefront (a workgroup is one wavefront: nothing in
// this kernel needs a barrier).  The wavefront visits its slice twice:
//   phase 1  K only: S^T = K Q^T on the matrix cores, running (max, sum) per
//            row -> the slice's (m, l), published.  The last slice of a pair
//            to publish combines all (m, l) into the final log-sum-exp.
//   wait     until the pair's log-sum-exp is there.  The slices of a pair are
//            handed out together, so this takes a few microseconds, during
//            which the other wavefronts of the compute unit keep HBM busy.
//   phase 2  K (now from the Infinity Cache) and V: p = exp2(s - lse) is the
//            exact probability, so the score statistic is written directly,
//            and O = sum p V needs no running maximum and no rescaling; slice
//            partials of O add linearly and the last slice to finish sums them.
//
// Progress: slices are handed out by one atomic ticket in pair-major order.  A
// wavefront holds one slice; it publishes phase 1 before it waits, and waits
// only for slices of its own pair.  The lowest slice nobody has taken yet
// belongs to some pair; every wavefront waiting on another pair is released
// once that pair's (already taken, never waiting) phase-1 work is done, and
// the pair itself cannot occupy every wavefront as long as it has no more
// slices than there are resident wavefronts: the host selects this kernel only
// below that bound.  The wait is a bounded spin that poisons the slice's
// scores with NaN instead of hanging.
#include "launch.hpp"
#include "mfma_tile.hpp"
#include "verify_stream.hpp"

namespace pillar {
namespace {

constexpr int kThreads = 64;                   // one wavefront per workgroup
constexpr int kSpinLimit = 1 << 20;
constexpr int kDefaultSlice = 512;
constexpr int kMaxBatchInLds = 4096;
constexpr int kWavesPerCu = 8;
constexpr uint32_t kNotYet = 0xffffffffu;      // bit pattern no computed log-sum-exp has

struct FusedWs {
  int32_t* ctrl;        // [0] ticket  [1] slice count  [2] timeouts
  int32_t* slice_base;  // [B+1] first slice of request b; its slices are head-major
  int32_t* slices;      // [max_slices][4] = {b, g, c, L}
  int32_t* cnt1;        // [pairs] slices that finished phase 1
  int32_t* cnt2;        // [pairs] slices that finished phase 2
  float* part_m;        // [max_slices][RB*16]  log2 domain
  float* part_l;        // [max_slices][RB*16]
  float* part_o;        // [max_slices][R][128]
  float* lse2;          // [pairs][RB*16]       log2 domain; kNotYet until the pair's phase 1 is complete
  int32_t rows_pad;     // RB*16
  int32_t grid;         // wavefronts in the persistent grid
  int32_t slice_tokens;
  int32_t max_slices;
  int32_t debug;
  long long* trace;     // [8192] timestamps of workgroup 0 (tracing builds only)
};

__host__ __device__ inline int slices_of(int len, int slice_tokens) { return (len + slice_tokens - 1) / slice_tokens; }

// ---------------------------------------------------------------- plan ------
__global__ __launch_bounds__(1024) void fused_plan(KvView kv, FusedWs ws) {
  __shared__ int32_t base[kMaxBatchInLds + 1];
  __shared__ int32_t scan[1024];
  __shared__ int32_t carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int b0 = 0; b0 < kv.batch; b0 += 1024) {
    const int b = b0 + threadIdx.x;
    const int mine = b < kv.batch ? slices_of(kv.seq_lens[b], ws.slice_tokens) * kv.num_kv_heads : 0;
    scan[threadIdx.x] = mine;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int v = threadIdx.x >= o ? scan[threadIdx.x - o] : 0;
      __syncthreads();
      scan[threadIdx.x] += v;
      __syncthreads();
    }
    if (b < kv.batch) base[b] = carry + scan[threadIdx.x] - mine;
    __syncthreads();
    if (threadIdx.x == 1023) carry += scan[1023];
    __syncthreads();
  }
  const int total = carry;
  if (threadIdx.x == 0) base[kv.batch] = total;
  __syncthreads();
  for (int b = threadIdx.x; b <= kv.batch; b += 1024) ws.slice_base[b] = base[b];
  for (int j = threadIdx.x; j < total; j += 1024) {
    int lo = 0, hi = kv.batch - 1;            // last b with base[b] <= j
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (base[mid] <= j) lo = mid; else hi = mid - 1;
    }
    const int L = kv.seq_lens[lo];
    const int ns = slices_of(L, ws.slice_tokens);
    const int rel = j - base[lo];
    int4 e;
    e.x = lo;
    e.y = rel / ns;
    e.z = rel - e.y * ns;
    e.w = L;
    reinterpret_cast<int4*>(ws.slices)[j] = e;
  }
  const int pairs = kv.batch * kv.num_kv_heads;
  for (int p = threadIdx.x; p < pairs; p += 1024) {
    ws.cnt1[p] = 0;
    ws.cnt2[p] = 0;
  }
  for (int i = threadIdx.x; i < pairs * ws.rows_pad; i += 1024) reinterpret_cast<uint32_t*>(ws.lse2)[i] = kNotYet;
  if (threadIdx.x == 0) {
    ws.ctrl[0] = ws.grid;                   // wavefront w starts on slice w
    ws.ctrl[1] = total;
    ws.ctrl[2] = 0;
  }
}

// ------------------------------------------------------------- helpers ------
struct Slice {
  int id, b, g, c, L, t_begin, t_end, nslices, first, pair;
};

__device__ __forceinline__ int4 slice_entry(const FusedWs& ws, int id) { return reinterpret_cast<const int4*>(ws.slices)[id]; }

__device__ __forceinline__ Slice make_slice(const KvView& kv, const FusedWs& ws, int id, const int4& e) {
  Slice s;                                  // the same for every lane: keep it in scalar registers
  s.id = __builtin_amdgcn_readfirstlane(id);
  s.b = __builtin_amdgcn_readfirstlane(e.x);
  s.g = __builtin_amdgcn_readfirstlane(e.y);
  s.c = __builtin_amdgcn_readfirstlane(e.z);
  s.L = __builtin_amdgcn_readfirstlane(e.w);
  s.t_begin = s.c * ws.slice_tokens;
  s.t_end = min(s.L, s.t_begin + ws.slice_tokens);
  s.nslices = slices_of(s.L, ws.slice_tokens);
  s.first = s.id - s.c;                     // slice 0 of this (request, head)
  s.pair = s.b * kv.num_kv_heads + s.g;
  return s;
}

// tells the compiler that a slice descriptor is the same in every lane
__device__ __forceinline__ Slice uniform(const Slice& s) {
  Slice u;
  u.id = __builtin_amdgcn_readfirstlane(s.id);
  u.b = __builtin_amdgcn_readfirstlane(s.b);
  u.g = __builtin_amdgcn_readfirstlane(s.g);
  u.c = __builtin_amdgcn_readfirstlane(s.c);
  u.L = __builtin_amdgcn_readfirstlane(s.L);
  u.t_begin = __builtin_amdgcn_readfirstlane(s.t_begin);
  u.t_end = __builtin_amdgcn_readfirstlane(s.t_end);
  u.nslices = __builtin_amdgcn_readfirstlane(s.nslices);
  u.first = __builtin_amdgcn_readfirstlane(s.first);
  u.pair = __builtin_amdgcn_readfirstlane(s.pair);
  return u;
}

template <int RB>
__device__ __forceinline__ void load_q(const KvView& kv, const uint16_t* q, int n_q, int G, int R, const Slice& it,
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

// lane j: page id of page (first page of the slice + j) of the request
__device__ __forceinline__ int load_pages(const KvView& kv, const Slice& it, int lane) {
  const int first_page = it.t_begin >> kv.page_shift;
  const int last_page = (it.L - 1) >> kv.page_shift;
  return kv.block_table[static_cast<int64_t>(it.b) * kv.block_table_stride + min(first_page + lane, last_page)];
}

// Issues the loads of the tile at token tb: K rows into rk, and V rows into rv
// when WITH_V.  A 16-token group lies in one page whose id is wave-uniform, so
// the address is a scalar base per group plus a 32-bit per-lane offset.  Groups
// (or rows) beyond the end of the sequence read the last page of the request:
// pages are whole, so the rows exist; the caller masks them.
template <bool FP8, bool WITH_V, bool WITH_K = true>
__device__ __forceinline__ void issue_rows(const KvView& kv, const Slice& it, int tb, int pg, const LaneGeom<FP8>& geo,
                                           u32x4 (&rk)[TileRegs<FP8>::kLoads], u32x4 (&rv)[TileRegs<FP8>::kLoads]) {
  constexpr int kLoads = TileRegs<FP8>::kLoads;
  constexpr int kPerGroup = kLoads / 2;
  const int esz = FP8 ? 1 : 2;
  const int first_page = it.t_begin >> kv.page_shift;
  const int last_page = (it.L - 1) >> kv.page_shift;
#pragma unroll
  for (int grp = 0; grp < 2; ++grp) {
    const int tok0 = tb + 16 * grp;
    const int page = __builtin_amdgcn_readlane(pg, min(tok0 >> kv.page_shift, last_page) - first_page);
    const int64_t base = (static_cast<int64_t>(page) * kv.stride_page + static_cast<int64_t>(it.g) * kv.stride_head +
                          static_cast<int64_t>(tok0 & (kv.page_size - 1)) * kv.stride_slot) * esz;
    const char* gk = static_cast<const char*>(kv.k_pool) + base;
    const char* gv = static_cast<const char*>(kv.v_pool) + base;
#pragma unroll
    for (int u = 0; u < kPerGroup; ++u) {
      const uint32_t off = geo.lane_off + u * geo.row_step;
      if constexpr (WITH_K) rk[grp * kPerGroup + u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gk + off));
      if constexpr (WITH_V) rv[grp * kPerGroup + u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gv + off));
    }
  }
}

// fp8: dequantisation scales of the two 16-token halves of a tile
__device__ __forceinline__ void half_scales(const KvView& kv, const Slice& it, int tb, int pg, const float* table, float (&sc)[2]) {
  const int first_page = it.t_begin >> kv.page_shift;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const int tok = min(tb + 16 * sub, it.L - 1);
    const int page = __builtin_amdgcn_readlane(pg, (tok >> kv.page_shift) - first_page);
    sc[sub] = table[static_cast<int64_t>(page) * kv.num_kv_heads + it.g];
  }
}

// Stores that another wavefront (possibly on another XCD, behind another L2)
// will read are written through to memory (sc1), so publishing them needs no
// L2 write-back, only a wait for the acknowledgements; the reader either loads
// with sc1 or invalidates once (acquire fence) before plain loads.
__device__ __forceinline__ void publish(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float peek(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void wait_stores() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

// eight 16-byte write-through stores (dims 16db + 4g .. +3 of one row); the caller waits for the acknowledgements
__device__ __forceinline__ void publish_row(float* p, const f32x4 (&v)[8]) {
  asm volatile(
      "global_store_dwordx4 %0, %1, off sc1\n\t"
      "global_store_dwordx4 %0, %2, off offset:64 sc1\n\t"
      "global_store_dwordx4 %0, %3, off offset:128 sc1\n\t"
      "global_store_dwordx4 %0, %4, off offset:192 sc1\n\t"
      "global_store_dwordx4 %0, %5, off offset:256 sc1\n\t"
      "global_store_dwordx4 %0, %6, off offset:320 sc1\n\t"
      "global_store_dwordx4 %0, %7, off offset:384 sc1\n\t"
      "global_store_dwordx4 %0, %8, off offset:448 sc1"
      :
      : "v"(p), "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7])
      : "memory");
}

__device__ __forceinline__ int tiles_of(const Slice& s) { return (s.t_end - s.t_begin + kTileTokens - 1) / kTileTokens; }

#ifdef PILLAR_TRACING
#define PILLAR_TRACE(tag) do { if ((blockIdx.x & 255) == 0 && blockIdx.x < 2048 && threadIdx.x == 0 && tr_n < 1022) { ws.trace[(blockIdx.x >> 8) * 1024 + tr_n++] = (static_cast<long long>(tag) << 48) | (wall_clock64() & 0xffffffffffffll); } } while (0)
#else
#define PILLAR_TRACE(tag) do { } while (0)
#endif

// ---------------------------------------------------------------- kernel ----
template <int RB, bool FP8>
__global__ __launch_bounds__(kThreads, RB >= 3 ? 1 : 2) void verify_fused_mfma(KvView kv, const uint16_t* q, int n_q, FusedWs ws,
                                                                 uint16_t* out, float* lse_out, float* scores,
                                                                 int64_t score_stride) {
  // one tile buffer: K rows in phase 1; in phase 2 K rows, then (once S^T is done) the V rows of the same tile
  __shared__ __attribute__((aligned(16))) uint8_t s_tile[kVTileBytes];
  __shared__ __attribute__((aligned(16))) uint8_t s_q[(RB * 16 + 1) * kKRow];
  const int lane = threadIdx.x;
  const int n = lane & 15, g4 = lane >> 4;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const float c2 = kv.sm_scale * kLog2e;
  const float inv_r = 1.0f / static_cast<float>(R);
  const int total = ws.ctrl[1];
  const LaneGeom<FP8> geo = lane_geom<FP8>(kv, lane);
  constexpr int kLoads = TileRegs<FP8>::kLoads;
  constexpr int kQIters = ((RB * 16 + 1) * 16 + kThreads - 1) / kThreads;
  [[maybe_unused]] int tr_n = 1;

  // The first slice of a wavefront is its own number (the ticket counter starts behind the
  // grid), so the start of the kernel does not queue up on one atomic.
  Slice cur = {}, prev = {};
  int cur_pg = 0, prev_pg = 0;
  bool has_cur = static_cast<int>(blockIdx.x) < total, has_prev = false;
  if (has_cur) {
    cur = make_slice(kv, ws, blockIdx.x, slice_entry(ws, blockIdx.x));
    cur_pg = load_pages(kv, cur, lane);
  }

  // Software pipeline over the slices of this wavefront: phase 1 of the slice just taken runs
  // between phase 1 and phase 2 of the previous one, so that the publish / combine round trips
  // of a pair are hidden behind streaming instead of being waited for.
  u32x4 rk[kLoads], rv[kLoads];
  while (has_cur || has_prev) {
    PILLAR_TRACE(1);
    // =================== phase 1: K only -> (m, l) of the slice ===================
    // K tiles travel two deep: even tiles through rk, odd tiles through rv (V is not read in
    // this phase).  Behind the first tile, the Q rows of the previous slice's pair go to LDS
    // for its phase 2.
    bf16x8 qf[RB][4];
    u32x4 unused[kLoads];
    const int nt1 = has_cur ? tiles_of(cur) : 0;
    if (has_cur) issue_rows<FP8, false>(kv, cur, cur.t_begin, cur_pg, geo, rk, unused);
    if (has_prev) {
      u32x4 qtmp[kQIters];
#pragma unroll
      for (int j = 0; j < kQIters; ++j) {
        const int ch = lane + kThreads * j;
        const int r = ch >> 4, c = ch & 15;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r < R) {
          const int i = r / G, hg = r - i * G;
          v = *reinterpret_cast<const u32x4*>(q + ((static_cast<int64_t>(prev.b) * n_q + i) * kv.num_q_heads + prev.g * G + hg) * kHeadDim + 8 * c);
        }
        qtmp[j] = v;
      }
#pragma unroll
      for (int j = 0; j < kQIters; ++j) {
        const int ch = lane + kThreads * j;
        if (ch < (R + 1) * 16) *reinterpret_cast<u32x4*>(s_q + k_lds_addr(ch >> 4, ch & 15)) = qtmp[j];
      }
    }
    if (has_cur) {
      if (nt1 > 1) issue_rows<FP8, false>(kv, cur, cur.t_begin + kTileTokens, cur_pg, geo, rv, unused);
      load_q<RB>(kv, q, n_q, G, R, cur, qf, lane);
    }
    PILLAR_TRACE(2);
    if (has_cur) {
      const Slice& it = cur;
      const int pg = cur_pg;
      const int nt = nt1;
      float m_run[RB], l_run[RB];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) { m_run[rb] = -INFINITY; l_run[rb] = 0.f; }
      auto phase1_tile = [&](int ti, u32x4 (&regs)[kLoads]) {
        const int tb = it.t_begin + ti * kTileTokens;
        if (ws.debug & 256) {                      // experiment: memory traffic only
          u32x4 x = regs[0];
#pragma unroll
          for (int u = 1; u < kLoads; ++u) x ^= regs[u];
          if (ti + 2 < nt) issue_rows<FP8, false>(kv, it, tb + 2 * kTileTokens, pg, geo, regs, unused);
          l_run[0] += __uint_as_float((x.x ^ x.y ^ x.z ^ x.w) & 0x3fffffffu);
          return;
        }
        rows_to_lds<FP8, false>(regs, s_tile, lane);
        float ks[2] = {1.f, 1.f};
        if constexpr (FP8) half_scales(kv, it, tb, pg, kv.k_scale, ks);
        if (ti + 2 < nt) issue_rows<FP8, false>(kv, it, tb + 2 * kTileTokens, pg, geo, regs, unused);
        f32x4 s[2][RB];
        tile_qk<RB>(s_tile, qf, s, lane);
        const bool edge = tb + kTileTokens > it.L - n_q;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
          for (int sub = 0; sub < 2; ++sub) s[sub][rb] *= c2 * ks[sub];
          if (edge) {
            const int r = 16 * rb + n;
            const int last = it.L - n_q + (r < R ? r / G : n_q - 1);
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
              for (int i = 0; i < 4; ++i)
                if (tb + 16 * sub + 4 * g4 + i > last) s[sub][rb][i] = -INFINITY;
          }
          const float mx = fmaxf(fmaxf(fmaxf(s[0][rb][0], s[0][rb][1]), fmaxf(s[0][rb][2], s[0][rb][3])),
                                 fmaxf(fmaxf(s[1][rb][0], s[1][rb][1]), fmaxf(s[1][rb][2], s[1][rb][3])));
          const float m_new = fmaxf(m_run[rb], mx);
          const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
          float sum = 0.f;
#pragma unroll
          for (int i = 0; i < 4; ++i) sum += fast_exp2(s[0][rb][i] - m_use) + fast_exp2(s[1][rb][i] - m_use);
          l_run[rb] = l_run[rb] * fast_exp2(m_run[rb] - m_use) + sum;
          m_run[rb] = m_new;
        }
      };
      for (int ti = 0; ti < ((ws.debug & 512) ? 0 : nt); ti += 2) {
        phase1_tile(ti, rk);
        if (ti + 1 < nt) phase1_tile(ti + 1, rv);
      }
      PILLAR_TRACE(3);
      // the tile registers are free: the first tile of the previous slice's phase 2 travels
      // while this slice's (m, l) are published
      if (has_prev) issue_rows<FP8, true>(kv, prev, prev.t_begin, prev_pg, geo, rk, rv);
      if (!(ws.debug & 8)) {
      // the 4 token groups of a row -> the slice's (m, l), published by the lanes of group 0
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        float mx = fmaxf(m_run[rb], xor16(m_run[rb]));
        mx = fmaxf(mx, xor32(mx));
        const float m_use = (mx == -INFINITY) ? 0.f : mx;
        float l = l_run[rb] * fast_exp2(m_run[rb] - m_use);
        l += xor16(l);
        l += xor32(l);
        if (g4 == 0) {
          publish(&ws.part_m[static_cast<int64_t>(it.id) * (RB * 16) + 16 * rb + n], mx);
          publish(&ws.part_l[static_cast<int64_t>(it.id) * (RB * 16) + 16 * rb + n], l);
        }
      }
      wait_stores();
      int old = 0;
      if (lane == 0) old = atomicAdd(&ws.cnt1[it.pair], 1);
      old = __builtin_amdgcn_readfirstlane(old);
      if (old == it.nslices - 1) {               // every slice of the pair has published: final log-sum-exp
        if (lane < RB * 16) {
          const float* pm = ws.part_m + static_cast<int64_t>(it.first) * (RB * 16) + lane;
          const float* pl = ws.part_l + static_cast<int64_t>(it.first) * (RB * 16) + lane;
          float m = -INFINITY, l = 0.f;
          for (int c0 = 0; c0 < it.nslices; c0 += 8) {
            float pmv[8], plv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              const int c = min(c0 + u, it.nslices - 1);
              pmv[u] = peek(pm + c * (RB * 16));
              plv[u] = peek(pl + c * (RB * 16));
            }
            float mb = m;
#pragma unroll
            for (int u = 0; u < 8; ++u) if (c0 + u < it.nslices) mb = fmaxf(mb, pmv[u]);
            const float mb_use = (mb == -INFINITY) ? 0.f : mb;
            l *= fast_exp2(m - mb_use);
#pragma unroll
            for (int u = 0; u < 8; ++u) if (c0 + u < it.nslices) l += plv[u] * fast_exp2(pmv[u] - mb_use);
            m = mb;
          }
          // rows beyond R get +inf so that their probabilities vanish in phase 2
          const float v = lane < R ? m + log2f(l) : INFINITY;
          publish(&ws.lse2[static_cast<int64_t>(it.pair) * (RB * 16) + lane], v);
          if (lse_out && lane < R) {
            const int i = lane / G, hg = lane - i * G;
            lse_out[(static_cast<int64_t>(it.b) * n_q + i) * kv.num_q_heads + it.g * G + hg] = v * kLn2;
          }
        }
      }
      }
    } else if (has_prev) {
      issue_rows<FP8, true>(kv, prev, prev.t_begin, prev_pg, geo, rk, rv);
    }
    PILLAR_TRACE(4);

    int next_ticket = total;
    bool took = false;
    Slice nxt = {};
    int nxt_pg = 0;
    bool has_next = false;

    if (has_prev) {
      const Slice& it = prev;
      const int pg = prev_pg;
      const int nt = tiles_of(it);
      // ====== the previous slice's pair should be complete by now: its log-sum-exp replaces the
      // ====== "not yet" pattern the plan kernel left there
      float lse2[RB];
      int spins = 0;
      for (;;) {
        bool miss = false;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          lse2[rb] = peek(&ws.lse2[static_cast<int64_t>(it.pair) * (RB * 16) + 16 * rb + n]);
          miss |= __float_as_uint(lse2[rb]) == kNotYet;
        }
        if (__builtin_amdgcn_readfirstlane(__any(miss) ? 1 : 0) == 0 || spins >= kSpinLimit || (ws.debug & 8)) break;
        ++spins;
        __builtin_amdgcn_s_sleep(8);
      }
      const bool ok = __builtin_amdgcn_readfirstlane(spins) < kSpinLimit;
      PILLAR_TRACE(5);

      // ================= phase 2: scores and O (K again, and V) =================
      float* sdst = scores + (static_cast<int64_t>(it.b) * kv.num_kv_heads + it.g) * score_stride;
      if (ok) {
        f32x4 o[RB][8];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int d = 0; d < 8; ++d) o[rb][d] = f32x4{0.f, 0.f, 0.f, 0.f};
        // the next slice is reserved shortly before this one ends, so that its descriptor and
        // page list arrive while the results below are published
        const int take_at = max(nt - 2, 0);
        int next_v = total;
        for (int ti = 0; ti < nt; ++ti) {
          const int tb = it.t_begin + ti * kTileTokens;
          if (ti == take_at && has_cur) {
            if (lane == 0) next_v = atomicAdd(&ws.ctrl[0], 1);
            took = true;
          }
          if (ws.debug & 1024) continue;
          if (ws.debug & 256) {                      // experiment: memory traffic only
            u32x4 x = rk[0] ^ rv[0];
#pragma unroll
            for (int u = 1; u < kLoads; ++u) x ^= rk[u] ^ rv[u];
            if (ti + 1 < nt) issue_rows<FP8, true>(kv, it, tb + kTileTokens, pg, geo, rk, rv);
            o[0][0].x += __uint_as_float((x.x ^ x.y ^ x.z ^ x.w) & 0x3fffffffu);
            continue;
          }
          PILLAR_TRACE(20);
          rows_to_lds<FP8, false>(rk, s_tile, lane);
          // each register set goes back on the road as soon as its rows are in LDS
          if (ti + 1 < nt) issue_rows<FP8, false>(kv, it, tb + kTileTokens, pg, geo, rk, rv);
          float ks[2] = {1.f, 1.f}, vs[2] = {1.f, 1.f};
          if constexpr (FP8) { half_scales(kv, it, tb, pg, kv.k_scale, ks); half_scales(kv, it, tb, pg, kv.v_scale, vs); }
          f32x4 s[2][RB];
          tile_qk_ldsq<RB>(s_tile, s_q, R, s, lane);
          // the K rows are consumed: the V rows take their place
          if (tb + kTileTokens > it.L) zero_tail_rows<FP8>(rv, tb, it.L, geo);
          rows_to_lds<FP8, true>(rv, s_tile, lane);
          if (ti + 1 < nt) issue_rows<FP8, true, false>(kv, it, tb + kTileTokens, pg, geo, rk, rv);
          const bool edge = tb + kTileTokens > it.L - n_q;
          f32x4 tot[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
          bf16x8 p[RB];
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) {
            f32x4 pr[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
              const float sc = c2 * ks[sub];
#pragma unroll
              for (int i = 0; i < 4; ++i) pr[sub][i] = fast_exp2(fmaf(s[sub][rb][i], sc, -lse2[rb]));
            }
            if (edge) {
              const int r = 16 * rb + n;
              const int last = it.L - n_q + (r < R ? r / G : n_q - 1);
#pragma unroll
              for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                  if (tb + 16 * sub + 4 * g4 + i > last) pr[sub][i] = 0.f;
            }
            tot[0] += pr[0];
            tot[1] += pr[1];
            if constexpr (FP8) { pr[0] *= vs[0]; pr[1] *= vs[1]; }
            p[rb] = pack_p(pr[0], pr[1]);
          }
#pragma unroll
          for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
            for (int i = 0; i < 4; ++i) tot[sub][i] = row16_sum(tot[sub][i]) * inv_r;
            const int tok0 = tb + 16 * sub + 4 * g4;
            if (n == 0) {
              if (tok0 + 3 < it.L) {
                *reinterpret_cast<f32x4*>(sdst + tok0) = tot[sub];
              } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                  if (tok0 + i < it.L) sdst[tok0 + i] = tot[sub][i];
              }
            }
          }
          tile_pv<RB>(s_tile, p, o, lane);
          PILLAR_TRACE(25);
        }
        PILLAR_TRACE(6);
        int4 nxt_e = {0, 0, 0, 0};
        if (took) {
          next_ticket = __builtin_amdgcn_readfirstlane(next_v);
          has_next = next_ticket < total;
          if (has_next) nxt_e = slice_entry(ws, next_ticket);
        }
        if (it.nslices == 1 || (ws.debug & 8)) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) {
            const int r = 16 * rb + n;
            if (r < R && !(ws.debug & 8)) {
              const int i = r / G, hg = r - i * G;
              uint16_t* dst = out + ((static_cast<int64_t>(it.b) * n_q + i) * kv.num_q_heads + it.g * G + hg) * kHeadDim;
#pragma unroll
              for (int db = 0; db < 8; ++db) {
                u32x2 pk;
                pk.x = pack2(o[rb][db][0], o[rb][db][1]);
                pk.y = pack2(o[rb][db][2], o[rb][db][3]);
                *reinterpret_cast<u32x2*>(dst + 16 * db + 4 * g4) = pk;
              }
            }
          }
          if (has_next) {
            nxt = make_slice(kv, ws, next_ticket, nxt_e);
            nxt_pg = load_pages(kv, nxt, lane);
          }
        } else {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) {
            const int r = 16 * rb + n;
            if (r < R && !(ws.debug & 2)) publish_row(ws.part_o + (static_cast<int64_t>(it.id) * R + r) * kHeadDim + 4 * g4, o[rb]);
          }
          PILLAR_TRACE(61);
          wait_stores();
          PILLAR_TRACE(62);
          if (has_next) {                        // its descriptor has arrived with the acknowledgements
            nxt = make_slice(kv, ws, next_ticket, nxt_e);
            nxt_pg = load_pages(kv, nxt, lane);
          }
          int old = 0;
          if (lane == 0) old = atomicAdd(&ws.cnt2[it.pair], 1);
          old = __builtin_amdgcn_readfirstlane(old);
          PILLAR_TRACE(63);
          if (old == it.nslices - 1) {             // last slice of the pair: O = sum of the slice partials
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            for (int idx = lane; idx < R * (kHeadDim / 4); idx += kThreads) {
              const int r = idx / (kHeadDim / 4), d4 = idx - r * (kHeadDim / 4);
              f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
              for (int c = 0; c < it.nslices; ++c)
                acc += *reinterpret_cast<const f32x4*>(ws.part_o + (static_cast<int64_t>(it.first + c) * R + r) * kHeadDim + 4 * d4);
              const int i = r / G, hg = r - i * G;
              uint16_t* dst = out + ((static_cast<int64_t>(it.b) * n_q + i) * kv.num_q_heads + it.g * G + hg) * kHeadDim;
              u32x2 pk;
              pk.x = pack2(acc.x, acc.y);
              pk.y = pack2(acc.z, acc.w);
              *reinterpret_cast<u32x2*>(dst + 4 * d4) = pk;
            }
          }
        }
      } else {
        // the pair never became ready: make the failure visible instead of hanging
        if (lane == 0) atomicAdd(&ws.ctrl[2], 1);
        for (int t = it.t_begin + lane; t < it.t_end; t += kThreads) sdst[t] = __uint_as_float(0x7fc00000u);
      }
    }
    if (has_cur && !took) {                      // no phase 2 ran in this round: reserve the next slice now
      int v = 0;
      if (lane == 0) v = atomicAdd(&ws.ctrl[0], 1);
      next_ticket = __builtin_amdgcn_readfirstlane(v);
      has_next = next_ticket < total;
      if (has_next) {
        nxt = make_slice(kv, ws, next_ticket, slice_entry(ws, next_ticket));
        nxt_pg = load_pages(kv, nxt, lane);
      }
    }
    PILLAR_TRACE(7);
    prev = cur;
    prev_pg = cur_pg;
    has_prev = has_cur;
    cur = uniform(nxt);
    cur_pg = nxt_pg;
    has_cur = __builtin_amdgcn_readfirstlane(has_next ? 1 : 0) != 0;
  }
#ifdef PILLAR_TRACING
  if ((blockIdx.x & 255) == 0 && blockIdx.x < 2048 && threadIdx.x == 0) ws.trace[(blockIdx.x >> 8) * 1024] = tr_n;
#endif
}

// ------------------------------------------------ two-pass kernels ----------
// The same two phases as separate launches, one workgroup (one wavefront) per slice: the
// kernel boundary is the only synchronisation, so nothing is published, counted or waited for.
//   verify_lse_pass    phase 1 of every slice: (m, l) per row
//   verify_lse_combine per pair: final log-sum-exp (log2 domain in the workspace, natural in lse_out)
//   verify_score_pass  phase 2 of every slice: scores, and O (direct for one-slice pairs, else a partial)
//   verify_o_merge     per pair with several slices: O = sum of the partials
template <int RB, bool FP8>
__global__ __launch_bounds__(kThreads, 2) void verify_lse_pass(KvView kv, const uint16_t* q, int n_q, FusedWs ws) {
  __shared__ __attribute__((aligned(16))) uint8_t s_tile[kKTileBytes];
  if (static_cast<int>(blockIdx.x) >= ws.ctrl[1]) return;      // the grid is sized for the longest possible batch
  const int lane = threadIdx.x;
  const int n = lane & 15, g4 = lane >> 4;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const float c2 = kv.sm_scale * kLog2e;
  const LaneGeom<FP8> geo = lane_geom<FP8>(kv, lane);
  constexpr int kLoads = TileRegs<FP8>::kLoads;
  const Slice it = make_slice(kv, ws, blockIdx.x, slice_entry(ws, blockIdx.x));
  const int pg = load_pages(kv, it, lane);
  const int nt = tiles_of(it);
  u32x4 ra[kLoads], rb_[kLoads], unused[kLoads];
  issue_rows<FP8, false>(kv, it, it.t_begin, pg, geo, ra, unused);
  if (nt > 1) issue_rows<FP8, false>(kv, it, it.t_begin + kTileTokens, pg, geo, rb_, unused);
  bf16x8 qf[RB][4];
  load_q<RB>(kv, q, n_q, G, R, it, qf, lane);
  float m_run[RB], l_run[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) { m_run[rb] = -INFINITY; l_run[rb] = 0.f; }
  auto tile = [&](int ti, u32x4 (&regs)[kLoads]) {
    const int tb = it.t_begin + ti * kTileTokens;
    if (ws.debug & 256) {                      // experiment: memory traffic only
      u32x4 x = regs[0];
#pragma unroll
      for (int u = 1; u < kLoads; ++u) x ^= regs[u];
      if (ti + 2 < nt) issue_rows<FP8, false>(kv, it, tb + 2 * kTileTokens, pg, geo, regs, unused);
      l_run[0] += __uint_as_float((x.x ^ x.y ^ x.z ^ x.w) & 0x3fffffffu);
      return;
    }
    rows_to_lds<FP8, false>(regs, s_tile, lane);
    float ks[2] = {1.f, 1.f};
    if constexpr (FP8) half_scales(kv, it, tb, pg, kv.k_scale, ks);
    if (ti + 2 < nt) issue_rows<FP8, false>(kv, it, tb + 2 * kTileTokens, pg, geo, regs, unused);
    f32x4 s[2][RB];
    tile_qk<RB>(s_tile, qf, s, lane);
    const bool edge = tb + kTileTokens > it.L - n_q;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) s[sub][rb] *= c2 * ks[sub];
      if (edge) {
        const int r = 16 * rb + n;
        const int last = it.L - n_q + (r < R ? r / G : n_q - 1);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (tb + 16 * sub + 4 * g4 + i > last) s[sub][rb][i] = -INFINITY;
      }
      const float mx = fmaxf(fmaxf(fmaxf(s[0][rb][0], s[0][rb][1]), fmaxf(s[0][rb][2], s[0][rb][3])),
                             fmaxf(fmaxf(s[1][rb][0], s[1][rb][1]), fmaxf(s[1][rb][2], s[1][rb][3])));
      const float m_new = fmaxf(m_run[rb], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) sum += fast_exp2(s[0][rb][i] - m_use) + fast_exp2(s[1][rb][i] - m_use);
      l_run[rb] = l_run[rb] * fast_exp2(m_run[rb] - m_use) + sum;
      m_run[rb] = m_new;
    }
  };
  for (int ti = 0; ti < nt; ti += 2) {
    tile(ti, ra);
    if (ti + 1 < nt) tile(ti + 1, rb_);
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float mx = fmaxf(m_run[rb], xor16(m_run[rb]));
    mx = fmaxf(mx, xor32(mx));
    const float m_use = (mx == -INFINITY) ? 0.f : mx;
    float l = l_run[rb] * fast_exp2(m_run[rb] - m_use);
    l += xor16(l);
    l += xor32(l);
    if (g4 == 0) {
      ws.part_m[static_cast<int64_t>(it.id) * (RB * 16) + 16 * rb + n] = mx;
      ws.part_l[static_cast<int64_t>(it.id) * (RB * 16) + 16 * rb + n] = l;
    }
  }
}

// one thread per (pair, padded row)
__global__ __launch_bounds__(256) void verify_lse_combine(KvView kv, int n_q, FusedWs ws, float* lse_out) {
  const int rows = ws.rows_pad;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int pairs = kv.batch * kv.num_kv_heads;
  if (idx >= pairs * rows) return;
  const int pair = idx / rows, row = idx - pair * rows;
  const int b = pair / kv.num_kv_heads, g = pair - b * kv.num_kv_heads;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int ns = slices_of(kv.seq_lens[b], ws.slice_tokens);
  const int first = ws.slice_base[b] + g * ns;
  const float* pm = ws.part_m + static_cast<int64_t>(first) * rows + row;
  const float* pl = ws.part_l + static_cast<int64_t>(first) * rows + row;
  float m = -INFINITY;
  for (int c = 0; c < ns; ++c) m = fmaxf(m, pm[static_cast<int64_t>(c) * rows]);
  float l = 0.f;
  for (int c = 0; c < ns; ++c) l += pl[static_cast<int64_t>(c) * rows] * fast_exp2(pm[static_cast<int64_t>(c) * rows] - m);
  // rows beyond R get +inf so that their probabilities vanish in the score pass
  const float v = row < R ? m + log2f(l) : INFINITY;
  ws.lse2[idx] = v;
  if (lse_out && row < R) {
    const int i = row / G, hg = row - i * G;
    lse_out[(static_cast<int64_t>(b) * n_q + i) * kv.num_q_heads + g * G + hg] = v * kLn2;
  }
}

template <int RB, bool FP8>
__global__ __launch_bounds__(kThreads, RB >= 3 ? 1 : 2) void verify_score_pass(KvView kv, const uint16_t* q, int n_q, FusedWs ws,
                                                                                uint16_t* out, float* scores, int64_t score_stride) {
  __shared__ __attribute__((aligned(16))) uint8_t s_tile[kVTileBytes];
  __shared__ __attribute__((aligned(16))) uint8_t s_q[(RB * 16 + 1) * kKRow];
#ifdef PILLAR_TRACING
  const long long t_start = wall_clock64();
#endif
  if (static_cast<int>(blockIdx.x) >= ws.ctrl[1]) return;      // the grid is sized for the longest possible batch
  const int lane = threadIdx.x;
  const int n = lane & 15, g4 = lane >> 4;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const float c2 = kv.sm_scale * kLog2e;
  const float inv_r = 1.0f / static_cast<float>(R);
  const LaneGeom<FP8> geo = lane_geom<FP8>(kv, lane);
  constexpr int kLoads = TileRegs<FP8>::kLoads;
  constexpr int kQIters = ((RB * 16 + 1) * 16 + kThreads - 1) / kThreads;
  const Slice it = make_slice(kv, ws, blockIdx.x, slice_entry(ws, blockIdx.x));
  const int pg = load_pages(kv, it, lane);
  const int nt = tiles_of(it);
  u32x4 rk[kLoads], rv[kLoads];
  issue_rows<FP8, true>(kv, it, it.t_begin, pg, geo, rk, rv);
  {
    u32x4 qtmp[kQIters];
#pragma unroll
    for (int j = 0; j < kQIters; ++j) {
      const int ch = lane + kThreads * j;
      const int r = ch >> 4, c = ch & 15;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (r < R) {
        const int i = r / G, hg = r - i * G;
        v = *reinterpret_cast<const u32x4*>(q + ((static_cast<int64_t>(it.b) * n_q + i) * kv.num_q_heads + it.g * G + hg) * kHeadDim + 8 * c);
      }
      qtmp[j] = v;
    }
#pragma unroll
    for (int j = 0; j < kQIters; ++j) {
      const int ch = lane + kThreads * j;
      if (ch < (R + 1) * 16) *reinterpret_cast<u32x4*>(s_q + k_lds_addr(ch >> 4, ch & 15)) = qtmp[j];
    }
  }
  float lse2[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) lse2[rb] = ws.lse2[static_cast<int64_t>(it.pair) * (RB * 16) + 16 * rb + n];
  float* sdst = scores + (static_cast<int64_t>(it.b) * kv.num_kv_heads + it.g) * score_stride;
  f32x4 o[RB][8];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int d = 0; d < 8; ++d) o[rb][d] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int ti = 0; ti < nt; ++ti) {
    const int tb = it.t_begin + ti * kTileTokens;
    if (ws.debug & 256) {                      // experiment: memory traffic only
      u32x4 x = rk[0] ^ rv[0];
#pragma unroll
      for (int u = 1; u < kLoads; ++u) x ^= rk[u] ^ rv[u];
      if (ti + 1 < nt) issue_rows<FP8, true>(kv, it, tb + kTileTokens, pg, geo, rk, rv);
      o[0][0].x += __uint_as_float((x.x ^ x.y ^ x.z ^ x.w) & 0x3fffffffu);
      continue;
    }
    rows_to_lds<FP8, false>(rk, s_tile, lane);
    // each register set goes back on the road as soon as its rows are in LDS
    if (ti + 1 < nt) issue_rows<FP8, false>(kv, it, tb + kTileTokens, pg, geo, rk, rv);
    float ks[2] = {1.f, 1.f}, vs[2] = {1.f, 1.f};
    if constexpr (FP8) { half_scales(kv, it, tb, pg, kv.k_scale, ks); half_scales(kv, it, tb, pg, kv.v_scale, vs); }
    f32x4 s[2][RB];
    tile_qk_ldsq<RB>(s_tile, s_q, R, s, lane);
    // the K rows are consumed: the V rows take their place
    if (tb + kTileTokens > it.L) zero_tail_rows<FP8>(rv, tb, it.L, geo);
    rows_to_lds<FP8, true>(rv, s_tile, lane);
    if (ti + 1 < nt) issue_rows<FP8, true, false>(kv, it, tb + kTileTokens, pg, geo, rk, rv);
    const bool edge = tb + kTileTokens > it.L - n_q;
    f32x4 tot[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    bf16x8 p[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      f32x4 pr[2];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const float sc = c2 * ks[sub];
#pragma unroll
        for (int i = 0; i < 4; ++i) pr[sub][i] = fast_exp2(fmaf(s[sub][rb][i], sc, -lse2[rb]));
      }
      if (edge) {
        const int r = 16 * rb + n;
        const int last = it.L - n_q + (r < R ? r / G : n_q - 1);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (tb + 16 * sub + 4 * g4 + i > last) pr[sub][i] = 0.f;
      }
      tot[0] += pr[0];
      tot[1] += pr[1];
      if constexpr (FP8) { pr[0] *= vs[0]; pr[1] *= vs[1]; }
      p[rb] = pack_p(pr[0], pr[1]);
    }
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int i = 0; i < 4; ++i) tot[sub][i] = row16_sum(tot[sub][i]) * inv_r;
      const int tok0 = tb + 16 * sub + 4 * g4;
      if (n == 0) {
        if (tok0 + 3 < it.L) {
          *reinterpret_cast<f32x4*>(sdst + tok0) = tot[sub];
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (tok0 + i < it.L) sdst[tok0 + i] = tot[sub][i];
        }
      }
    }
    tile_pv<RB>(s_tile, p, o, lane);
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int r = 16 * rb + n;
    if (r >= R) continue;
    if (it.nslices == 1) {
      const int i = r / G, hg = r - i * G;
      uint16_t* dst = out + ((static_cast<int64_t>(it.b) * n_q + i) * kv.num_q_heads + it.g * G + hg) * kHeadDim;
#pragma unroll
      for (int db = 0; db < 8; ++db) {
        u32x2 pk;
        pk.x = pack2(o[rb][db][0], o[rb][db][1]);
        pk.y = pack2(o[rb][db][2], o[rb][db][3]);
        *reinterpret_cast<u32x2*>(dst + 16 * db + 4 * g4) = pk;
      }
    } else {
      float* dst = ws.part_o + (static_cast<int64_t>(it.id) * R + r) * kHeadDim + 4 * g4;
#pragma unroll
      for (int db = 0; db < 8; ++db) *reinterpret_cast<f32x4*>(dst + 16 * db) = o[rb][db];
    }
  }
#ifdef PILLAR_TRACING
  if ((blockIdx.x & 3) == 0 && blockIdx.x < 16384 && threadIdx.x == 0) {
    ws.trace[(blockIdx.x >> 2) * 2] = t_start;
    ws.trace[(blockIdx.x >> 2) * 2 + 1] = wall_clock64();
  }
#endif
}

// one workgroup per pair; pairs with a single slice were written by the score pass
__global__ __launch_bounds__(256) void verify_o_merge(KvView kv, int n_q, FusedWs ws, uint16_t* out) {
  const int pair = blockIdx.x;
  const int b = pair / kv.num_kv_heads, g = pair - b * kv.num_kv_heads;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int ns = slices_of(kv.seq_lens[b], ws.slice_tokens);
  if (ns <= 1) return;
  const int first = ws.slice_base[b] + g * ns;
  for (int idx = threadIdx.x; idx < R * (kHeadDim / 4); idx += 256) {
    const int r = idx / (kHeadDim / 4), d4 = idx - r * (kHeadDim / 4);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int c = 0; c < ns; ++c)
      acc += *reinterpret_cast<const f32x4*>(ws.part_o + (static_cast<int64_t>(first + c) * R + r) * kHeadDim + 4 * d4);
    const int i = r / G, hg = r - i * G;
    uint16_t* dst = out + ((static_cast<int64_t>(b) * n_q + i) * kv.num_q_heads + g * G + hg) * kHeadDim;
    u32x2 pk;
    pk.x = pack2(acc.x, acc.y);
    pk.y = pack2(acc.z, acc.w);
    *reinterpret_cast<u32x2*>(dst + 4 * d4) = pk;
  }
}

int num_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    cus = v;
  }
  return cus;
}

// wavefronts in the persistent grid: what the registers and LDS of this kernel let a compute unit hold
// (3 or more row blocks need the whole register file of a SIMD: one wavefront each)
int rows_blocks(const KvView& kv, int n_q) { return (n_q * (kv.num_q_heads / kv.num_kv_heads) + 15) / 16; }
int grid_size(int rb) {
  const int per_cu = rb >= 3 ? kWavesPerCu / 2 : kWavesPerCu;
  return (options().verify_grid > 0 ? min(options().verify_grid, per_cu) : per_cu) * num_cus();
}

FusedWs carve(const KvView& kv, int n_q, int slice_tokens, void* workspace, size_t* total_bytes) {
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const size_t R = static_cast<size_t>(n_q) * G;
  const size_t rpad = (R + 15) / 16 * 16;
  const size_t pairs = static_cast<size_t>(kv.batch) * kv.num_kv_heads;
  const size_t max_slices = pairs * slices_of(kv.max_seq_len, slice_tokens);
  char* p = static_cast<char*>(workspace);
  size_t off = 0;
  auto take = [&](size_t bytes) { char* r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
  FusedWs w;
  w.ctrl = reinterpret_cast<int32_t*>(take(64 * 4));
  w.slice_base = reinterpret_cast<int32_t*>(take((static_cast<size_t>(kv.batch) + 1) * 4));
  w.slices = reinterpret_cast<int32_t*>(take(max_slices * 16));
  w.cnt1 = reinterpret_cast<int32_t*>(take(pairs * 4));
  w.cnt2 = reinterpret_cast<int32_t*>(take(pairs * 4));
  w.part_m = reinterpret_cast<float*>(take(max_slices * rpad * 4));
  w.part_l = reinterpret_cast<float*>(take(max_slices * rpad * 4));
  w.part_o = reinterpret_cast<float*>(take(max_slices * R * kHeadDim * 4));
  w.lse2 = reinterpret_cast<float*>(take(pairs * rpad * 4));
  w.trace = reinterpret_cast<long long*>(take(8192 * 8));
  w.slice_tokens = slice_tokens;
  w.rows_pad = static_cast<int32_t>(rpad);
  w.grid = grid_size(rows_blocks(kv, n_q));
  w.debug = options().debug;
  w.max_slices = static_cast<int32_t>(max_slices);
  if (total_bytes) *total_bytes = off;
  return w;
}

int pick_slice_tokens(const KvView& kv) {
  int s = options().verify_chunk > 0 ? options().verify_chunk : kDefaultSlice;
  const int cap = 64 * kv.page_size;              // page ids of a slice live in one register per lane
  if (s > cap) s = cap;
  return s;
}

template <int RB, bool FP8>
hipError_t run(const VerifyArgs& a, hipStream_t st) {
  const KvView& kv = a.kv;
  const FusedWs ws = carve(kv, a.n_q, pick_slice_tokens(kv), a.workspace, nullptr);
  const uint16_t* q = static_cast<const uint16_t*>(a.q);
  uint16_t* out = static_cast<uint16_t*>(a.out);
  {
    KernelTimer t("verify_fused_plan", st);
    hipLaunchKernelGGL(fused_plan, dim3(1), dim3(1024), 0, st, kv, ws);
  }
  if (options().verify_mode == 1) {
    KernelTimer t("verify_fused_mfma", st);
    hipLaunchKernelGGL((verify_fused_mfma<RB, FP8>), dim3(grid_size(RB)), dim3(kThreads), 0, st, kv, q, a.n_q, ws, out, a.lse,
                       a.scores, a.score_stride);
    return hipGetLastError();
  }
  // the host knows the slice count exactly only through seq_lens on the device; launch the bound and let
  // surplus workgroups leave
  const int pairs = kv.batch * kv.num_kv_heads;
  {
    KernelTimer t("verify_lse_pass", st);
    hipLaunchKernelGGL((verify_lse_pass<RB, FP8>), dim3(ws.max_slices), dim3(kThreads), (options().debug >> 16) * 1024, st, kv, q, a.n_q, ws);
  }
  {
    KernelTimer t("verify_lse_combine", st);
    hipLaunchKernelGGL(verify_lse_combine, dim3((pairs * ws.rows_pad + 255) / 256), dim3(256), 0, st, kv, a.n_q, ws, a.lse);
  }
  {
    KernelTimer t("verify_score_pass", st);
    hipLaunchKernelGGL((verify_score_pass<RB, FP8>), dim3(ws.max_slices), dim3(kThreads), (options().debug >> 16) * 1024, st, kv, q, a.n_q, ws, out,
                       a.scores, a.score_stride);
  }
  {
    KernelTimer t("verify_o_merge", st);
    hipLaunchKernelGGL(verify_o_merge, dim3(pairs), dim3(256), 0, st, kv, a.n_q, ws, out);
  }
  return hipGetLastError();
}

}  // namespace

bool verify_fused_supported(const VerifyArgs& a) {
  if (!a.scores || !verify_mfma_supported(a)) return false;
  const KvView& kv = a.kv;
  if (kv.batch > kMaxBatchInLds) return false;
  // a pair must not be able to occupy every resident wavefront (see the progress argument above)
  if (slices_of(kv.max_seq_len, pick_slice_tokens(kv)) > grid_size(rows_blocks(kv, a.n_q)) / 2) return false;
  return true;
}

size_t verify_fused_trace_offset(const KvView& kv, int n_q) {
  const FusedWs w = carve(kv, n_q, pick_slice_tokens(kv), reinterpret_cast<void*>(0x1000), nullptr);
  return reinterpret_cast<uintptr_t>(w.trace) - 0x1000;
}

size_t verify_fused_workspace(const KvView& kv, int n_q) {
  size_t total = 0;
  carve(kv, n_q, pick_slice_tokens(kv), nullptr, &total);
  return total;
}

hipError_t launch_verify_fused(const VerifyArgs& a, hipStream_t s) {
  const int G = a.kv.num_q_heads / a.kv.num_kv_heads;
  const int rb = (a.n_q * G + 15) / 16;
  const bool fp8 = a.kv_dtype == PILLAR_FP8_E4M3;
#define PILLAR_CASE(N) \
  if (rb == N) return fp8 ? run<N, true>(a, s) : run<N, false>(a, s);
  PILLAR_CASE(1)
  PILLAR_CASE(2)
  PILLAR_CASE(3)
  PILLAR_CASE(4)
#undef PILLAR_CASE
  return hipErrorInvalidValue;
}

}  // namespace pillar
