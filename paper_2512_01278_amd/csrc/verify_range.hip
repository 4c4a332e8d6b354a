// Verification attention with the score statistic (paper Section 4.1) as
// streaming passes over an evenly divided token range.
//
// The probability of a token needs the row's log-sum-exp over the WHOLE
// context, which is known only after the last token.  Two ways round it live
// here; kernel boundaries are the only synchronisation in both.
//
// Default, K read once:
//   single pass       S^T = K Q^T and O^T = V^T P^T on the matrix cores the
//                     flash-decoding way (running max and sum per row, one
//                     unnormalised (m, l, O) partial per segment); the
//                     exponentials e = exp2(s - m_tile) are left behind as
//                     16-bit values (verify_flash_range; verify_flash_pair
//                     with two wavefronts per range for more than 32 rows;
//                     mixed_flash_span with the draft step of other requests
//                     in the same grid, paper Section 4.2)
//   finish            per (request, KV head), one launch (verify_finish):
//                     log-sum-exp per row from the segments, O of pairs cut
//                     into several segments, scores = mean over rows of
//                     e * exp2(m_tile - lse) read back from the stash, and
//                     Top-K of those scores while they are still on the chip
//                     (long rows with few pairs: several workgroups per pair,
//                     then verify_select_rows)
//
// Variant with fp32 probabilities, K read twice (PILLAR_FLAG_EXACT_SCORES):
//   pass 1 (K only)   running (max, sum) per row -> (m, l) per row and segment
//   combine           as above
//   pass 2 (K and V)  p = exp2(s - lse) is the exact probability: the score is
//                     written directly, and O needs no running maximum;
//                     segment partials of O add linearly
//   merge             O = sum of the partials
//
// Work division.  The unit of work is a tile of 32 tokens of one (request, KV
// head) pair; all units are laid out pair-major (request, head, tile) and the
// T units are cut into N equal contiguous ranges, one per wavefront, N being
// the number of wavefronts the chip holds at once.  Every wavefront therefore
// streams the same number of bytes and the grid drains all at once; a fixed
// slice size instead leaves the last round of workgroups on a half-empty chip
// (measured: a third of the pass-2 time at batch 128).  A range crosses pair
// boundaries; the stretch of one pair inside one range is a segment, and the
// segment of pair p in range w owns partial-result slot p + w (distinct
// segments have distinct sums because both indices grow along the layout).
// The plan (unit prefix per request, order of the pairs for the finish kernel)
// is a small kernel of its own (range_plan), or, for the single pass with up to
// 1024 requests, worked out by the wavefronts of the pass themselves (wave_plan).
#include "launch.hpp"
#include "mfma_tile.hpp"
#include "topk_core.hpp"
#include "verify_stream.hpp"
#include "decode_span.hpp"

namespace pillar {
namespace {

constexpr int kThreads = 64;                   // one wavefront per workgroup
constexpr int kWindowPages = 64;               // page ids held per register: one per lane
constexpr int kFinishMaxTokens = 32768;        // longest row whose Top-K the finish kernel selects itself

struct RangeWs {
  int32_t* ctrl;        // [0] total units T
  int32_t* ureq;        // [B+1] first unit of request b (its heads follow each other)
  int32_t* order;       // [pairs] (request, head) pairs in the order the finish kernel takes them: longest rows first
  float* scratch_scores;  // [pairs][scratch_stride] statistic of the split finish kernel when the caller wants none
  int64_t scratch_stride;
  float* part_m;        // [pairs + N][rows_pad]  log2 domain
  float* part_l;        // [pairs + N][rows_pad]
  float* part_o;        // [pairs + N][R][128]
  float* lse2;          // [pairs][rows_pad]      log2 domain
  uint8_t* stash;       // single-pass variant: [units][tile lanes][16 bytes]
  float* m_ref;         //                      [units][rows_pad] running maximum the stash of a tile refers to
  const int32_t* spec_lens;   // [B] speculative length of each request, or null: all use the call's k
  int32_t rows_pad;     // 16 * row blocks
  int32_t n_ranges;     // N
  int32_t plan_in_wave; // ctrl / ureq / order are not there yet: the wavefronts of the single pass work them out (wave_plan)
};

__host__ __device__ inline int tiles_of_len(int len) { return (len + kTileTokens - 1) / kTileTokens; }

// query positions of request b: all n_q slots, or as many as the request speculates
__device__ __forceinline__ int queries_of(const KvView& kv, const RangeWs& ws, int b, int n_q) {
  return ws.spec_lens ? min(ws.spec_lens[request_of(kv, b)] + 1, n_q) : n_q;
}

// first unit of range w, and the range a unit falls in
__device__ __forceinline__ int range_begin(int w, int total, int n) { return static_cast<int>(static_cast<int64_t>(w) * total / n); }
__device__ __forceinline__ int range_of(int unit, int total, int n) {
  return static_cast<int>(((static_cast<int64_t>(unit) + 1) * n - 1) / total);
}

// ---------------------------------------------------------------- plan ------
// Unit prefix per request, and the order in which the finish kernel takes the (request, head) pairs:
// longest requests first, so that the workgroups still running when the grid drains are short ones.
__global__ __launch_bounds__(1024) void range_plan(KvView kv, RangeWs ws) {
  __shared__ int32_t scan[1024];
  __shared__ int32_t carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  int first_len = 0;                           // length of request threadIdx.x (first pass), for the ranking below
  for (int b0 = 0; b0 < kv.batch; b0 += 1024) {
    const int b = b0 + threadIdx.x;
    const int len_b = b < kv.batch ? kv.seq_lens[request_of(kv, b)] : 0;
    if (b0 == 0) first_len = len_b;
    const int mine = b < kv.batch ? tiles_of_len(len_b) * kv.num_kv_heads : 0;
    scan[threadIdx.x] = mine;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int v = threadIdx.x >= o ? scan[threadIdx.x - o] : 0;
      __syncthreads();
      scan[threadIdx.x] += v;
      __syncthreads();
    }
    if (b < kv.batch) ws.ureq[b] = carry + scan[threadIdx.x] - mine;
    __syncthreads();
    if (threadIdx.x == 1023) carry += scan[1023];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    ws.ureq[kv.batch] = carry;
    ws.ctrl[0] = carry;
  }
  // rank of every request by length (ties by index); batches beyond one workgroup keep their own order
  if (kv.batch <= 1024) {
    __syncthreads();
    const int b = threadIdx.x;
    const int len = first_len;
    scan[threadIdx.x] = len;
    __syncthreads();
    if (b < kv.batch) {
      int rank = 0;
      for (int o = 0; o < kv.batch; ++o) {
        const int lo = scan[o];
        rank += (lo > len || (lo == len && o < b)) ? 1 : 0;
      }
      for (int g = 0; g < kv.num_kv_heads; ++g) ws.order[rank * kv.num_kv_heads + g] = b * kv.num_kv_heads + g;
    }
  } else {
    for (int i = threadIdx.x; i < kv.batch * kv.num_kv_heads; i += 1024) ws.order[i] = i;
  }
}

// ------------------------------------------------------------- helpers ------
// One stretch of one pair inside one range.
struct Segment {
  int b, g, L, tiles, tile0, tile1, pair, slot;   // b: slot of the request in this launch
  int rq;                                          // the request's id: index into everything the request owns
};

// request whose units contain `unit`: two rounds of 64-way search, the prefix table stays in L2
__device__ __forceinline__ int find_request(const RangeWs& ws, int batch, int unit, int lane) {
  int lo = 0, n = batch;                       // answer in [lo, lo + n)
  while (n > 1) {
    const int step = (n + kThreads - 1) / kThreads;
    const int probe = lo + min(lane * step, n - 1);
    const bool le = ws.ureq[probe] <= unit;    // true for a prefix of the lanes (lane 0 always)
    const int hits = __popcll(__ballot(le));
    const int first = lo + min((hits - 1) * step, n - 1);
    n = min(step, lo + n - first);
    lo = first;
  }
  return __builtin_amdgcn_readfirstlane(lo);
}

// page ids of the 64-page windows `win` and `win + 1` of a request: lane j holds page 64 * win + j
struct PageWin {
  int pg_a, pg_b, win;
};

__device__ __forceinline__ int load_window(const KvView& kv, int b, int win, int lane);

// Issues the loads of the tile at token tb (K rows into rk when WITH_K, V rows into rv when
// WITH_V) and reports the pages of its two 16-token halves.  Tiles are issued in ascending
// order, so the page window only ever moves forward; a 16-token group lies in one page whose
// id is wave-uniform, which makes the address a scalar base plus a 32-bit per-lane offset.
// Groups beyond the end of the sequence read the last page of the request: pages are whole, so
// the rows exist; the caller masks them.
template <bool FP8, bool WITH_K, bool WITH_V>
__device__ __forceinline__ void issue_tile(const KvView& kv, const Segment& sg, int tb, PageWin& pw, const LaneGeom<FP8>& geo,
                                           int lane, u32x4 (&rk)[TileRegs<FP8>::kLoads], u32x4 (&rv)[TileRegs<FP8>::kLoads],
                                           int (&pages)[2]) {
  constexpr int kLoads = TileRegs<FP8>::kLoads;
  constexpr int kPerGroup = kLoads / 2;
  const int esz = FP8 ? 1 : 2;
  const int last_page = (sg.L - 1) >> kv.page_shift;
  // both 16-token groups of a tile lie in the same 64-page window (pages hold >= 16 tokens and a tile starts
  // at a multiple of 32 tokens), so the window moves at most once per tile, before any row load is issued
  if (min(tb >> kv.page_shift, last_page) / kWindowPages > pw.win) {          // wave-uniform
    pw.pg_a = pw.pg_b;
    pw.win += 1;
    pw.pg_b = load_window(kv, sg.b, pw.win + 1, lane);
  }
#pragma unroll
  for (int grp = 0; grp < 2; ++grp) {
    const int tok0 = tb + 16 * grp;
    const int lp = min(tok0 >> kv.page_shift, last_page);
    const int page = __builtin_amdgcn_readlane(pw.pg_a, lp - pw.win * kWindowPages);
    pages[grp] = page;
    const int64_t base = (static_cast<int64_t>(page) * kv.stride_page + static_cast<int64_t>(sg.g) * kv.stride_head +
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
__device__ __forceinline__ void half_scales(const KvView& kv, int g, const int (&pages)[2], const float* table, float (&sc)[2]) {
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) sc[sub] = table[static_cast<int64_t>(pages[sub]) * kv.num_kv_heads + g];
}

template <int RB>
__device__ __forceinline__ void load_q_regs(const KvView& kv, const uint16_t* q, int n_q, int G, int R, const Segment& sg,
                                            bf16x8 (&qf)[RB][4], int lane) {
  const int n = lane & 15, g4 = lane >> 4;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int r = 16 * rb + n;
    const int i = r / G, hg = r - i * G;
    const uint16_t* row = q + ((static_cast<int64_t>(sg.rq) * n_q + i) * kv.num_q_heads + sg.g * G + hg) * kHeadDim;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (r < R) v = *reinterpret_cast<const u32x4*>(row + 32 * s + 8 * g4);
      qf[rb][s] = as_bf16x8(v);
    }
  }
}

// A tile on its way from HBM to a register set: which segment it belongs to and where it starts.
struct Flight {
  Segment sg;
  int tb;            // first token of the tile
  int pages[2];      // pages of its two 16-token halves
  float ks[2], vs[2];  // fp8: dequantisation scales of those pages, fetched along with the rows (a load at the
                     // tile's turn would keep a round trip to memory in every tile)
  bool valid;
};

template <bool FP8>
__device__ __forceinline__ void fetch_scales(const KvView& kv, Flight& f) {
  f.ks[0] = f.ks[1] = f.vs[0] = f.vs[1] = 1.f;
  if constexpr (FP8) {
    half_scales(kv, f.sg.g, f.pages, kv.k_scale, f.ks);
    half_scales(kv, f.sg.g, f.pages, kv.v_scale, f.vs);
  }
}

// Issue side of the tile stream of one range.  The stream runs ahead of the arithmetic by the
// tiles in flight and crosses pair boundaries without draining: when it enters a pair it already
// holds the page ids of the pair after it (they were fetched one pair earlier).
struct Cursor {
  int unit, end, w;  // next unit to issue, end of the range, index of the range
  Segment sg;        // the segment that unit belongs to
  int tile;          // next tile of sg
  PageWin pw;
  int pg_next;       // page window 0 of the request of the following pair
  int len_next;      // sequence length of that request (per-lane copy)
  bool live;
};

__device__ __forceinline__ int load_window(const KvView& kv, int b, int win, int lane) {
  // entries past the last page of the request are never used as addresses (issue_tile clamps), so
  // it is enough to stay inside the table row
  return kv.block_table[static_cast<int64_t>(request_of(kv, b)) * kv.block_table_stride + min(win * kWindowPages + lane, kv.block_table_stride - 1)];
}

__device__ __forceinline__ void prefetch_following(const KvView& kv, Cursor& c, int lane) {
  int nb = c.sg.b + (c.sg.g + 1 == kv.num_kv_heads ? 1 : 0);
  nb = min(nb, kv.batch - 1);                  // past the last request nothing of this is used
  c.len_next = kv.seq_lens[request_of(kv, nb)];
  c.pg_next = load_window(kv, nb, 0, lane);
}

__device__ __forceinline__ Segment uniform(const Segment& s) {
  Segment u;
  u.b = __builtin_amdgcn_readfirstlane(s.b);
  u.g = __builtin_amdgcn_readfirstlane(s.g);
  u.L = __builtin_amdgcn_readfirstlane(s.L);
  u.tiles = __builtin_amdgcn_readfirstlane(s.tiles);
  u.tile0 = __builtin_amdgcn_readfirstlane(s.tile0);
  u.tile1 = __builtin_amdgcn_readfirstlane(s.tile1);
  u.pair = __builtin_amdgcn_readfirstlane(s.pair);
  u.slot = __builtin_amdgcn_readfirstlane(s.slot);
  u.rq = __builtin_amdgcn_readfirstlane(s.rq);
  return u;
}

// The plan without a launch of its own, for batches of up to 64 * kPlanRegs requests: every wavefront of the
// single pass reads all lengths (lane l, register j: request 64 j + l) and scans them into the unit prefix, which
// costs one round trip to memory where reading a finished plan costs three dependent ones.
constexpr int kPlanRegs = 16;
struct WavePlan {
  int len[kPlanRegs];
  int first[kPlanRegs];   // units before the request
  int total;
};

__device__ __forceinline__ WavePlan wave_plan(const KvView& kv, int lane) {
  WavePlan p;
#pragma unroll
  for (int j = 0; j < kPlanRegs; ++j) {
    p.len[j] = 0;
    if (kWave * j < kv.batch) {                // wave-uniform
      const int b = kWave * j + lane;
      if (b < kv.batch) p.len[j] = kv.seq_lens[request_of(kv, b)];
    }
  }
  int carry = 0;
#pragma unroll
  for (int j = 0; j < kPlanRegs; ++j) {
    p.first[j] = carry;
    if (kWave * j < kv.batch) {
      const int mine = tiles_of_len(p.len[j]) * kv.num_kv_heads;         // 0 beyond the batch
      const int incl = static_cast<int>(wave_inclusive_sum(static_cast<uint32_t>(mine)));
      p.first[j] = carry + incl - mine;
      carry += __builtin_amdgcn_readlane(incl, kWave - 1);
    }
  }
  p.total = carry;
  return p;
}

// value of register set v for request b (wave-uniform)
__device__ __forceinline__ int plan_get(const int (&v)[kPlanRegs], int b) {
  int r = 0;
#pragma unroll
  for (int j = 0; j < kPlanRegs; ++j)
    if (j == (b >> 6)) r = __builtin_amdgcn_readlane(v[j], b & (kWave - 1));
  return r;
}

// What range_plan leaves in memory for the kernels after the pass, written by the pass itself: wavefront w ranks
// requests w, w + N, ... by length (the order of the finish kernel: longest first, ties by index), wavefront 0
// also writes the prefix.
__device__ __forceinline__ void publish_plan(const KvView& kv, const RangeWs& ws, const WavePlan& p, int w, int lane) {
  for (int r = w; r < kv.batch; r += ws.n_ranges) {
    const int len_r = plan_get(p.len, r);
    int rank = 0;
#pragma unroll
    for (int j = 0; j < kPlanRegs; ++j) {
      if (kWave * j < kv.batch) {
        const int b = kWave * j + lane;
        const bool ahead = b < kv.batch && (p.len[j] > len_r || (p.len[j] == len_r && b < r));
        rank += __popcll(__ballot(ahead));
      }
    }
    for (int g = lane; g < kv.num_kv_heads; g += kWave) ws.order[rank * kv.num_kv_heads + g] = r * kv.num_kv_heads + g;
  }
  if (w == 0) {
#pragma unroll
    for (int j = 0; j < kPlanRegs; ++j) {
      const int b = kWave * j + lane;
      if (b < kv.batch) ws.ureq[b] = p.first[j];
    }
    if (lane == 0) {
      ws.ureq[kv.batch] = p.total;
      ws.ctrl[0] = p.total;
    }
  }
}

__device__ __forceinline__ Cursor open_cursor(const KvView& kv, const RangeWs& ws, int w, int lane) {
  Cursor c;
  c.w = w;
  c.sg = Segment{};
  c.tile = 0;
  c.pw = PageWin{};
  c.pg_next = 0;
  c.len_next = 0;
  Segment sg;
  int first_unit;                              // of the request the range begins in
  if (ws.plan_in_wave) {                       // the same for the whole grid
    const WavePlan p = wave_plan(kv, lane);
    publish_plan(kv, ws, p, w, lane);
    c.unit = range_begin(c.w, p.total, ws.n_ranges);
    c.end = range_begin(c.w + 1, p.total, ws.n_ranges);
    c.live = c.unit < c.end;
    if (!c.live) return c;
    int upto = 0;                              // requests that begin at or before the unit
#pragma unroll
    for (int j = 0; j < kPlanRegs; ++j) {
      if (kWave * j < kv.batch) upto += __popcll(__ballot(kWave * j + lane < kv.batch && p.first[j] <= c.unit));
    }
    sg.b = upto - 1;
    sg.rq = __builtin_amdgcn_readfirstlane(request_of(kv, sg.b));
    sg.L = plan_get(p.len, sg.b);
    first_unit = plan_get(p.first, sg.b);
  } else {
    const int total = ws.ctrl[0];
    c.unit = range_begin(c.w, total, ws.n_ranges);
    c.end = range_begin(c.w + 1, total, ws.n_ranges);
    c.live = c.unit < c.end;
    if (!c.live) return c;
    sg.b = find_request(ws, kv.batch, c.unit, lane);
    sg.rq = __builtin_amdgcn_readfirstlane(request_of(kv, sg.b));
    sg.L = __builtin_amdgcn_readfirstlane(kv.seq_lens[sg.rq]);
    first_unit = __builtin_amdgcn_readfirstlane(ws.ureq[sg.b]);
  }
  sg.tiles = tiles_of_len(sg.L);
  const int rel = c.unit - first_unit;
  sg.g = rel / sg.tiles;
  sg.tile0 = rel - sg.g * sg.tiles;
  sg.tile1 = min(sg.tiles, sg.tile0 + (c.end - c.unit));
  sg.pair = sg.b * kv.num_kv_heads + sg.g;
  sg.slot = sg.pair + c.w;
  c.sg = sg;
  c.tile = sg.tile0;
  c.pw.win = ((sg.tile0 * kTileTokens) >> kv.page_shift) / kWindowPages;
  c.pw.pg_a = load_window(kv, sg.b, c.pw.win, lane);
  c.pw.pg_b = load_window(kv, sg.b, c.pw.win + 1, lane);
  prefetch_following(kv, c, lane);
  return c;
}

// Steps the cursor past the tile just issued; entering the next pair costs no wait (its pages were
// fetched one pair earlier).
__device__ __forceinline__ void advance_cursor(const KvView& kv, Cursor& c, int lane) {
  c.tile += 1;
  c.unit += 1;
  if (c.unit >= c.end) {
    c.live = false;
  } else if (c.tile == c.sg.tile1) {           // on to the next pair
    Segment sg = c.sg;
    sg.g += 1;
    if (sg.g == kv.num_kv_heads) {
      sg.g = 0;
      sg.b += 1;
    }
    sg.L = __builtin_amdgcn_readfirstlane(c.len_next);
    sg.tiles = tiles_of_len(sg.L);
    sg.tile0 = 0;
    sg.tile1 = min(sg.tiles, c.end - c.unit);
    sg.pair = sg.b * kv.num_kv_heads + sg.g;
    sg.slot = sg.pair + c.w;
    sg.rq = request_of(kv, sg.b);
    c.sg = uniform(sg);
    c.tile = 0;
    c.pw.win = 0;
    c.pw.pg_a = c.pg_next;
    c.pw.pg_b = load_window(kv, c.sg.b, 1, lane);
    prefetch_following(kv, c, lane);
  }
}

// Issues the next tile of the stream into a register set and steps the cursor.
template <bool FP8, bool WITH_V>
__device__ __forceinline__ Flight issue_next(const KvView& kv, Cursor& c, const LaneGeom<FP8>& geo, int lane,
                                             u32x4 (&rk)[TileRegs<FP8>::kLoads], u32x4 (&rv)[TileRegs<FP8>::kLoads]) {
  Flight f;
  f.valid = c.live;
  f.sg = c.sg;
  f.tb = c.tile * kTileTokens;
  f.pages[0] = f.pages[1] = 0;
  f.ks[0] = f.ks[1] = f.vs[0] = f.vs[1] = 1.f;
  if (!c.live) return f;
  issue_tile<FP8, true, WITH_V>(kv, c.sg, f.tb, c.pw, geo, lane, rk, rv, f.pages);
  fetch_scales<FP8>(kv, f);
  advance_cursor(kv, c, lane);
  return f;
}

// The same in two steps, so that the K rows of the next tile can leave as soon as the K registers are free
// and its V rows as soon as the V registers are: issue_next_k fills the flight and leaves the cursor on the
// tile, issue_next_v sends the V loads of that tile and steps the cursor.
template <bool FP8>
__device__ __forceinline__ Flight issue_next_k(const KvView& kv, Cursor& c, const LaneGeom<FP8>& geo, int lane,
                                               u32x4 (&rk)[TileRegs<FP8>::kLoads], u32x4 (&rv)[TileRegs<FP8>::kLoads]) {
  Flight f;
  f.valid = c.live;
  f.sg = c.sg;
  f.tb = c.tile * kTileTokens;
  f.pages[0] = f.pages[1] = 0;
  f.ks[0] = f.ks[1] = f.vs[0] = f.vs[1] = 1.f;
  if (!c.live) return f;
  issue_tile<FP8, true, false>(kv, c.sg, f.tb, c.pw, geo, lane, rk, rv, f.pages);
  fetch_scales<FP8>(kv, f);
  return f;
}
template <bool FP8>
__device__ __forceinline__ void issue_next_v(const KvView& kv, Cursor& c, const Flight& f, const LaneGeom<FP8>& geo, int lane,
                                             u32x4 (&rk)[TileRegs<FP8>::kLoads], u32x4 (&rv)[TileRegs<FP8>::kLoads]) {
  if (!f.valid) return;
  int pages[2];
  issue_tile<FP8, false, true>(kv, f.sg, f.tb, c.pw, geo, lane, rk, rv, pages);
  advance_cursor(kv, c, lane);
}

// ---------------------------------------------------------------- pass 1 ----
template <int RB, bool FP8>
__global__ __launch_bounds__(kThreads, 2) void verify_lse_range(KvView kv, const uint16_t* q, int n_q, RangeWs ws) {
  __shared__ __attribute__((aligned(16))) uint8_t s_tile[kKTileBytes];
  const int lane = threadIdx.x;
  const int n = lane & 15, g4 = lane >> 4;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const float c2 = kv.sm_scale * kLog2e;
  const LaneGeom<FP8> geo = lane_geom<FP8>(kv, lane);
  constexpr int kLoads = TileRegs<FP8>::kLoads;
  Cursor cur = open_cursor(kv, ws, blockIdx.x, lane);
  if (!cur.live) return;
  // K tiles travel two deep: even tiles through ra, odd tiles through rb_
  u32x4 ra[kLoads], rb_[kLoads], unused[kLoads];
  Flight fa = issue_next<FP8, false>(kv, cur, geo, lane, ra, unused);
  Flight fb = issue_next<FP8, false>(kv, cur, geo, lane, rb_, unused);
  Segment cs = fa.sg;
  bool started = false;
  bf16x8 qf[RB][4];
  float m_run[RB], l_run[RB];
  auto finish = [&]() {                        // the 4 token groups of a row -> the segment's (m, l)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float mx = max_over_groups(m_run[rb]);
      const float m_use = (mx == -INFINITY) ? 0.f : mx;
      float l = l_run[rb] * fast_exp2(m_run[rb] - m_use);
      l = sum_over_groups(l);
      if (g4 == 0) {
        ws.part_m[static_cast<int64_t>(cs.slot) * (RB * 16) + 16 * rb + n] = mx;
        ws.part_l[static_cast<int64_t>(cs.slot) * (RB * 16) + 16 * rb + n] = l;
      }
    }
  };
  auto tile = [&](Flight& f, u32x4 (&regs)[kLoads]) {
    if (!started || f.sg.slot != cs.slot) {    // wave-uniform: the stream has entered another pair
      if (started) finish();
      cs = f.sg;
      started = true;
      load_q_regs<RB>(kv, q, n_q, G, R, cs, qf, lane);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) { m_run[rb] = -INFINITY; l_run[rb] = 0.f; }
    }
    const int tb = f.tb;
    rows_to_lds<FP8, false>(regs, s_tile, lane);
    const float ks[2] = {f.ks[0], f.ks[1]};
    f = issue_next<FP8, false>(kv, cur, geo, lane, regs, unused);
    f32x4 s[2][RB];
    tile_qk<RB>(s_tile, qf, s, lane);
    const bool edge = tb + kTileTokens > cs.L - n_q;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) s[sub][rb] *= c2 * ks[sub];
      if (edge) {
        const int r = 16 * rb + n;
        const int last = cs.L - n_q + (r < R ? r / G : n_q - 1);
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
  for (;;) {
    if (!fa.valid) break;
    tile(fa, ra);
    if (!fb.valid) break;
    tile(fb, rb_);
  }
  finish();
}

// ---------------------------------------------------------------- combine ---
// one thread per (pair, padded row)
__global__ __launch_bounds__(256) void verify_lse_combine_range(KvView kv, int n_q, RangeWs ws, float* lse_out) {
  const int rows = ws.rows_pad;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int pairs = kv.batch * kv.num_kv_heads;
  if (idx >= pairs * rows) return;
  const int pair = idx / rows, row = idx - pair * rows;
  const int b = pair / kv.num_kv_heads, g = pair - b * kv.num_kv_heads;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int total = ws.ctrl[0];
  const int rq = request_of(kv, b);
  const int tiles = tiles_of_len(kv.seq_lens[rq]);
  const int u0 = ws.ureq[b] + g * tiles;
  const int w0 = range_of(u0, total, ws.n_ranges), w1 = range_of(u0 + tiles - 1, total, ws.n_ranges);
  const float* pm = ws.part_m + static_cast<int64_t>(pair + w0) * rows + row;
  const float* pl = ws.part_l + static_cast<int64_t>(pair + w0) * rows + row;
  float m = -INFINITY, l = 0.f;
  for (int c = 0; c <= w1 - w0; ++c) {
    // with fewer units than ranges some ranges are empty and own no segment
    if (range_begin(w0 + c, total, ws.n_ranges) == range_begin(w0 + c + 1, total, ws.n_ranges)) continue;
    const float mc = pm[static_cast<int64_t>(c) * rows], lc = pl[static_cast<int64_t>(c) * rows];
    const float mn = fmaxf(m, mc);
    const float mu = (mn == -INFINITY) ? 0.f : mn;
    l = l * fast_exp2(m - mu) + lc * fast_exp2(mc - mu);
    m = mn;
  }
  // rows beyond the request's R, and rows that see no token at all (a context shorter than the request's
  // queries), get +inf so that their probabilities vanish where the log-sum-exp is applied
  const int Rb = queries_of(kv, ws, b, n_q) * G;
  const bool live = row < Rb && l > 0.f;
  const float v = live ? m + log2f(l) : INFINITY;
  ws.lse2[idx] = v;
  if (lse_out && row < Rb) {
    const int i = row / G, hg = row - i * G;
    lse_out[(static_cast<int64_t>(rq) * n_q + i) * kv.num_q_heads + g * G + hg] = live ? v * kLn2 : -INFINITY;
  }
}

// ---------------------------------------------------------------- pass 2 ----
template <int RB, bool FP8>
__global__ __launch_bounds__(kThreads, RB >= 3 ? 1 : 2) void verify_score_range(KvView kv, const uint16_t* q, int n_q, RangeWs ws,
                                                                                 uint16_t* out, float* scores, int64_t score_stride) {
  // one tile buffer: the K rows, then (once S^T is done) the V rows of the same tile
  __shared__ __attribute__((aligned(16))) uint8_t s_tile[kVTileBytes];
  __shared__ __attribute__((aligned(16))) uint8_t s_q[(RB * 16 + 1) * kKRow];
  const int lane = threadIdx.x;
  const int n = lane & 15, g4 = lane >> 4;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const float c2 = kv.sm_scale * kLog2e;
  const float inv_r = 1.0f / static_cast<float>(R);
  const LaneGeom<FP8> geo = lane_geom<FP8>(kv, lane);
  constexpr int kLoads = TileRegs<FP8>::kLoads;
  constexpr int kQIters = ((RB * 16 + 1) * 16 + kThreads - 1) / kThreads;
  Cursor cur = open_cursor(kv, ws, blockIdx.x, lane);
  if (!cur.live) return;
  u32x4 rk[kLoads], rv[kLoads];
  Flight f = issue_next<FP8, true>(kv, cur, geo, lane, rk, rv);
  Segment cs = f.sg;
  bool started = false;
  float lse2[RB];
  float* sdst = scores;
  f32x4 o[RB][8];
  auto finish = [&]() {                        // O of the segment: final when it is the whole pair, else a partial
    const bool whole = cs.tile0 == 0 && cs.tile1 == cs.tiles;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int r = 16 * rb + n;
      if (r >= R) continue;
      if (whole) {
        const int i = r / G, hg = r - i * G;
        uint16_t* dst = out + ((static_cast<int64_t>(cs.rq) * n_q + i) * kv.num_q_heads + cs.g * G + hg) * kHeadDim;
#pragma unroll
        for (int db = 0; db < 8; ++db) {
          u32x2 pk;
          pk.x = pack2(o[rb][db][0], o[rb][db][1]);
          pk.y = pack2(o[rb][db][2], o[rb][db][3]);
          *reinterpret_cast<u32x2*>(dst + 16 * db + 4 * g4) = pk;
        }
      } else {
        float* dst = ws.part_o + (static_cast<int64_t>(cs.slot) * R + r) * kHeadDim + 4 * g4;
#pragma unroll
        for (int db = 0; db < 8; ++db) *reinterpret_cast<f32x4*>(dst + 16 * db) = o[rb][db];
      }
    }
  };
  while (f.valid) {
    if (!started || f.sg.slot != cs.slot) {    // wave-uniform: the stream has entered another pair
      if (started) finish();
      cs = f.sg;
      started = true;
      {                                        // Q rows of the pair -> LDS (row R is the zero row of the padding)
        u32x4 qtmp[kQIters];
#pragma unroll
        for (int j = 0; j < kQIters; ++j) {
          const int ch = lane + kThreads * j;
          const int r = ch >> 4, c = ch & 15;
          u32x4 v = {0u, 0u, 0u, 0u};
          if (r < R) {
            const int i = r / G, hg = r - i * G;
            v = *reinterpret_cast<const u32x4*>(q + ((static_cast<int64_t>(cs.rq) * n_q + i) * kv.num_q_heads + cs.g * G + hg) * kHeadDim + 8 * c);
          }
          qtmp[j] = v;
        }
#pragma unroll
        for (int j = 0; j < kQIters; ++j) {
          const int ch = lane + kThreads * j;
          if (ch < (R + 1) * 16) *reinterpret_cast<u32x4*>(s_q + k_lds_addr(ch >> 4, ch & 15)) = qtmp[j];
        }
      }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) lse2[rb] = ws.lse2[static_cast<int64_t>(cs.pair) * (RB * 16) + 16 * rb + n];
      sdst = scores + (static_cast<int64_t>(cs.rq) * kv.num_kv_heads + cs.g) * score_stride;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int d = 0; d < 8; ++d) o[rb][d] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const int tb = f.tb;
    rows_to_lds<FP8, false>(rk, s_tile, lane);
    const float ks[2] = {f.ks[0], f.ks[1]}, vs[2] = {f.vs[0], f.vs[1]};
    f32x4 s[2][RB];
    tile_qk_ldsq<RB>(s_tile, s_q, R, s, lane);
    // the K rows are consumed: the V rows take their place, and both register sets carry the next tile
    if (tb + kTileTokens > cs.L) zero_tail_rows<FP8>(rv, tb, cs.L, geo);
    rows_to_lds<FP8, true>(rv, s_tile, lane);
    f = issue_next<FP8, true>(kv, cur, geo, lane, rk, rv);
    const bool edge = tb + kTileTokens > cs.L - n_q;
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
        const int last = cs.L - n_q + (r < R ? r / G : n_q - 1);
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
        if (tok0 + 3 < cs.L) {
          *reinterpret_cast<f32x4*>(sdst + tok0) = tot[sub];
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (tok0 + i < cs.L) sdst[tok0 + i] = tot[sub][i];
        }
      }
    }
    tile_pv<RB>(s_tile, p, o, lane);
  }
  finish();
}

// ---------------------------------------------------------------- merge -----
// one workgroup per pair; a pair inside one range was written by pass 2 itself
__global__ __launch_bounds__(256) void verify_o_merge_range(KvView kv, int n_q, RangeWs ws, uint16_t* out) {
  const int pair = blockIdx.x;
  const int b = pair / kv.num_kv_heads, g = pair - b * kv.num_kv_heads;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int total = ws.ctrl[0];
  const int rq = request_of(kv, b);
  const int tiles = tiles_of_len(kv.seq_lens[rq]);
  const int u0 = ws.ureq[b] + g * tiles;
  const int w0 = range_of(u0, total, ws.n_ranges), w1 = range_of(u0 + tiles - 1, total, ws.n_ranges);
  if (w1 == w0) return;
  for (int idx = threadIdx.x; idx < R * (kHeadDim / 4); idx += 256) {
    const int r = idx / (kHeadDim / 4), d4 = idx - r * (kHeadDim / 4);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int w = w0; w <= w1; ++w) {
      if (range_begin(w, total, ws.n_ranges) == range_begin(w + 1, total, ws.n_ranges)) continue;   // empty range
      acc += *reinterpret_cast<const f32x4*>(ws.part_o + (static_cast<int64_t>(pair + w) * R + r) * kHeadDim + 4 * d4);
    }
    const int i = r / G, hg = r - i * G;
    uint16_t* dst = out + ((static_cast<int64_t>(rq) * n_q + i) * kv.num_q_heads + g * G + hg) * kHeadDim;
    u32x2 pk;
    pk.x = pack2(acc.x, acc.y);
    pk.y = pack2(acc.z, acc.w);
    *reinterpret_cast<u32x2*>(dst + 4 * d4) = pk;
  }
}

// ------------------------------------------------ single-pass variant -------
// The same result with K read once: one streaming pass computes O the flash-decoding way (running
// maximum per row, unnormalised partials) and leaves behind, per token and row, the exponential
// e = exp2(s - m_tile) relative to the running maximum m_tile at that tile.  Once the pair's
// log-sum-exp is known, a small streaming kernel turns the stash into probabilities,
// p = e * exp2(m_tile - lse), and sums them over the rows: 2 bytes per (token, row) written and
// read back, against the 2 * head_dim bytes per token of the second K read it replaces.
//
// A stashed value is 16 bits: e lies in [0, 1], so it is kept as 6 bits of exponent (2^-62 .. 1,
// smaller values become 0) and 10 bits of mantissa, rounded to nearest: relative error at most 2^-11
// per term, hence at most 2^-11 (4.9e-4) on a score, which is a sum of positive terms.  That is inside
// the 1e-3 the statistic is specified to, and far inside what Top-K needs; the two-pass variant keeps
// full fp32 probabilities.
//
// Stash layout per tile: the lanes of every full 16-row block (64 lanes), then of the last block
// only the lanes of real rows (4 * nv, nv = R - 16 (RB - 1)); per lane 16 bytes = 8 values (tokens
// 16 sub + 4 g4 + i, sub < 2, i < 4).
__device__ __forceinline__ uint32_t stash_encode(float e) {
  // bits 28..13 of (e's float pattern - 64 exponent steps), rounded to nearest at the 10th mantissa bit.
  // Exponent field 0 is kept for zero alone, so that the decoder's shift never makes a denormal: what lies
  // below 2^-62 becomes 0.
  const int d = static_cast<int>(__float_as_uint(e)) + (0x1000 - 0x20000000);
  return d >= 0x00800000 ? static_cast<uint32_t>(d) >> 13 : 0u;
}
// The stashed value times 2^-64: a plain shift into float position (0 stays 0).  Readers fold the 2^64 into
// the per-row weight, see kStashBias.
__device__ __forceinline__ float stash_decode_scaled(uint32_t c) { return __uint_as_float(c << 13); }
constexpr float kStashBias = 64.f;

__device__ __forceinline__ int stash_lane(int rb, int nblocks, int nv, int n, int g4, int lane) {
  return rb < nblocks - 1 ? rb * 64 + lane : (n < nv ? (nblocks - 1) * 64 + g4 * nv + n : -1);
}

// Range w of the single pass, by one wavefront (lane = its lane index) with its own LDS: a tile buffer of
// kVTileBytes and (RB * 16 + 1) query rows of kKRow bytes.
template <int RB, bool FP8, bool STASH>
__device__ __forceinline__ void flash_range_body(const KvView& kv, const uint16_t* q, int n_q, const RangeWs& ws, uint16_t* out,
                                                 uint8_t* s_tile, uint8_t* s_q, int w, int lane) {
  static_assert(RB <= 2, "3 and 4 row blocks run verify_flash_pair");
  constexpr int DEPTH = 1;                     // tiles in flight (two wavefronts share a SIMD's registers: no room for more)
  const int n = lane & 15, g4 = lane >> 4;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int nv = R - 16 * (RB - 1);
  const int tile_lanes = (RB - 1) * 64 + 4 * nv;
  const float c2 = kv.sm_scale * kLog2e;
  const LaneGeom<FP8> geo = lane_geom<FP8>(kv, lane);
  constexpr int kLoads = TileRegs<FP8>::kLoads;
  constexpr int kQIters = ((RB * 16 + 1) * 16 + kThreads - 1) / kThreads;
  Cursor cur = open_cursor(kv, ws, w, lane);
  if (!cur.live) return;
  int unit = cur.unit;                         // global index of the tile being computed
  u32x4 rk[DEPTH][kLoads], rv[DEPTH][kLoads];
  Flight fl[DEPTH];
#pragma unroll
  for (int j = 0; j < DEPTH; ++j) fl[j] = issue_next<FP8, true>(kv, cur, geo, lane, rk[j], rv[j]);
  Segment cs = fl[0].sg;
  bool started = false;
  float m_run[RB], l_run[RB];
  f32x4 o[RB][8];
  int nq_b = n_q, Rb = R;                      // query positions and rows of the current pair's request
  auto finish = [&]() {
    const bool whole = cs.tile0 == 0 && cs.tile1 == cs.tiles;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float l = l_run[rb];
      l = sum_over_groups(l);
      const int r = 16 * rb + n;
      if (g4 == 0) {
        ws.part_m[static_cast<int64_t>(cs.slot) * (RB * 16) + r] = m_run[rb];
        ws.part_l[static_cast<int64_t>(cs.slot) * (RB * 16) + r] = l;
      }
      if (r >= Rb) continue;               // rows of query slots the request does not use are left alone
      if (whole) {
        const float inv = l > 0.f ? 1.0f / l : 0.f;       // a row that sees no token: zeros
        const int i = r / G, hg = r - i * G;
        uint16_t* dst = out + ((static_cast<int64_t>(cs.rq) * n_q + i) * kv.num_q_heads + cs.g * G + hg) * kHeadDim;
#pragma unroll
        for (int db = 0; db < 8; ++db) {
          u32x2 pk;
          pk.x = pack2(o[rb][db][0] * inv, o[rb][db][1] * inv);
          pk.y = pack2(o[rb][db][2] * inv, o[rb][db][3] * inv);
          *reinterpret_cast<u32x2*>(dst + 16 * db + 4 * g4) = pk;
        }
      } else {
        float* dst = ws.part_o + (static_cast<int64_t>(cs.slot) * R + r) * kHeadDim + 4 * g4;
#pragma unroll
        for (int db = 0; db < 8; ++db) *reinterpret_cast<f32x4*>(dst + 16 * db) = o[rb][db];
      }
    }
  };
  auto tile = [&](Flight& f, u32x4 (&rk)[kLoads], u32x4 (&rv)[kLoads]) {
    if (!started || f.sg.slot != cs.slot) {    // wave-uniform: the stream has entered another pair
      if (started) finish();
      cs = f.sg;
      started = true;
      nq_b = __builtin_amdgcn_readfirstlane(queries_of(kv, ws, cs.b, n_q));
      Rb = nq_b * G;
      {                                        // Q rows of the pair -> LDS (row R is the zero row of the padding)
        u32x4 qtmp[kQIters];
#pragma unroll
        for (int j = 0; j < kQIters; ++j) {
          const int ch = lane + kThreads * j;
          const int r = ch >> 4, c = ch & 15;
          u32x4 v = {0u, 0u, 0u, 0u};
          if (r < Rb) {
            const int i = r / G, hg = r - i * G;
            v = *reinterpret_cast<const u32x4*>(q + ((static_cast<int64_t>(cs.rq) * n_q + i) * kv.num_q_heads + cs.g * G + hg) * kHeadDim + 8 * c);
          }
          qtmp[j] = v;
        }
#pragma unroll
        for (int j = 0; j < kQIters; ++j) {
          const int ch = lane + kThreads * j;
          if (ch < (R + 1) * 16) *reinterpret_cast<u32x4*>(s_q + k_lds_addr(ch >> 4, ch & 15)) = qtmp[j];
        }
      }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        m_run[rb] = -INFINITY;
        l_run[rb] = 0.f;
#pragma unroll
        for (int d = 0; d < 8; ++d) o[rb][d] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
    const int tb = f.tb;
    rows_to_lds<FP8, false>(rk, s_tile, lane);
    const float ks[2] = {f.ks[0], f.ks[1]}, vs[2] = {f.vs[0], f.vs[1]};
    f = issue_next_k<FP8>(kv, cur, geo, lane, rk, rv);       // the K registers are free: next tile's K rows leave now
    f32x4 s[2][RB];
    tile_qk_ldsq<RB>(s_tile, s_q, R, s, lane);
    if (tb + kTileTokens > cs.L) zero_tail_rows<FP8>(rv, tb, cs.L, geo);
    rows_to_lds<FP8, true>(rv, s_tile, lane);
    issue_next_v<FP8>(kv, cur, f, geo, lane, rk, rv);        // and its V rows once the V registers are
    const bool edge = tb + kTileTokens > cs.L - n_q;
    bf16x8 p[RB];
    uint8_t* st_base = ws.stash + static_cast<int64_t>(unit) * tile_lanes * 16;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      // logits stay unscaled until the exponential: the scales are positive, so the maximum commutes with them
      f32x4 pr[2] = {s[0][rb], s[1][rb]};
      if (edge) {
        const int r = 16 * rb + n;
        const int last = cs.L - nq_b + (r < Rb ? r / G : nq_b - 1);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (tb + 16 * sub + 4 * g4 + i > last) pr[sub][i] = -INFINITY;
      }
      const float sc0 = c2 * ks[0], sc1 = c2 * ks[1];
      float mx = fmaxf(fmaxf(fmaxf(pr[0][0], pr[0][1]), fmaxf(pr[0][2], pr[0][3])) * sc0,
                       fmaxf(fmaxf(pr[1][0], pr[1][1]), fmaxf(pr[1][2], pr[1][3])) * sc1);
      mx = max_over_groups(mx);                 // the same in the four lanes of a row
      const float m_new = fmaxf(m_run[rb], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      if (__any(m_new > m_run[rb])) {          // some row's maximum moved: rescale what is accumulated
        const float alpha = fast_exp2(m_run[rb] - m_use);
        l_run[rb] *= alpha;
#pragma unroll
        for (int d = 0; d < 8; ++d) o[rb][d] *= alpha;
      }
      m_run[rb] = m_new;
      float sum = 0.f;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          pr[sub][i] = fast_exp2(fmaf(pr[sub][i], sub == 0 ? sc0 : sc1, -m_use));
          sum += pr[sub][i];
        }
      l_run[rb] += sum;
      // the exponentials, 24 bits each, and the maximum they refer to
      const int sl = STASH ? stash_lane(rb, RB, nv, n, g4, lane) : -1;
      if (sl >= 0) {
        uint32_t c[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) c[k] = stash_encode(pr[k >> 2][k & 3]);
        u32x4 packed;
        packed.x = c[0] | (c[1] << 16);
        packed.y = c[2] | (c[3] << 16);
        packed.z = c[4] | (c[5] << 16);
        packed.w = c[6] | (c[7] << 16);
        *reinterpret_cast<u32x4*>(st_base + sl * 16) = packed;
      }
      if (STASH && g4 == 0) ws.m_ref[static_cast<int64_t>(unit) * (RB * 16) + 16 * rb + n] = m_use;
      if constexpr (FP8) { pr[0] *= vs[0]; pr[1] *= vs[1]; }
      p[rb] = pack_p(pr[0], pr[1]);
    }
    tile_pv<RB>(s_tile, p, o, lane);
    unit += 1;
  };
  for (bool more = true; more;) {
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      if (!fl[j].valid) { more = false; break; }     // slots are refilled in order: the first empty one ends the stream
      tile(fl[j], rk[j], rv[j]);
    }
  }
  finish();
}

template <int RB, bool FP8, bool STASH>
__global__ __launch_bounds__(kThreads, 2) void verify_flash_range(KvView kv, const uint16_t* q, int n_q, RangeWs ws, uint16_t* out) {
  __shared__ __attribute__((aligned(16))) uint8_t s_tile[kVTileBytes];
  __shared__ __attribute__((aligned(16))) uint8_t s_q[(RB * 16 + 1) * kKRow];
  flash_range_body<RB, FP8, STASH>(kv, q, n_q, ws, out, s_tile, s_q, blockIdx.x, threadIdx.x);
}

// A unified batch in one grid (paper Section 4.2, "Fused Sparse and Full Attention"): the first n_groups
// workgroups carry four ranges of the verification pass each (one per wavefront, as independent as in their own
// kernel), the workgroups after them one (request, KV head, span) of the draft step each.  Which path a
// workgroup takes is decided on the chip from its index; the draft workgroups come last in dispatch order, so
// they fill the compute units as the ranges drain.
template <int RB, bool FP8>
__global__ __launch_bounds__(4 * kThreads, 2) void mixed_flash_span(KvView kv, const uint16_t* q, int n_q, RangeWs ws, uint16_t* out,
                                                                    int n_groups, DecodeArgs da, DecWs dws, int span_rows, int nspan) {
  constexpr int kFlashLds = kVTileBytes + (RB * 16 + 1) * kKRow;        // of one wavefront of the verification pass
  static_assert(kFlashLds % 16 == 0 && kFlashLds >= kVTileBytes, "the draft path uses the same memory as four tile buffers");
  __shared__ __attribute__((aligned(16))) uint8_t smem[4 * kFlashLds];
  if (static_cast<int>(blockIdx.x) < n_groups) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kThreads), lane = threadIdx.x & (kThreads - 1);   // scalar: LDS bases stay out of the vector registers
    const int w = blockIdx.x * 4 + wave;
    if (w < ws.n_ranges)
      flash_range_body<RB, FP8, true>(kv, q, n_q, ws, out, smem + wave * kFlashLds, smem + wave * kFlashLds + kVTileBytes, w, lane);
  } else {
    const int i = blockIdx.x - n_groups;
    const int sp = i % nspan, pg = i / nspan;
    decode_span_body<FP8, 4>(da, dws, span_rows, nspan, pg / da.kv.num_kv_heads, pg % da.kv.num_kv_heads, sp,
                          reinterpret_cast<uint8_t (*)[kVTileBytes]>(smem));
  }
}

// ------------------------------------------ 3 and 4 row blocks: two wavefronts per range ----
// With more than 32 query rows the accumulators of a wavefront leave room for one wavefront per
// SIMD only, and the pass is bound by that wavefront's own instruction stream.  Here two
// wavefronts share a range: both walk the same tile stream, each fetches one 16-token half of
// every tile into the shared LDS tile, and each keeps the accumulators of its own row blocks
// (blocks 0-1, and the rest).  Four workgroup barriers per tile order the use of the one buffer:
// K halves written | S^T read | V halves written | O^T read.
template <bool FP8> struct HalfRegs { static constexpr int kLoads = TileRegs<FP8>::kLoads / 2; };

// pages of both 16-token groups of the tile at tb (the window only moves forward), loads of group `half` only
template <bool FP8>
__device__ __forceinline__ void issue_half(const KvView& kv, const Segment& sg, int tb, int half, PageWin& pw, const LaneGeom<FP8>& geo,
                                           int lane, u32x4 (&rk)[HalfRegs<FP8>::kLoads], u32x4 (&rv)[HalfRegs<FP8>::kLoads],
                                           int (&pages)[2]) {
  constexpr int kPerGroup = HalfRegs<FP8>::kLoads;
  const int esz = FP8 ? 1 : 2;
  const int last_page = (sg.L - 1) >> kv.page_shift;
#pragma unroll
  for (int grp = 0; grp < 2; ++grp) {
    const int lp = min((tb + 16 * grp) >> kv.page_shift, last_page);
    if (lp / kWindowPages > pw.win) {          // wave-uniform
      pw.pg_a = pw.pg_b;
      pw.win += 1;
      pw.pg_b = load_window(kv, sg.b, pw.win + 1, lane);
    }
    pages[grp] = __builtin_amdgcn_readlane(pw.pg_a, lp - pw.win * kWindowPages);
  }
  const int tok0 = tb + 16 * half;
  const int page = half == 0 ? pages[0] : pages[1];
  const int64_t base = (static_cast<int64_t>(page) * kv.stride_page + static_cast<int64_t>(sg.g) * kv.stride_head +
                        static_cast<int64_t>(tok0 & (kv.page_size - 1)) * kv.stride_slot) * esz;
  const char* gk = static_cast<const char*>(kv.k_pool) + base;
  const char* gv = static_cast<const char*>(kv.v_pool) + base;
#pragma unroll
  for (int u = 0; u < kPerGroup; ++u) {
    const uint32_t off = geo.lane_off + u * geo.row_step;
    rk[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gk + off));
    rv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gv + off));
  }
}

template <bool FP8>
__device__ __forceinline__ Flight issue_next_half(const KvView& kv, Cursor& c, int half, const LaneGeom<FP8>& geo, int lane,
                                                  u32x4 (&rk)[HalfRegs<FP8>::kLoads], u32x4 (&rv)[HalfRegs<FP8>::kLoads]) {
  Flight f;
  f.valid = c.live;
  f.sg = c.sg;
  f.tb = c.tile * kTileTokens;
  f.pages[0] = f.pages[1] = 0;
  f.ks[0] = f.ks[1] = f.vs[0] = f.vs[1] = 1.f;
  if (!c.live) return f;
  issue_half<FP8>(kv, c.sg, f.tb, half, c.pw, geo, lane, rk, rv, f.pages);
  fetch_scales<FP8>(kv, f);
  advance_cursor(kv, c, lane);
  return f;
}

template <bool FP8, bool IS_V>
__device__ __forceinline__ void half_to_lds(const u32x4 (&regs)[HalfRegs<FP8>::kLoads], uint8_t* tile, int lane, int half) {
  if constexpr (!FP8) {
    const int c = lane & 15;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = 16 * half + 4 * u + (lane >> 4);
      *reinterpret_cast<u32x4*>(tile + (IS_V ? v_lds_addr(r, c) : k_lds_addr(r, c))) = regs[u];
    }
  } else {
    const int c = (lane & 7) * 2;          // 16 fp8 = two 16-byte bf16 chunks
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int r = 16 * half + 8 * u + (lane >> 3);
      u32x4 lo, hi;
      widen_fp8x16(regs[u], lo, hi);
      *reinterpret_cast<u32x4*>(tile + (IS_V ? v_lds_addr(r, c) : k_lds_addr(r, c))) = lo;
      *reinterpret_cast<u32x4*>(tile + (IS_V ? v_lds_addr(r, c + 1) : k_lds_addr(r, c + 1))) = hi;
    }
  }
}

// S^T of the tile for row blocks rb0 .. rb0+RBW-1, Q operand from LDS
template <int RBW>
__device__ __forceinline__ void tile_qk_ldsq_at(const uint8_t* ktile, const uint8_t* qtile, int R, int rb0, f32x4 (&acc)[2][RBW], int lane) {
  const int n = lane & 15, g = lane >> 4;
  int qrow[RBW];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) qrow[rb] = min(16 * (rb0 + rb) + n, R);
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) acc[sub][rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const bf16x8 a0 = as_bf16x8(*reinterpret_cast<const u32x4*>(ktile + k_lds_addr(n, 4 * s + g)));
    const bf16x8 a1 = as_bf16x8(*reinterpret_cast<const u32x4*>(ktile + k_lds_addr(16 + n, 4 * s + g)));
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      const bf16x8 b = as_bf16x8(*reinterpret_cast<const u32x4*>(qtile + k_lds_addr(qrow[rb], 4 * s + g)));
      acc[0][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, acc[0][rb], 0, 0, 0);
      acc[1][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, acc[1][rb], 0, 0, 0);
    }
    if (RBW > 1) __builtin_amdgcn_sched_barrier(0);
  }
}

// the same with the Q operand in registers: qf[rb][s] holds, for lane (n, g), Q[16 (RB0 + rb) + n][32 s + 8 g .. + 7]
template <int RBW>
__device__ __forceinline__ void tile_qk_regq(const uint8_t* ktile, const bf16x8 (&qf)[RBW][4], f32x4 (&acc)[2][RBW], int lane) {
  const int n = lane & 15, g = lane >> 4;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) acc[sub][rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const bf16x8 a0 = as_bf16x8(*reinterpret_cast<const u32x4*>(ktile + k_lds_addr(n, 4 * s + g)));
    const bf16x8 a1 = as_bf16x8(*reinterpret_cast<const u32x4*>(ktile + k_lds_addr(16 + n, 4 * s + g)));
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      acc[0][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qf[rb][s], acc[0][rb], 0, 0, 0);
      acc[1][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qf[rb][s], acc[1][rb], 0, 0, 0);
    }
  }
}

// one of the two wavefronts: `half` = which 16 tokens of every tile it fetches, RB0 / RBW = its row blocks
template <int RB, bool FP8, bool STASH, int RBW, int RB0>
__device__ __forceinline__ void flash_pair_wave(const KvView& kv, const uint16_t* q, int n_q, const RangeWs& ws, uint16_t* out,
                                                uint8_t* s_tile, uint8_t* s_q, int half) {
  constexpr int kPairThreads = 2 * kThreads;
  const int lane = threadIdx.x & (kThreads - 1);
  const int n = lane & 15, g4 = lane >> 4;
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int nv = R - 16 * (RB - 1);
  const int tile_lanes = (RB - 1) * 64 + 4 * nv;
  const float c2 = kv.sm_scale * kLog2e;
  const LaneGeom<FP8> geo = lane_geom<FP8>(kv, lane);
  constexpr int kHalf = HalfRegs<FP8>::kLoads;
  constexpr int kRowsPerLoad = FP8 ? 8 : 4;
  constexpr int kQIters = ((RB * 16 + 1) * 16 + kPairThreads - 1) / kPairThreads;
  Cursor cur = open_cursor(kv, ws, blockIdx.x, lane);
  if (!cur.live) return;                       // the same for both wavefronts
  int unit = cur.unit;
  // Half tiles in flight per wavefront: two where the registers allow it.  Three row blocks of bf16: 402 against
  // 414 us at 16 requests of 24-32 K tokens (four row blocks would spill).  fp8: the dequantisation scales of a
  // tile must then be fetched along with its rows (issue_next_half), or their load at the tile's turn keeps a
  // round trip to memory in every tile: 394 against 415 us at 64 requests, neither change gains anything alone.
  constexpr int DEPTH = (FP8 || RB == 3) ? 2 : 1;
  u32x4 rk[DEPTH][kHalf], rv[DEPTH][kHalf];
  Flight fl[DEPTH];
#pragma unroll
  for (int j = 0; j < DEPTH; ++j) fl[j] = issue_next_half<FP8>(kv, cur, half, geo, lane, rk[j], rv[j]);
  Segment cs = fl[0].sg;
  bool started = false;
  float m_run[RBW], l_run[RBW];
  f32x4 o[RBW][8];
  int nq_b = n_q, Rb = R;                      // query positions and rows of the current pair's request
  // fp8 with three row blocks: the Q operand lives in registers (there is room, and the LDS of the two-wavefront
  // pass is its busiest unit: 416 -> 407 us at 64 requests of 40 query rows)
  constexpr bool kQRegs = FP8 && RB == 3;
  [[maybe_unused]] bf16x8 qf[RBW][4];
  [[maybe_unused]] bool q_stale = true;
  auto finish = [&]() {
    const bool whole = cs.tile0 == 0 && cs.tile1 == cs.tiles;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      const float l = sum_over_groups(l_run[rb]);
      const int r = 16 * (RB0 + rb) + n;
      if (g4 == 0) {
        ws.part_m[static_cast<int64_t>(cs.slot) * (RB * 16) + r] = m_run[rb];
        ws.part_l[static_cast<int64_t>(cs.slot) * (RB * 16) + r] = l;
      }
      if (r >= Rb) continue;               // rows of query slots the request does not use are left alone
      if (whole) {
        const float inv = l > 0.f ? 1.0f / l : 0.f;       // a row that sees no token: zeros
        const int i = r / G, hg = r - i * G;
        uint16_t* dst = out + ((static_cast<int64_t>(cs.rq) * n_q + i) * kv.num_q_heads + cs.g * G + hg) * kHeadDim;
#pragma unroll
        for (int db = 0; db < 8; ++db) {
          u32x2 pk;
          pk.x = pack2(o[rb][db][0] * inv, o[rb][db][1] * inv);
          pk.y = pack2(o[rb][db][2] * inv, o[rb][db][3] * inv);
          *reinterpret_cast<u32x2*>(dst + 16 * db + 4 * g4) = pk;
        }
      } else {
        float* dst = ws.part_o + (static_cast<int64_t>(cs.slot) * R + r) * kHeadDim + 4 * g4;
#pragma unroll
        for (int db = 0; db < 8; ++db) *reinterpret_cast<f32x4*>(dst + 16 * db) = o[rb][db];
      }
    }
  };
  auto tile = [&](Flight& f, u32x4 (&rk)[kHalf], u32x4 (&rv)[kHalf]) {
    __syncthreads();                           // the previous tile's V rows have been read by both wavefronts
    if (!started || f.sg.slot != cs.slot) {    // workgroup-uniform: the stream has entered another pair
      if (started) finish();
      cs = f.sg;
      started = true;
      q_stale = true;
      nq_b = __builtin_amdgcn_readfirstlane(queries_of(kv, ws, cs.b, n_q));
      Rb = nq_b * G;
      {                                        // Q rows of the pair -> LDS, by both wavefronts (row R is the zero row)
        u32x4 qtmp[kQIters];
#pragma unroll
        for (int j = 0; j < kQIters; ++j) {
          const int ch = static_cast<int>(threadIdx.x) + kPairThreads * j;
          const int r = ch >> 4, c = ch & 15;
          u32x4 v = {0u, 0u, 0u, 0u};
          if (r < Rb) {
            const int i = r / G, hg = r - i * G;
            v = *reinterpret_cast<const u32x4*>(q + ((static_cast<int64_t>(cs.rq) * n_q + i) * kv.num_q_heads + cs.g * G + hg) * kHeadDim + 8 * c);
          }
          qtmp[j] = v;
        }
#pragma unroll
        for (int j = 0; j < kQIters; ++j) {
          const int ch = static_cast<int>(threadIdx.x) + kPairThreads * j;
          if (ch < (R + 1) * 16) *reinterpret_cast<u32x4*>(s_q + k_lds_addr(ch >> 4, ch & 15)) = qtmp[j];
        }
      }
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        m_run[rb] = -INFINITY;
        l_run[rb] = 0.f;
#pragma unroll
        for (int d = 0; d < 8; ++d) o[rb][d] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
    const int tb = f.tb;
    half_to_lds<FP8, false>(rk, s_tile, lane, half);
    const float ks[2] = {f.ks[0], f.ks[1]}, vs[2] = {f.vs[0], f.vs[1]};
    __syncthreads();                           // the K tile (and Q) is complete
    f32x4 s[2][RBW];
    if constexpr (kQRegs) {
      if (q_stale) {                           // first tile of a pair: this wavefront's Q rows, once, from LDS
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
          const int qrow = min(16 * (RB0 + rb) + n, R);
#pragma unroll
          for (int sx = 0; sx < 4; ++sx) qf[rb][sx] = as_bf16x8(*reinterpret_cast<const u32x4*>(s_q + k_lds_addr(qrow, 4 * sx + g4)));
        }
        q_stale = false;
      }
      tile_qk_regq<RBW>(s_tile, qf, s, lane);
    } else {
      tile_qk_ldsq_at<RBW>(s_tile, s_q, R, RB0, s, lane);
    }
    if (tb + kTileTokens > cs.L) {
#pragma unroll
      for (int u = 0; u < kHalf; ++u)
        if (tb + 16 * half + kRowsPerLoad * u + geo.row >= cs.L) rv[u] = u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();                           // both wavefronts have read the K rows
    half_to_lds<FP8, true>(rv, s_tile, lane, half);
    f = issue_next_half<FP8>(kv, cur, half, geo, lane, rk, rv);
    const bool edge = tb + kTileTokens > cs.L - n_q;
    bf16x8 p[RBW];
    uint8_t* st_base = ws.stash + static_cast<int64_t>(unit) * tile_lanes * 16;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      f32x4 pr[2] = {s[0][rb], s[1][rb]};
      if (edge) {
        const int r = 16 * (RB0 + rb) + n;
        const int last = cs.L - nq_b + (r < Rb ? r / G : nq_b - 1);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (tb + 16 * sub + 4 * g4 + i > last) pr[sub][i] = -INFINITY;
      }
      const float sc0 = c2 * ks[0], sc1 = c2 * ks[1];
      float mx = fmaxf(fmaxf(fmaxf(pr[0][0], pr[0][1]), fmaxf(pr[0][2], pr[0][3])) * sc0,
                       fmaxf(fmaxf(pr[1][0], pr[1][1]), fmaxf(pr[1][2], pr[1][3])) * sc1);
      mx = max_over_groups(mx);
      const float m_new = fmaxf(m_run[rb], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      if (__any(m_new > m_run[rb])) {
        const float alpha = fast_exp2(m_run[rb] - m_use);
        l_run[rb] *= alpha;
#pragma unroll
        for (int d = 0; d < 8; ++d) o[rb][d] *= alpha;
      }
      m_run[rb] = m_new;
      float sum = 0.f;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          pr[sub][i] = fast_exp2(fmaf(pr[sub][i], sub == 0 ? sc0 : sc1, -m_use));
          sum += pr[sub][i];
        }
      l_run[rb] += sum;
      const int sl = STASH ? stash_lane(RB0 + rb, RB, nv, n, g4, lane) : -1;
      if (sl >= 0) {
        uint32_t c[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) c[k] = stash_encode(pr[k >> 2][k & 3]);
        u32x4 packed;
        packed.x = c[0] | (c[1] << 16);
        packed.y = c[2] | (c[3] << 16);
        packed.z = c[4] | (c[5] << 16);
        packed.w = c[6] | (c[7] << 16);
        *reinterpret_cast<u32x4*>(st_base + sl * 16) = packed;
      }
      if (STASH && g4 == 0) ws.m_ref[static_cast<int64_t>(unit) * (RB * 16) + 16 * (RB0 + rb) + n] = m_use;
      if constexpr (FP8) { pr[0] *= vs[0]; pr[1] *= vs[1]; }
      p[rb] = pack_p(pr[0], pr[1]);
    }
    __syncthreads();                           // the V tile is complete
    tile_pv<RBW>(s_tile, p, o, lane);
    unit += 1;
  };
  for (bool more = true; more;) {
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      if (!fl[j].valid) { more = false; break; }     // register sets are refilled in order: the first empty one ends the stream
      tile(fl[j], rk[j], rv[j]);
    }
  }
  finish();
}

template <int RB, bool FP8, bool STASH>
__global__ __launch_bounds__(2 * kThreads, RB >= 3 ? 2 : 3) void verify_flash_pair(KvView kv, const uint16_t* q, int n_q, RangeWs ws, uint16_t* out) {
  static_assert(RB >= 2, "two wavefronts need two row blocks");
  // (with 2 row blocks, one each at 3 wavefronts per SIMD, the pass took as long as the one-wavefront kernel:
  // 518 against 523 us at batch 128, so that case keeps the simpler kernel)
  constexpr int kFirst = (RB + 1) / 2;         // row blocks of the first wavefront
  __shared__ __attribute__((aligned(16))) uint8_t s_tile[kVTileBytes];
  __shared__ __attribute__((aligned(16))) uint8_t s_q[(RB * 16 + 1) * kKRow];
  if (threadIdx.x < kThreads) flash_pair_wave<RB, FP8, STASH, kFirst, 0>(kv, q, n_q, ws, out, s_tile, s_q, 0);
  else flash_pair_wave<RB, FP8, STASH, RB - kFirst, kFirst>(kv, q, n_q, ws, out, s_tile, s_q, 1);
}

// A unified batch with more than 32 query rows per KV head: the first n_ranges workgroups are those of
// verify_flash_pair, the others carry one (request, KV head, span) of the draft step each, with two wavefronts.
template <int RB, bool FP8>
__global__ __launch_bounds__(2 * kThreads, 2) void mixed_flash_pair(KvView kv, const uint16_t* q, int n_q, RangeWs ws, uint16_t* out,
                                                                    DecodeArgs da, DecWs dws, int span_rows, int nspan) {
  static_assert(RB >= 3, "up to two row blocks run mixed_flash_span");
  constexpr int kFirst = (RB + 1) / 2;
  constexpr int kPassLds = kVTileBytes + (RB * 16 + 1) * kKRow;
  static_assert(kPassLds >= 2 * kVTileBytes, "the draft path uses the same memory as two tile buffers");
  __shared__ __attribute__((aligned(16))) uint8_t smem[kPassLds];
  if (static_cast<int>(blockIdx.x) < ws.n_ranges) {
    if (threadIdx.x < kThreads) flash_pair_wave<RB, FP8, true, kFirst, 0>(kv, q, n_q, ws, out, smem, smem + kVTileBytes, 0);
    else flash_pair_wave<RB, FP8, true, RB - kFirst, kFirst>(kv, q, n_q, ws, out, smem, smem + kVTileBytes, 1);
  } else {
    const int i = blockIdx.x - ws.n_ranges;
    const int sp = i % nspan, pg = i / nspan;
    decode_span_body<FP8, 2>(da, dws, span_rows, nspan, pg / da.kv.num_kv_heads, pg % da.kv.num_kv_heads, sp,
                             reinterpret_cast<uint8_t (*)[kVTileBytes]>(smem));
  }
}

// Sort key of a score of the statistic: a mean of probabilities lies in [0, 1] (below 2 with any rounding), so the
// sign bit and the top exponent bit of its pattern are zero and can go: the first 12-bit digit of the selection
// then holds 6 exponent and 6 mantissa bits, 64 histogram bins per binade instead of 8, and scores that share a
// few exponents queue up on far fewer LDS addresses.
__device__ __forceinline__ uint32_t score_key(float f) { return __float_as_uint(f) << 2; }

// ------------------------------------------------ finish ---------------------
// Everything that needs the whole pair, in one kernel: one workgroup per (request, KV head), longest
// rows first.
//   1. the log-sum-exp of every row from the (m, l) of the pair's segments;
//   2. O of a pair that was cut into several segments: sum over segments of exp2(m_seg - lse) O_seg
//      (a pair inside one range was finished by the pass itself);
//   3. the score statistic from the stash, scores = mean over rows of e * exp2(m_tile - lse): wavefronts take
//      the pair's tiles in turn, two in flight each, and leave the scores of one chunk of tokens at a time in
//      LDS, from where every thread takes 8 consecutive ones as sort keys into registers (and writes them out
//      if the caller wants the statistic itself);
//   4. SELECT: Top-K of the keys in registers (topk_core.hpp) -- the statistic makes no round trip through
//      memory between two launches (paper Section 4.1: identification from the verification's own
//      intermediates).
// Rows of up to CH * THREADS * 8 tokens; without SELECT any length (the chunk loop is then a run-time one).
// SPLIT (long rows): a pair is shared by up to CH workgroups, blockIdx.y = the chunk of THREADS * 8 tokens each
// of them rebuilds; the statistic goes to memory (the caller's buffer, else scratch) and verify_select_rows, the
// next launch, selects from it.  The first chunk's workgroup also does step 1's output and step 2.  (Handing the
// chunks to the last workgroup to arrive inside one launch was measured: the device-wide release every workgroup
// then needs writes back the whole L2 behind it, 3 to 5 times the cost of the extra launch.)
template <int RB, int THREADS, int CH, bool SELECT, bool SPLIT>
__global__ __launch_bounds__(THREADS) void verify_finish(KvView kv, int n_q, RangeWs ws, uint16_t* out, float* lse_out,
                                                         float* scores, int64_t score_stride, SelectOut sel) {
  static_assert(!SPLIT || !SELECT, "a split pair is selected by verify_select_rows");
  constexpr int KPC = 8;
  constexpr int kChunk = THREADS * KPC;                      // tokens whose scores LDS holds at a time
  constexpr int kChunkTiles = kChunk / kTileTokens;
  constexpr int kWaves = THREADS / kWave;
  __shared__ __attribute__((aligned(16))) float s_scores[kChunk];
  __shared__ float s_lse[RB * 16];
  __shared__ SelectLds<THREADS, CH> lds;
  const int pair = ws.order[blockIdx.x];
  const int b = pair / kv.num_kv_heads, g = pair - b * kv.num_kv_heads;
  const int rq = request_of(kv, b);
  const int L = kv.seq_lens[rq];
  const int tiles = tiles_of_len(L);
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int R = n_q * G;
  const int Rb = queries_of(kv, ws, b, n_q) * G;
  constexpr int rows = RB * 16;
  const int total = ws.ctrl[0];
  const int u0 = ws.ureq[b] + g * tiles;
  const int w0 = range_of(u0, total, ws.n_ranges), w1 = range_of(u0 + tiles - 1, total, ws.n_ranges);
  const int my_chunk = SPLIT ? static_cast<int>(blockIdx.y) : 0;
  if (SPLIT && my_chunk * kChunk >= L) return;          // this pair has fewer chunks (uniform over the workgroup)
  const bool lead = my_chunk == 0;                       // the workgroup that writes what exists once per pair
  int K = 0;
  int32_t* out_idx = nullptr;
  if constexpr (SELECT) {
    K = max(0, min(min(sel.budgets[rq], L), sel.max_budget));
    out_idx = sel.indices + (static_cast<int64_t>(rq) * kv.num_kv_heads + g) * sel.max_budget;
    if (g == 0 && threadIdx.x == 0) sel.counts[rq] = K;
    for (int j = K + threadIdx.x; j < sel.max_budget; j += THREADS) out_idx[j] = -1;
  }

  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int n = lane & 15, g4 = lane >> 4;
  const int nv = R - 16 * (RB - 1);
  const int tile_lanes = (RB - 1) * 64 + 4 * nv;
  const bool want_scores = SELECT || SPLIT || scores;

  // The stash stream: wavefronts take the tiles of a chunk in turn, kBufs tiles in flight each.
  constexpr int kBufs = THREADS >= 1024 ? 2 : 4;       // (a 1024-thread workgroup has 128 registers per lane)
  int sl[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) sl[rb] = stash_lane(rb, RB, nv, n, g4, lane);
  u32x4 st[kBufs][RB];
  float mref[kBufs][RB];
  auto fetch = [&](int tile, int buf) {
    const int64_t u = u0 + tile;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      st[buf][rb] = u32x4{0u, 0u, 0u, 0u};
      if (sl[rb] >= 0)
        st[buf][rb] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ws.stash + (u * tile_lanes + sl[rb]) * 16));
      mref[buf][rb] = __builtin_nontemporal_load(ws.m_ref + u * rows + 16 * rb + n);
    }
  };
  auto prime = [&](int c) {                              // first tiles of chunk c on their way
    const int t_begin = c * kChunkTiles, t_end = min(tiles, t_begin + kChunkTiles);
#pragma unroll
    for (int i = 0; i < kBufs; ++i)
      if (t_begin + wave + i * kWaves < t_end) fetch(t_begin + wave + i * kWaves, i);
  };
  if (want_scores) prime(my_chunk);                    // needs nothing of steps 1 and 2: in flight meanwhile

  // 1. log-sum-exp per row (log2 domain).  Rows beyond the request's own, and rows that see no token at all,
  // get +inf: their probabilities vanish wherever the log-sum-exp is applied.
  // 2. O of a pair cut into several segments.  The partials of up to kSegs segments are fetched before the
  // log-sum-exp is known (every thread owns up to kOuts pieces of 4 dims), so both waits overlap.
  constexpr int kSegs = THREADS >= 1024 ? 2 : 5;
  constexpr int kOuts = (RB * 16 * (kHeadDim / 4) + THREADS - 1) / THREADS;
  const int nseg = w1 - w0 + 1;
  const bool split = w1 > w0 && lead;
  const bool early = split && nseg <= kSegs && total >= ws.n_ranges;     // (no empty ranges when there are as many units as ranges)
  f32x4 po[kOuts][kSegs];
  float pm[kOuts][kSegs];
  if (early) {
#pragma unroll
    for (int o = 0; o < kOuts; ++o) {
      const int idx = threadIdx.x + o * THREADS;
      const int r = idx / (kHeadDim / 4), d4 = idx - r * (kHeadDim / 4);
#pragma unroll
      for (int sg = 0; sg < kSegs; ++sg) {
        po[o][sg] = f32x4{0.f, 0.f, 0.f, 0.f};
        pm[o][sg] = -INFINITY;
        if (r < Rb && sg < nseg) {
          po[o][sg] = *reinterpret_cast<const f32x4*>(ws.part_o + (static_cast<int64_t>(pair + w0 + sg) * R + r) * kHeadDim + 4 * d4);
          pm[o][sg] = ws.part_m[static_cast<int64_t>(pair + w0 + sg) * rows + r];
        }
      }
    }
  }
  if (threadIdx.x < rows) {
    const int row = threadIdx.x;
    float m = -INFINITY, l = 0.f;
    auto add = [&](float mc, float lc) {
      const float mn = fmaxf(m, mc);
      const float mu = (mn == -INFINITY) ? 0.f : mn;
      l = l * fast_exp2(m - mu) + lc * fast_exp2(mc - mu);
      m = mn;
    };
    if (nseg <= kSegs && total >= ws.n_ranges) {       // all segments exist: their (m, l) leave together
      float mc[kSegs], lc[kSegs];
#pragma unroll
      for (int sg = 0; sg < kSegs; ++sg) {
        mc[sg] = -INFINITY;
        lc[sg] = 0.f;
        if (sg < nseg) {
          mc[sg] = ws.part_m[static_cast<int64_t>(pair + w0 + sg) * rows + row];
          lc[sg] = ws.part_l[static_cast<int64_t>(pair + w0 + sg) * rows + row];
        }
      }
#pragma unroll
      for (int sg = 0; sg < kSegs; ++sg) add(mc[sg], lc[sg]);     // an absent segment adds exp2(-inf) * 0
    } else {
      for (int w = w0; w <= w1; ++w) {
        // with fewer units than ranges some ranges are empty and own no segment
        if (range_begin(w, total, ws.n_ranges) == range_begin(w + 1, total, ws.n_ranges)) continue;
        add(ws.part_m[static_cast<int64_t>(pair + w) * rows + row], ws.part_l[static_cast<int64_t>(pair + w) * rows + row]);
      }
    }
    const bool live = row < Rb && l > 0.f;
    const float v = live ? m + log2f(l) : INFINITY;
    s_lse[row] = v;
    if (lse_out && row < Rb && lead) {
      const int i = row / G, hg = row - i * G;
      lse_out[(static_cast<int64_t>(rq) * n_q + i) * kv.num_q_heads + g * G + hg] = live ? v * kLn2 : -INFINITY;
    }
  }
  __syncthreads();
  if (split) {
    auto store_o = [&](int r, int d4, const f32x4& acc) {
      const int i = r / G, hg = r - i * G;
      uint16_t* dst = out + ((static_cast<int64_t>(rq) * n_q + i) * kv.num_q_heads + g * G + hg) * kHeadDim;
      u32x2 pk;
      pk.x = pack2(acc.x, acc.y);
      pk.y = pack2(acc.z, acc.w);
      *reinterpret_cast<u32x2*>(dst + 4 * d4) = pk;
    };
    if (early) {
#pragma unroll
      for (int o = 0; o < kOuts; ++o) {
        const int idx = threadIdx.x + o * THREADS;
        const int r = idx / (kHeadDim / 4), d4 = idx - r * (kHeadDim / 4);
        if (r < Rb) {
          const float lse = s_lse[r];
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int sg = 0; sg < kSegs; ++sg) acc += po[o][sg] * fast_exp2(pm[o][sg] - lse);   // absent segments: exp2(-inf) = 0
          store_o(r, d4, acc);
        }
      }
    } else {
      for (int idx = threadIdx.x; idx < Rb * (kHeadDim / 4); idx += THREADS) {
        const int r = idx / (kHeadDim / 4), d4 = idx - r * (kHeadDim / 4);
        const float lse = s_lse[r];
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int w = w0; w <= w1; ++w) {
          if (range_begin(w, total, ws.n_ranges) == range_begin(w + 1, total, ws.n_ranges)) continue;   // empty range
          const float f = fast_exp2(ws.part_m[static_cast<int64_t>(pair + w) * rows + r] - lse);
          acc += *reinterpret_cast<const f32x4*>(ws.part_o + (static_cast<int64_t>(pair + w) * R + r) * kHeadDim + 4 * d4) * f;
        }
        store_o(r, d4, acc);
      }
    }
  }
  if (!want_scores) return;

  // 3. scores of the pair, chunk by chunk
  const float log2_inv_r = -log2f(static_cast<float>(Rb));
  float bias[RB];                                      // per row: -lse + the stash's 2^64 + log2(1 / rows)
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) bias[rb] = kStashBias + log2_inv_r - s_lse[16 * rb + n];   // -inf for rows that carry no weight
  auto tile_out = [&](int slot, int buf) {             // slot = tile within the chunk
    f32x4 tot[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float w = fast_exp2(mref[buf][rb] + bias[rb]);
      const uint32_t h[4] = {st[buf][rb].x, st[buf][rb].y, st[buf][rb].z, st[buf][rb].w};
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const uint32_t c = (k & 1) ? (h[k >> 1] >> 16) : (h[k >> 1] & 0xffffu);
        tot[k >> 2][k & 3] = fmaf(stash_decode_scaled(c), w, tot[k >> 2][k & 3]);
      }
    }
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int i = 0; i < 4; ++i) tot[sub][i] = row16_sum(tot[sub][i]);
      if (n == 0) *reinterpret_cast<f32x4*>(s_scores + slot * kTileTokens + 16 * sub + 4 * g4) = tot[sub];
    }
  };
  float* sdst = scores ? scores + (static_cast<int64_t>(rq) * kv.num_kv_heads + g) * score_stride : nullptr;
  if (SPLIT && !sdst) sdst = ws.scratch_scores + static_cast<int64_t>(pair) * ws.scratch_stride;
  uint32_t key[CH][KPC];
  auto chunk = [&](int c, uint32_t (&keys)[KPC]) {
    const int t_begin = c * kChunkTiles, t_end = min(tiles, t_begin + kChunkTiles);
    for (int tile = t_begin + wave; tile < t_end;) {
#pragma unroll
      for (int i = 0; i < kBufs; ++i) {
        if (tile < t_end) {
          tile_out(tile - t_begin, i);
          if (tile + kBufs * kWaves < t_end) fetch(tile + kBufs * kWaves, i);      // buffer i is free again
          tile += kWaves;
        }
      }
    }
    if (!SPLIT && (c + 1) * kChunk < L) prime(c + 1);   // the next chunk's first tiles leave before the barriers
    __syncthreads();
    const int p0 = c * kChunk + static_cast<int>(threadIdx.x) * KPC;      // this thread's 8 positions
#pragma unroll
    for (int j = 0; j < KPC; j += 4) {
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (p0 + j < t_end * kTileTokens) v = *reinterpret_cast<const f32x4*>(s_scores + static_cast<int>(threadIdx.x) * KPC + j);
#pragma unroll
      for (int i = 0; i < 4; ++i) keys[j + i] = score_key(v[i]);
      if (sdst) {
        if (p0 + j + 3 < L) {
          *reinterpret_cast<f32x4*>(sdst + p0 + j) = v;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (p0 + j + i < L) sdst[p0 + j + i] = v[i];
        }
      }
    }
    __syncthreads();                                   // the next chunk overwrites the scores
  };
  if constexpr (SPLIT) {
    chunk(my_chunk, key[0]);                           // the scores of this chunk go to memory
  } else if constexpr (SELECT) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      if (c * kChunk < L) {                            // uniform over the workgroup
        chunk(c, key[c]);
      } else {
#pragma unroll
        for (int j = 0; j < KPC; ++j) key[c][j] = 0u;
      }
    }
    if (K > 0) select_topk_in_registers<THREADS, KPC, CH>(key, L, K, out_idx, lds);
  } else {
    for (int c = 0; c * kChunk < L; ++c) chunk(c, key[0]);
  }
}

// Top-K of the statistic of long rows, from memory: one workgroup per (request, KV head), longest first; thread t
// holds positions c * 8192 + 8 t .. + 7 of each chunk c (the same ownership as in verify_finish).
template <int CH>
__global__ __launch_bounds__(1024) void verify_select_rows(KvView kv, RangeWs ws, const float* scores, int64_t score_stride,
                                                           SelectOut sel) {
  constexpr int THREADS = 1024, KPC = 8, kChunk = THREADS * KPC;
  __shared__ SelectLds<THREADS, CH> lds;
  const int pair = ws.order[blockIdx.x];
  const int b = pair / kv.num_kv_heads, g = pair - b * kv.num_kv_heads;
  const int rq = request_of(kv, b);
  const int L = kv.seq_lens[rq];
  const int K = max(0, min(min(sel.budgets[rq], L), sel.max_budget));
  int32_t* out_idx = sel.indices + (static_cast<int64_t>(rq) * kv.num_kv_heads + g) * sel.max_budget;
  if (g == 0 && threadIdx.x == 0) sel.counts[rq] = K;
  for (int j = K + threadIdx.x; j < sel.max_budget; j += THREADS) out_idx[j] = -1;
  if (K == 0) return;
  const float* src = scores ? scores + (static_cast<int64_t>(rq) * kv.num_kv_heads + g) * score_stride
                            : ws.scratch_scores + static_cast<int64_t>(pair) * ws.scratch_stride;
  uint32_t key[CH][KPC];
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    const int p0 = c * kChunk + static_cast<int>(threadIdx.x) * KPC;
#pragma unroll
    for (int j = 0; j < KPC; j += 4) {
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (p0 + j + 3 < L) {
        v = *reinterpret_cast<const f32x4*>(src + p0 + j);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (p0 + j + i < L) v[i] = src[p0 + j + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) key[c][j + i] = score_key(v[i]);
    }
  }
  select_topk_in_registers<THREADS, KPC, CH>(key, L, K, out_idx, lds);
}

// ---------------------------------------------------------------- host ------
int num_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    cus = v;
  }
  return cus;
}

// Ranges per compute unit: as many wavefronts as it holds at once (registers: 2 per SIMD up to 32 rows, else 1;
// LDS allows as many).  Small workloads take fewer, down to half: below about 24 tiles per range the pass gains
// nothing from more wavefronts, and every further cut of a pair is one more segment for the finish kernel to
// merge (32 requests of 4096 tokens: finish 27 us with 8 per compute unit, 23 with 5, pass unchanged).
int ranges_for(const KvView& kv, int rb) {
  int per_cu = rb >= 3 ? 4 : 8;
  const int opt = options().verify_waves;
  if (opt > 0 && opt <= per_cu) return opt * num_cus();
  const int64_t units_max = static_cast<int64_t>(kv.batch) * kv.num_kv_heads * tiles_of_len(kv.max_seq_len);
  const int fit = static_cast<int>(std::min<int64_t>(per_cu, units_max / (24 * static_cast<int64_t>(num_cus()))));
  per_cu = std::max(per_cu / 2, fit);
  return per_cu * num_cus();
}

int row_blocks(const KvView& kv, int n_q) { return (n_q * (kv.num_q_heads / kv.num_kv_heads) + 15) / 16; }

RangeWs carve(const KvView& kv, int n_q, void* workspace, size_t* total_bytes) {
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const size_t R = static_cast<size_t>(n_q) * G;
  const size_t rpad = (R + 15) / 16 * 16;
  const size_t pairs = static_cast<size_t>(kv.batch) * kv.num_kv_heads;
  const size_t n = static_cast<size_t>(ranges_for(kv, static_cast<int>(rpad / 16)));
  const size_t slots = pairs + n;
  char* p = static_cast<char*>(workspace);
  size_t off = 0;
  auto take = [&](size_t bytes) { char* r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
  RangeWs w;
  w.ctrl = reinterpret_cast<int32_t*>(take(64 * 4));
  w.ureq = reinterpret_cast<int32_t*>(take((static_cast<size_t>(kv.batch) + 1) * 4));
  w.order = reinterpret_cast<int32_t*>(take(pairs * 4));
  w.scratch_scores = nullptr;
  w.scratch_stride = 0;
  w.part_m = reinterpret_cast<float*>(take(slots * rpad * 4));
  w.part_l = reinterpret_cast<float*>(take(slots * rpad * 4));
  w.part_o = reinterpret_cast<float*>(take(slots * R * kHeadDim * 4));
  w.lse2 = reinterpret_cast<float*>(take(pairs * rpad * 4));
  const size_t units = pairs * tiles_of_len(kv.max_seq_len);
  const size_t tile_lanes = (rpad / 16 - 1) * 64 + 4 * (R - (rpad - 16));
  w.stash = reinterpret_cast<uint8_t*>(take(units * tile_lanes * 16));
  w.m_ref = reinterpret_cast<float*>(take(units * rpad * 4));
  w.spec_lens = nullptr;
  w.rows_pad = static_cast<int32_t>(rpad);
  w.n_ranges = static_cast<int32_t>(n);
  w.plan_in_wave = 0;
  if (total_bytes) *total_bytes = off;
  return w;
}

template <int RB, bool FP8>
hipError_t run(const VerifyArgs& a, hipStream_t st, const DecodeArgs* draft) {
  const KvView& kv = a.kv;
  RangeWs ws = carve(kv, a.n_q, a.workspace, nullptr);
  ws.spec_lens = a.spec_lens;
  ws.scratch_scores = a.scratch_scores;
  ws.scratch_stride = a.scratch_stride;
  const uint16_t* q = static_cast<const uint16_t*>(a.q);
  uint16_t* out = static_cast<uint16_t*>(a.out);
  const int pairs = kv.batch * kv.num_kv_heads;
  const bool single_pass = !a.exact_scores || !(a.scores || a.select);
  ws.plan_in_wave = single_pass && kv.batch <= kWave * kPlanRegs;
  if (!ws.plan_in_wave) {
    KernelTimer t("verify_range_plan", st);
    hipLaunchKernelGGL(range_plan, dim3(1), dim3(1024), 0, st, kv, ws);
  }
  if (single_pass) {
    bool fused = false;
    if constexpr (RB <= 2) {
      if (draft) {                             // a unified batch: the draft step of other requests rides in the same grid
        fused = true;
        KernelTimer t("mixed_flash_span", st);
        const int span_rows = decode_span_rows(draft->kv, draft->max_budget);
        const int nspan = (draft->max_budget + span_rows - 1) / span_rows;
        const DecWs dws = decode_carve(draft->kv, draft->max_budget, draft->workspace);
        const int n_groups = (ws.n_ranges + 3) / 4;
        const int n_draft = nspan * draft->kv.num_kv_heads * draft->kv.batch;
        hipLaunchKernelGGL((mixed_flash_span<RB, FP8>), dim3(n_groups + n_draft), dim3(4 * kThreads), 0, st, kv, q, a.n_q, ws, out,
                           n_groups, *draft, dws, span_rows, nspan);
      }
    } else {
      if (draft) {                             // the same with two wavefronts per range and per draft workgroup
        fused = true;
        KernelTimer t("mixed_flash_pair", st);
        const int span_rows = decode_span_rows(draft->kv, draft->max_budget);
        const int nspan = (draft->max_budget + span_rows - 1) / span_rows;
        const DecWs dws = decode_carve(draft->kv, draft->max_budget, draft->workspace);
        const int n_draft = nspan * draft->kv.num_kv_heads * draft->kv.batch;
        hipLaunchKernelGGL((mixed_flash_pair<RB, FP8>), dim3(ws.n_ranges + n_draft), dim3(2 * kThreads), 0, st, kv, q, a.n_q, ws, out,
                           *draft, dws, span_rows, nspan);
      }
    }
    if (!fused) {
      KernelTimer t("verify_flash_range", st);
      const bool stash = a.scores || a.select;
      if constexpr (RB >= 3) {                 // two wavefronts per range
        if (stash)
          hipLaunchKernelGGL((verify_flash_pair<RB, FP8, true>), dim3(ws.n_ranges), dim3(2 * kThreads), 0, st, kv, q, a.n_q, ws, out);
        else                                   // plain multi-query decode: nothing is stashed, nothing rebuilt
          hipLaunchKernelGGL((verify_flash_pair<RB, FP8, false>), dim3(ws.n_ranges), dim3(2 * kThreads), 0, st, kv, q, a.n_q, ws, out);
      } else {
        if (stash)
          hipLaunchKernelGGL((verify_flash_range<RB, FP8, true>), dim3(ws.n_ranges), dim3(kThreads), 0, st, kv, q, a.n_q, ws, out);
        else
          hipLaunchKernelGGL((verify_flash_range<RB, FP8, false>), dim3(ws.n_ranges), dim3(kThreads), 0, st, kv, q, a.n_q, ws, out);
      }
    }
    int split_select = 0;                      // chunks per row when the selection is a launch of its own
    SelectOut sel{};
    {
      // one workgroup per pair: log-sum-exp, O of split pairs, scores, selection
      KernelTimer t("verify_finish", st);
      sel = a.select ? *a.select : SelectOut{};
#define PILLAR_FINISH(THREADS, CH, SELECT)                                                                                           \
  hipLaunchKernelGGL((verify_finish<RB, THREADS, CH, SELECT, false>), dim3(pairs), dim3(THREADS), 0, st, kv, a.n_q, ws, out, a.lse, \
                     a.scores, a.score_stride, sel)
#define PILLAR_FINISH_SPLIT(CH)                                                                                                   \
  {                                                                                                                               \
    const int nchunks = (kv.max_seq_len + 8191) / 8192;                                                                           \
    hipLaunchKernelGGL((verify_finish<RB, 1024, 1, false, true>), dim3(pairs, nchunks), dim3(1024), 0, st, kv, a.n_q, ws, out,    \
                       a.lse, a.scores, a.score_stride, sel);                                                                     \
    split_select = CH;                                                                                                            \
  }
      // few pairs (a unified batch with a handful of verifying requests): every pair gets 16 wavefronts, the
      // kernel then lasts as long as its longest pair; rows beyond 8192 tokens are shared by several workgroups
      const bool few = pairs <= 2 * num_cus();
      if (!a.select && a.scores && kv.max_seq_len > 8192 && pairs <= num_cus()) PILLAR_FINISH_SPLIT(0)   // (statistic only)
      else if (!a.select) PILLAR_FINISH(512, 1, false);
      else if (kv.max_seq_len <= 4096 && !few) PILLAR_FINISH(512, 1, true);
      else if (kv.max_seq_len <= 8192 && few) PILLAR_FINISH(1024, 1, true);
      else if (kv.max_seq_len <= 8192) PILLAR_FINISH(512, 2, true);
      // long rows: with fewer pairs than compute units a pair is shared by several workgroups (measured at 128 pairs
      // of 28 K tokens: 121 against 142 us); with more pairs one workgroup per pair keeps everything in one launch
      // (512 pairs of up to 32 K tokens: 149 against 163 us)
      else if (kv.max_seq_len <= 16384 && pairs <= num_cus()) PILLAR_FINISH_SPLIT(2)
      else if (kv.max_seq_len <= 16384) PILLAR_FINISH(1024, 2, true);
      else if (pairs <= num_cus()) PILLAR_FINISH_SPLIT(4)
      else PILLAR_FINISH(1024, 4, true);
#undef PILLAR_FINISH_SPLIT
#undef PILLAR_FINISH
    }
    if (split_select) {
      KernelTimer t("verify_select_rows", st);
      if (split_select == 2) hipLaunchKernelGGL((verify_select_rows<2>), dim3(pairs), dim3(1024), 0, st, kv, ws, a.scores, a.score_stride, sel);
      else hipLaunchKernelGGL((verify_select_rows<4>), dim3(pairs), dim3(1024), 0, st, kv, ws, a.scores, a.score_stride, sel);
    }
    if (fused) {
      const hipError_t e = launch_decode_merge(*draft, st);      // only lists longer than one span leave partials
      if (e != hipSuccess) return e;
    }
    return hipGetLastError();
  }
  {
    KernelTimer t("verify_lse_range", st);
    hipLaunchKernelGGL((verify_lse_range<RB, FP8>), dim3(ws.n_ranges), dim3(kThreads), 0, st, kv, q, a.n_q, ws);
  }
  {
    KernelTimer t("verify_lse_combine", st);
    hipLaunchKernelGGL(verify_lse_combine_range, dim3((pairs * ws.rows_pad + 255) / 256), dim3(256), 0, st, kv, a.n_q, ws, a.lse);
  }
  {
    KernelTimer t("verify_score_range", st);
    hipLaunchKernelGGL((verify_score_range<RB, FP8>), dim3(ws.n_ranges), dim3(kThreads), 0, st, kv, q, a.n_q, ws, out, a.scores,
                       a.score_stride);
  }
  {
    KernelTimer t("verify_o_merge", st);
    hipLaunchKernelGGL(verify_o_merge_range, dim3(pairs), dim3(256), 0, st, kv, a.n_q, ws, out);
  }
  return hipGetLastError();
}

}  // namespace

bool verify_range_supported(const VerifyArgs& a) {
  const KvView& kv = a.kv;
  if (a.q_dtype != PILLAR_BF16) return false;
  if (a.kv_dtype != PILLAR_BF16 && a.kv_dtype != PILLAR_FP8_E4M3) return false;
  if (kv.head_dim != kHeadDim || kv.page_size < 16) return false;
  if (row_blocks(kv, a.n_q) > 4) return false;
  if (!(kv.sm_scale > 0.f)) return false;       // the kernels take row maxima before scaling
  if (a.spec_lens && a.exact_scores) return false;   // per-request lengths: single-pass kernels only
  const int64_t align = a.kv_dtype == PILLAR_BF16 ? 8 : 16;      // elements per 16 bytes
  if (kv.stride_page % align || kv.stride_head % align || kv.stride_slot % align) return false;
  if ((reinterpret_cast<uintptr_t>(kv.k_pool) | reinterpret_cast<uintptr_t>(kv.v_pool) | reinterpret_cast<uintptr_t>(a.q) |
       reinterpret_cast<uintptr_t>(a.out)) & 15u)
    return false;
  // the statistic is stored four tokens at a time
  if (a.scores && ((reinterpret_cast<uintptr_t>(a.scores) & 15u) || (a.score_stride & 3))) return false;
  // units are counted in 32 bits
  const int64_t units = static_cast<int64_t>(kv.batch) * kv.num_kv_heads * tiles_of_len(kv.max_seq_len);
  return units < (int64_t{1} << 30);
}

bool verify_select_fused(const VerifyArgs& a) {
  // the finish kernel keeps the keys of a row in registers: up to 4 chunks of 8192 tokens; longer rows take the two steps
  return a.select && verify_range_supported(a) && !a.exact_scores && a.kv.max_seq_len <= kFinishMaxTokens;
}

size_t verify_range_workspace(const KvView& kv, int n_q) {
  size_t total = 0;
  carve(kv, n_q, nullptr, &total);
  return total;
}

bool verify_fuses_draft(const VerifyArgs& a) {
  // the fused grid holds the single pass with its statistic and in-kernel selection
  return verify_select_fused(a);
}

hipError_t launch_verify_range(const VerifyArgs& a, hipStream_t s, const DecodeArgs* fused_draft) {
  const int rb = row_blocks(a.kv, a.n_q);
  const bool fp8 = a.kv_dtype == PILLAR_FP8_E4M3;
#define PILLAR_CASE(N) \
  if (rb == N) return fp8 ? run<N, true>(a, s, fused_draft) : run<N, false>(a, s, fused_draft);
  PILLAR_CASE(1)
  PILLAR_CASE(2)
  PILLAR_CASE(3)
  PILLAR_CASE(4)
#undef PILLAR_CASE
  return hipErrorInvalidValue;
}

}  // namespace pillar
