// Sparse draft attention on the matrix cores (bf16 queries, bf16 or fp8 KV,
// head_dim 128).
//
// Paper Sections 1 and 4.2: a draft step loads only the critical tokens chosen
// at the last verification; addressing the KV-Cache row by row ("page size 1")
// makes it the same pipeline as full attention, driven by an index list.  The
// step is a gather of 256-byte rows (128-byte for fp8) and is bound by memory
// latency, so the kernel's job is to get every row load of a (request, KV head)
// in flight as early as possible; the G query rows of the group ride along as
// one 16-row MFMA block (the tile engine of mfma_tile.hpp with R = G).
//
// One workgroup of kWaves wavefronts per (request, KV head, span of the index
// list): the wavefronts take the 32-row tiles of the span in turn, each with the
// gather of its next tile (index -> page id) resolved while the rows of the
// current one are in flight, and combine their (max, sum, O) through LDS at the
// end, so a list that fits one span (512 rows) is finished by the one launch.
// Longer lists leave one partial per span that a second small kernel combines.
// The count of a request and its first index entries are fetched side by side:
// the chain a wavefront waits through before its first row load is then
// count | index -> page id -> row.
#include <algorithm>
#include <mutex>

#include "decode_span.hpp"

namespace pillar {
namespace {

constexpr int kMergeThreads = 256;
constexpr int kSpanRows = 512;                 // rows of an index list one workgroup takes


template <bool FP8>
__global__ __launch_bounds__(kDecThreads, 3) void decode_span_mfma(DecodeArgs a, DecWs ws, int span_rows, int nspan_max) {
  __shared__ __attribute__((aligned(16))) uint8_t s_tiles[kDecWaves][kVTileBytes];
  decode_span_body<FP8, kDecWaves>(a, ws, span_rows, nspan_max, blockIdx.z, blockIdx.y, blockIdx.x, s_tiles);
}

__global__ __launch_bounds__(kMergeThreads) void decode_merge_mfma(DecodeArgs a, DecWs ws, int split_rows, int nsplit_max) {
  const KvView& kv = a.kv;
  const int slot_b = blockIdx.y, g = blockIdx.x;
  const int b = request_of(kv, slot_b);
  const int G = kv.num_q_heads / kv.num_kv_heads;
  const int count = min(max(a.counts[b], 0), a.max_budget);
  const int nsplit = (count + split_rows - 1) / split_rows;
  if (nsplit <= 1) return;
  uint16_t* out = static_cast<uint16_t*>(a.out);
  const int64_t base = (static_cast<int64_t>(slot_b) * kv.num_kv_heads + g) * nsplit_max;
  for (int idx = threadIdx.x; idx < G * (kHeadDim / 4); idx += kMergeThreads) {
    const int r = idx / (kHeadDim / 4), d4 = idx - r * (kHeadDim / 4);
    float m = -INFINITY;
    for (int s = 0; s < nsplit; ++s) m = fmaxf(m, ws.part_m[(base + s) * 16 + r]);
    float l = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < nsplit; ++s) {
      const float w = exp2f(ws.part_m[(base + s) * 16 + r] - m);
      l = fmaf(ws.part_l[(base + s) * 16 + r], w, l);
      acc += *reinterpret_cast<const f32x4*>(ws.part_o + ((base + s) * G + r) * kHeadDim + 4 * d4) * w;
    }
    const float inv = 1.0f / l;
    const int64_t row = static_cast<int64_t>(b) * kv.num_q_heads + g * G + r;
    u32x2 pk;
    pk.x = pack_bf16x2(acc.x * inv, acc.y * inv);
    pk.y = pack_bf16x2(acc.z * inv, acc.w * inv);
    *reinterpret_cast<u32x2*>(out + row * kHeadDim + 4 * d4) = pk;
    if (d4 == 0 && a.lse) a.lse[row] = (m + log2f(l)) * kLn2;
  }
}

// rows of the index list per workgroup
int pick_split_rows(const KvView& kv, int max_budget) {
  (void)kv;
  (void)max_budget;
  if (options().decode_rows > 0) return options().decode_rows;
  return kSpanRows;
}

DecWs carve(const KvView& kv, int max_budget, void* workspace, size_t* total) {
  const int split_rows = pick_split_rows(kv, max_budget);
  const size_t nsplit = (static_cast<size_t>(max_budget) + split_rows - 1) / split_rows;
  const size_t pairs = static_cast<size_t>(kv.batch) * kv.num_kv_heads;
  const size_t G = kv.num_q_heads / kv.num_kv_heads;
  char* p = static_cast<char*>(workspace);
  size_t off = 0;
  auto take = [&](size_t bytes) { char* r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
  DecWs w;
  w.part_m = reinterpret_cast<float*>(take(pairs * nsplit * 16 * 4));
  w.part_l = reinterpret_cast<float*>(take(pairs * nsplit * 16 * 4));
  w.part_o = reinterpret_cast<float*>(take(pairs * nsplit * G * kHeadDim * 4));
  if (total) *total = off;
  return w;
}

template <bool FP8>
hipError_t run(const DecodeArgs& a, hipStream_t st) {
  const KvView& kv = a.kv;
  const int split_rows = pick_split_rows(kv, a.max_budget);
  const int nsplit = (a.max_budget + split_rows - 1) / split_rows;
  const DecWs ws = carve(kv, a.max_budget, a.workspace, nullptr);
  {
    KernelTimer t("decode_span_mfma", st);
    hipLaunchKernelGGL((decode_span_mfma<FP8>), dim3(nsplit, kv.num_kv_heads, kv.batch), dim3(kDecThreads), 0, st, a, ws, split_rows,
                       nsplit);
  }
  if (nsplit > 1) {
    KernelTimer t("decode_merge_mfma", st);
    hipLaunchKernelGGL(decode_merge_mfma, dim3(kv.num_kv_heads, kv.batch), dim3(kMergeThreads), 0, st, a, ws, split_rows, nsplit);
  }
  return hipGetLastError();
}

}  // namespace

bool decode_mfma_supported(const DecodeArgs& a) {
  const KvView& kv = a.kv;
  if (a.q_dtype != PILLAR_BF16) return false;
  if (a.kv_dtype != PILLAR_BF16 && a.kv_dtype != PILLAR_FP8_E4M3) return false;
  if (kv.head_dim != kHeadDim) return false;
  const int64_t align = a.kv_dtype == PILLAR_BF16 ? 8 : 16;
  if (kv.stride_page % align || kv.stride_head % align || kv.stride_slot % align) return false;
  if ((reinterpret_cast<uintptr_t>(kv.k_pool) | reinterpret_cast<uintptr_t>(kv.v_pool) | reinterpret_cast<uintptr_t>(a.q) |
       reinterpret_cast<uintptr_t>(a.out)) & 15u)
    return false;
  return true;
}

// ---- scratch of the entry point that takes no workspace -------------------------------------
// Split partials of pillar_sparse_decode_static live in this array instead of a caller's buffer.
// Every GPU the library runs on holds its own copy at its own address until the process ends; the
// array's name is only a host-side handle, the address the kernels get comes from the runtime.
constexpr size_t kStaticScratchBytes = size_t{32} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up once per device)
hipError_t static_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace

size_t decode_static_scratch_bytes() { return kStaticScratchBytes; }

hipError_t launch_decode_mfma_static(const DecodeArgs& a, hipStream_t s) {
  DecodeArgs b = a;
  const hipError_t e = static_scratch(&b.workspace);
  if (e != hipSuccess) return e;
  return launch_decode_mfma(b, s);
}

size_t decode_mfma_workspace(const KvView& kv, int max_budget) {
  if (max_budget < 1) return 0;
  if (max_budget <= pick_split_rows(kv, max_budget)) return 0;     // one span per list: the workgroup finishes it
  size_t total = 0;
  carve(kv, max_budget, nullptr, &total);
  return total;
}

hipError_t launch_decode_mfma(const DecodeArgs& a, hipStream_t s) {
  return a.kv_dtype == PILLAR_FP8_E4M3 ? run<true>(a, s) : run<false>(a, s);
}

int decode_span_rows(const KvView& kv, int max_budget) { return pick_split_rows(kv, max_budget); }

DecWs decode_carve(const KvView& kv, int max_budget, void* workspace) { return carve(kv, max_budget, workspace, nullptr); }

hipError_t launch_decode_merge(const DecodeArgs& a, hipStream_t st) {
  const int split_rows = pick_split_rows(a.kv, a.max_budget);
  const int nsplit = (a.max_budget + split_rows - 1) / split_rows;
  if (nsplit <= 1) return hipSuccess;
  const DecWs ws = carve(a.kv, a.max_budget, a.workspace, nullptr);
  KernelTimer t("decode_merge_mfma", st);
  hipLaunchKernelGGL(decode_merge_mfma, dim3(a.kv.num_kv_heads, a.kv.batch), dim3(kMergeThreads), 0, st, a, ws, split_rows, nsplit);
  return hipGetLastError();
}

}  // namespace pillar
