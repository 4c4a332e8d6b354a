// Plain read kernel for measuring what the machine at hand delivers from HBM (declared in pillar_bench.h; a
// measurement helper, not part of the PillarAttn path): every wavefront reads whole chunks of a buffer with
// 16-byte streaming loads, four in flight per lane, and folds them into a value nobody uses.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pillar.h"
#include "pillar_bench.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void read_chunks(const u32x4* __restrict__ buf, const int32_t* __restrict__ order, int64_t n_chunks,
                                                   int vec_per_chunk, u32x4* sink) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * 4;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int64_t it = wave; it < n_chunks; it += nwaves) {
    const int64_t chunk = order ? order[it] : it;
    const u32x4* p = buf + chunk * vec_per_chunk;
    for (int v = lane; v < vec_per_chunk; v += 256) {
      u32x4 r[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) r[u] = (v + u * 64 < vec_per_chunk) ? __builtin_nontemporal_load(p + v + u * 64) : acc;
#pragma unroll
      for (int u = 0; u < 4; ++u) acc ^= r[u];
    }
  }
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) sink[0] = acc;      // never true for the buffers the benchmark fills
}

}  // namespace

extern "C" int pillar_bench_read(const void* buf, int64_t n_chunks, int32_t chunk_bytes, const int32_t* order, int32_t blocks,
                                 void* sink, void* hip_stream) {
  if (!buf || !sink || n_chunks < 1 || chunk_bytes < 16 || chunk_bytes % 16 || blocks < 1) return PILLAR_EINVAL;
  if (reinterpret_cast<uintptr_t>(buf) & 15u) return PILLAR_EINVAL;
  hipLaunchKernelGGL(read_chunks, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), static_cast<const u32x4*>(buf), order,
                     n_chunks, chunk_bytes / 16, static_cast<u32x4*>(sink));
  return hipGetLastError() == hipSuccess ? PILLAR_OK : PILLAR_EHIP;
}
