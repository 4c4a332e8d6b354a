/*
 * pillar_bench.h -- measurement helpers of libpillar.so.  NOT part of the
 * hot path declared in pillar.h: nothing here is needed to run PillarAttn,
 * and a serving loop should not call any of it.  The benchmark uses them to
 * time the kernels inside one entry point (HIP events recorded on the launch
 * stream, which is what a per-kernel roofline figure needs) and to sweep launch
 * shapes.
 */
#ifndef PILLAR_BENCH_H_
#define PILLAR_BENCH_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing.  pillar_profile_enable(1) creates a fixed pool of HIP
 * events (host objects; 8192 pairs) and makes every later launch of this
 * library be bracketed by one pair on its stream until the pool is used up;
 * the entry points themselves never create anything.  pillar_profile_read
 * waits for the recorded events, returns their pairs to the pool, then fills
 * up to `cap` entries (host memory) with the kernels seen since the last
 * pillar_profile_reset and returns how many there are.  pillar_profile_enable(0)
 * stops the bracketing.  Not thread-safe against running entry points. */
typedef struct {
  char   name[48];
  int64_t launches;
  double total_ms;
} pillar_kernel_time;
void pillar_profile_enable(int on);
void pillar_profile_reset(void);
int  pillar_profile_read(pillar_kernel_time* entries, int cap);

/* What the machine at hand delivers from HBM, for pricing a kernel against a measured ceiling beside the published
 * peak: one launch of a plain read kernel.  Every wavefront of `blocks` 256-thread workgroups reads whole chunks of
 * `chunk_bytes` (a multiple of 16) of `buf` (device, 16-byte aligned, at least n_chunks * chunk_bytes bytes past the
 * largest chunk index) with streaming 16-byte loads: chunk order[i] if `order` (device int32 [n_chunks]) is given,
 * else chunk i.  `sink`: 16 bytes of device memory that are never written in practice.  The caller times it. */
int pillar_bench_read(const void* buf, int64_t n_chunks, int32_t chunk_bytes, const int32_t* order, int32_t blocks,
                      void* sink, void* hip_stream);

/* Launch-shape knobs for sweeps (process-wide, not thread-safe against running
 * calls; they change how the work is divided, and with it the order of floating-point sums, never what is computed).  Known names: "verify_waves"
 * (wavefronts per compute unit that the verification pass is divided among,
 * 1..8) and "decode_rows" (rows of the index list per workgroup of the draft
 * kernel, a multiple of 32 up to 4096; default 512).  A value of 0 restores the default.  Returns
 * PILLAR_EINVAL for an unknown name or a value outside the knob's range. */
int pillar_set_option(const char* name, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* PILLAR_BENCH_H_ */
