// Measurement probes for the benchmark harness (no decoder arithmetic): what the device's memory
// system delivers for the two access patterns the decoder is made of, timed with HIP events in
// the same process as the benchmark.
//   probe_copy    a plain streaming copy (16 bytes per thread and step, grid-stride): the
//                 practical ceiling for sequential traffic, to set beside the 8 TB/s peak;
//   probe_gather  12-byte records fetched at pseudo-random indices from a table, `inflight`
//                 independent loads per thread and step, with the benchmark's own launch shape
//                 (lanes x threads): the ceiling for the decoder's random arc gathers when
//                 every thread always has loads in flight and nothing else to do.
#include <hip/hip_runtime.h>
#include <stdint.h>

__global__ void __launch_bounds__(256) k_probe_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

__device__ __forceinline__ uint32_t hash32(uint32_t x) {
  x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
  return x;
}

template <int U>
__global__ void k_probe_gather(const uint32_t *__restrict__ table, uint32_t num_records, int steps, uint32_t *sink) {
  uint32_t acc = 0;
  const uint32_t me = blockIdx.x * blockDim.x + threadIdx.x;
  for (int s = 0; s < steps; ++s) {
    uint32_t v[U][3];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t r = hash32(me * 0x9E3779B9u + (uint32_t)(s * U + u)) % num_records;
      const uint32_t *a = table + 3 * (size_t)r;
      v[u][0] = a[0]; v[u][1] = a[1]; v[u][2] = a[2];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) acc += v[u][0] ^ v[u][1] ^ v[u][2];
  }
  if (acc == 0x12345678u) sink[0] = acc;       // keeps the loads alive
}

static int timed(hipStream_t st, int reps, float *ms, void (*launch)(hipStream_t, void *), void *arg) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -2;
  launch(st, arg);                              // warm-up
  if (hipEventRecord(e0, st) != hipSuccess) return -2;
  for (int i = 0; i < reps; ++i) launch(st, arg);
  if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return -2;
  const int rc = hipEventElapsedTime(ms, e0, e1) == hipSuccess && hipGetLastError() == hipSuccess ? 0 : -2;
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  *ms /= (float)reps;
  return rc;
}

struct CopyArg { const uint4 *src; uint4 *dst; size_t n; };
static void launch_copy(hipStream_t st, void *p) {
  CopyArg *a = (CopyArg *)p;
  hipLaunchKernelGGL(k_probe_copy, dim3(256 * 32), dim3(256), 0, st, a->src, a->dst, a->n);
}
struct GatherArg { const uint32_t *table; uint32_t n; int lanes, threads, steps, inflight; uint32_t *sink; };
static void launch_gather(hipStream_t st, void *p) {
  GatherArg *a = (GatherArg *)p;
  if (a->inflight >= 8) hipLaunchKernelGGL(k_probe_gather<8>, dim3(a->lanes), dim3(a->threads), 0, st, a->table, a->n, a->steps, a->sink);
  else if (a->inflight >= 4) hipLaunchKernelGGL(k_probe_gather<4>, dim3(a->lanes), dim3(a->threads), 0, st, a->table, a->n, a->steps, a->sink);
  else hipLaunchKernelGGL(k_probe_gather<1>, dim3(a->lanes), dim3(a->threads), 0, st, a->table, a->n, a->steps, a->sink);
}

// src, dst: DEVICE buffers of `bytes` bytes (multiple of 16).  *ms = mean duration of one copy.
extern "C" int probe_copy(const void *src, void *dst, size_t bytes, int reps, void *stream, float *ms) {
  if (!src || !dst || !ms || bytes < 16 || (bytes & 15) || reps < 1) return -1;
  CopyArg a{(const uint4 *)src, (uint4 *)dst, bytes / 16};
  return timed((hipStream_t)stream, reps, ms, launch_copy, &a);
}
// table: DEVICE array of num_records 12-byte records; lanes x threads threads each fetch
// steps x inflight records.  sink: DEVICE word.  *ms = mean duration of one launch.
extern "C" int probe_gather(const void *table, uint32_t num_records, int lanes, int threads, int steps, int inflight,
                            void *sink, int reps, void *stream, float *ms) {
  if (!table || !sink || !ms || num_records < 1 || lanes < 1 || threads < 64 || threads > 1024 || steps < 1 || reps < 1) return -1;
  GatherArg a{(const uint32_t *)table, num_records, lanes, threads, steps, inflight, (uint32_t *)sink};
  return timed((hipStream_t)stream, reps, ms, launch_gather, &a);
}
