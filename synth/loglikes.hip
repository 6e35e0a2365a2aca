// Device-side generator for synthetic log-likelihood rows.
//
// Produces, directly in HBM, exactly the bytes the host generator (wfst_synth.c,
// synth_loglikes_fill) produces: the same integer mixing function and the same
// individually rounded fp32 operations (built with -ffp-contract=off).  Inputs only —
// nothing of the decoder lives here.
#include <hip/hip_runtime.h>
#include <stdint.h>

#define GOLDEN 0x9E3779B97F4A7C15ULL

__host__ __device__ static inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
  z ^= z >> 27; z *= 0x94D049BB133111EBULL;
  z ^= z >> 31;
  return z;
}
__host__ __device__ static inline uint64_t h3(uint64_t seed, uint64_t a, uint64_t b) {
  uint64_t z = mix64(seed + GOLDEN);
  z = mix64(z ^ (a * 0xD1342543DE82EF95ULL + 0x632BE59BD9B4E019ULL));
  return mix64(z + b * GOLDEN);
}
#define TAG_LL 15
#define TAG_TRUE 16

__global__ void __launch_bounds__(256)
k_loglikes(uint64_t seed, int32_t stream, int32_t frame0, int32_t n_frames, int32_t num_pdfs,
           float mu, float sigma, float boost, float *out, int64_t stride) {
  const int32_t f = blockIdx.y;
  const int32_t frame = frame0 + f;
  const uint64_t base = h3(seed, TAG_LL + ((uint64_t)stream << 8), (uint64_t)frame);
  const int32_t tp = (int32_t)(h3(seed ^ 0x5DEECE66DULL, TAG_TRUE + ((uint64_t)stream << 8), (uint64_t)frame)
                               % (uint64_t)num_pdfs);
  for (int32_t p = blockIdx.x * blockDim.x + threadIdx.x; p < num_pdfs; p += gridDim.x * blockDim.x) {
    uint64_t st = base + (uint64_t)(3 * (int64_t)p) * GOLDEN;
    int32_t sum = 0;
    for (int k = 0; k < 3; ++k) {
      uint64_t r = mix64(st + (uint64_t)k * GOLDEN);
      sum += (int32_t)(r & 0xFFFF) + (int32_t)((r >> 16) & 0xFFFF) + (int32_t)((r >> 32) & 0xFFFF) + (int32_t)(r >> 48);
    }
    float z = (float)(2 * sum - 12 * 65535) * (1.0f / 131072.0f);
    float sz = sigma * z;
    float v = mu + sz;
    if (p == tp) v = v + boost;
    out[(int64_t)f * stride + p] = v;
  }
}

extern "C" int synth_loglikes_device(uint64_t seed, int32_t stream, int32_t frame0, int32_t n_frames,
                                     int32_t num_pdfs, float mu, float sigma, float boost,
                                     float *out_device, int64_t stride, void *stream_handle) {
  if (!out_device || n_frames < 0 || num_pdfs < 1 || stride < num_pdfs) return -1;
  if (n_frames == 0) return 0;
  if (n_frames > 65535) return -1;
  int bx = (num_pdfs + 255) / 256; if (bx > 64) bx = 64;
  dim3 grid(bx, n_frames);
  hipLaunchKernelGGL(k_loglikes, grid, dim3(256), 0, (hipStream_t)stream_handle, seed, stream, frame0,
                     n_frames, num_pdfs, mu, sigma, boost, out_device, stride);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}
