// Pieces of the linear-dithering quantiser shared by the worker and the server kernels.
#pragma once
#include "cluster_launch.hpp"

namespace bpc {

// 0: nu is not positive, everything encodes to level 0; 1: a = |q| * (s/nu); 2: s/nu is not
// finite, a = (|q| * s) / nu per element.
__device__ inline int dither_mode(float nu, float s_over_nu) {
  return !(nu > 0.0f) ? 0 : s_over_nu <= 3.402823466e38f ? 1 : 2;
}

// Level, nibble and residual of one element.  `mag` is the LDS table of the s + 1 decoded
// magnitudes (nu * level) / s, `r` the element's random word.
template <bool SLOW>
__device__ inline uint32_t dither_quantise(float q, float nu, float s_over_nu, uint32_t s, uint32_t r,
                                           const float *mag, float *resid) {
  float a = SLOW ? (fabsf(q) * (float)s) / nu : fabsf(q) * s_over_nu;
  float l = floorf(a);
  float f = a - l;
  float u = (float)(r >> 8) * 0x1p-24f;
  uint32_t level = (uint32_t)l + (u < f ? 1u : 0u);
  level = level > s ? s : level;
  const float m = mag[level];
  *resid = q - (q < 0.0f ? -m : m);
  return (q < 0.0f ? 8u : 0u) | level;
}

// All threads of the workgroup: mag[l] = (nu * l) / s for l = 0..7.
__device__ inline void dither_fill_table(float nu, uint32_t levels, float *mag) {
  __syncthreads();
  if (threadIdx.x < 8) mag[threadIdx.x] = (nu * (float)threadIdx.x) / (float)levels;
  __syncthreads();
}

// One output row of 8 consecutive elements per thread: levels from two Philox blocks, the
// packed word and the 8 residuals.  j0 is the partition-local index of the first element.
template <int MODE>
__device__ inline uint32_t dither_row(const float q[8], float nu, float s_over_nu, uint32_t levels,
                                      const Philox &rng, uint32_t j0, const float *mag, float r[8]) {
  uint32_t word = 0;
  if (MODE == 0) {
#pragma unroll
    for (int c = 0; c < 8; ++c) r[c] = q[c];
    return 0;
  }
  uint32_t rnd[8];
  rng.block(j0 >> 2, rnd);
  rng.block((j0 >> 2) + 1, rnd + 4);
#pragma unroll
  for (int c = 0; c < 8; ++c)
    word |= dither_quantise<MODE == 2>(q[c], nu, s_over_nu, levels, rnd[c], mag, &r[c]) << (4 * c);
  return word;
}

}  // namespace bpc
