// Pieces of the dithering quantisers (linear and natural level maps) shared by the worker and
// the server kernels.
#pragma once
#include "cluster_launch.hpp"

namespace bpc {

// 0: nu is not positive, everything encodes to level 0; 1: a = |q| * (top/nu); 2: top/nu is
// not finite, a = (|q| * top) / nu per element (top = s, natural levels: 2^(s-1)).
__device__ inline int dither_mode(float nu, float s_over_nu) {
  return !(nu > 0.0f) ? 0 : s_over_nu <= 3.402823466e38f ? 1 : 2;
}

// Level, nibble and residual of one element.  `mag` is the LDS table of the s + 1 decoded
// magnitudes, `r` the element's random word, `top` = dither_top(s).
// Linear levels: lower level floor(a), up with probability a - floor(a).  Natural levels sit
// at a = 0, 1, 2, 4, ...: below 1 the lower level is 0 and a itself the probability; from 1
// on the lower level is floor(log2 a) + 1 (the exponent field) and the probability is
// a / 2^floor(log2 a) - 1 (the fraction bits), both exact.
// WIDE (linear levels beyond 7): the result is (sign << 6) | level instead of the nibble.
template <bool SLOW, bool NAT, bool WIDE = false>
__device__ inline uint32_t dither_quantise(float q, float nu, float top_over_nu, float top, uint32_t s, uint32_t r,
                                           const float *mag, float *resid) {
  const float a = SLOW ? (fabsf(q) * top) / nu : fabsf(q) * top_over_nu;
  uint32_t lower;
  float f;
  if (!NAT) {
    const float l = floorf(a);
    f = a - l;
    lower = (uint32_t)l;
  } else {
    const uint32_t bits = __float_as_uint(a);
    const bool below = a < 1.0f;
    lower = below ? 0u : (bits >> 23) - 126u;
    f = below ? a : __uint_as_float((bits & 0x007fffffu) | 0x3f800000u) - 1.0f;
  }
  const float u = (float)(r >> 8) * 0x1p-24f;
  uint32_t level = lower + (u < f ? 1u : 0u);
  level = level > s ? s : level;
  const float m = mag[level];
  *resid = q - (q < 0.0f ? -m : m);
  return (q < 0.0f ? (WIDE ? 64u : 8u) : 0u) | level;
}

// All threads of the workgroup: mag[l] = decoded magnitude of level l for l = 0..s.
__device__ inline void dither_fill_table(float nu, uint32_t levels, bool natural, float *mag) {
  __syncthreads();
  if (threadIdx.x <= levels) mag[threadIdx.x] = dither_mag(nu, threadIdx.x, levels, natural);
  __syncthreads();
}

// One output row of 8 consecutive elements per thread: levels from two Philox blocks, the
// packed word and the 8 residuals.  j0 is the partition-local index of the first element.
// WIDE: levels beyond 7; *plane0 receives bit 3 of the 8 levels (the caller has made sure the
// levels need no further plane).
template <int MODE, bool NAT, bool WIDE = false>
__device__ inline uint32_t dither_row(const float q[8], float nu, float top_over_nu, float top, uint32_t levels,
                                      const Philox &rng, uint32_t j0, const float *mag, float r[8],
                                      uint32_t *plane0 = nullptr) {
  uint32_t word = 0, hi = 0;
  if (MODE == 0) {
#pragma unroll
    for (int c = 0; c < 8; ++c) r[c] = q[c];
    if (WIDE) *plane0 = 0;
    return 0;
  }
  uint32_t rnd[8];
  rng.block(j0 >> 2, rnd);
  rng.block((j0 >> 2) + 1, rnd + 4);
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const uint32_t code = dither_quantise<MODE == 2, NAT, WIDE>(q[c], nu, top_over_nu, top, levels, rnd[c], mag, &r[c]);
    if (WIDE) {
      word |= (((code >> 6) << 3) | (code & 7u)) << (4 * c);
      hi |= ((code >> 3) & 1u) << c;
    } else {
      word |= code << (4 * c);
    }
  }
  if (WIDE) *plane0 = hi;
  return word;
}

}  // namespace bpc
