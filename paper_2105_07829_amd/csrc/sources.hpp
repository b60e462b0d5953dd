// "Sources": device functors that produce the vector a compressor is applied to.
//   worker side:  q_j     = g_j + e_j                          (Algorithm 4, worker lines)
//   server side:  Delta_j = (sum_i decode(delta_i)_j)/n + e~_j (Algorithm 4, server lines)
// Each kernel that needs the vector a second time (after the partition-wide norm is known)
// calls the same functor again, so both passes see identical bits.
#pragma once
#include "device_utils.hpp"
#include "kernels.hpp"
#include <type_traits>

namespace bpc {

// Eight consecutive f32 / f16 values from a 16-byte aligned position.
__device__ inline void load8_aligned(const float *p, float out[8]) {
  const float4 a = reinterpret_cast<const float4 *>(p)[0], b = reinterpret_cast<const float4 *>(p)[1];
  out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w; out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}
__device__ inline void load8_aligned(const __half *p, float out[8]) {
  const uint4 w = *reinterpret_cast<const uint4 *>(p);
  const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float2 f = __half22float2(*reinterpret_cast<const __half2 *>(&u[i]));
    out[2 * i] = f.x;
    out[2 * i + 1] = f.y;
  }
}

// q = g + e, or g alone without error feedback (Algorithm 3).
template <class T>
struct GradSource {
  using Elem = T;
  const T *grad;
  const float *res;
  static constexpr int kLdsFloats = 1;
  __device__ void begin(const Geo &, uint32_t, float *) const {}
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *) const {
    uint64_t i = g.part_base(p) + j;
    float x = load_grad(grad, i);
    return res ? x + res[i] : x;
  }
  // j0 a multiple of 8: a whole chunk inside the partition comes in with 16-byte loads (the
  // buffers are 16-byte aligned and partitions start at multiples of 1024 elements)
  __device__ void at8(const Geo &g, uint32_t p, uint32_t j0, uint32_t d, const float *, float out[8]) const {
    const uint64_t i0 = g.part_base(p) + j0;
    if (j0 + 8 <= d) {
      float x[8];
      load8_aligned(grad + i0, x);
      if (res) {
        float r[8];
        load8_aligned(res + i0, r);
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = x[e] + r[e];
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = x[e];
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = j0 + e < d ? at(g, p, j0 + e, nullptr) : 0.0f;
    }
  }
};

// Delta from n scaled-sign messages.
struct SignMsgSource {
  WorkerMsgs msgs;
  const float *res;
  uint64_t stride;
  static constexpr int kLdsFloats = kMaxWorkers;
  __device__ void begin(const Geo &, uint32_t p, float *lds) const {
    if ((int)threadIdx.x < msgs.n)
      lds[threadIdx.x] = *reinterpret_cast<const float *>(msgs.ptr[threadIdx.x] + (uint64_t)p * stride);
    __syncthreads();
  }
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *lds) const {
    float acc = 0.0f;
    for (int i = 0; i < msgs.n; ++i) {
      const uint32_t *bits = reinterpret_cast<const uint32_t *>(msgs.ptr[i] + (uint64_t)p * stride + kHeaderBytes);
      uint32_t w = bits[j >> 5];
      float s = lds[i];
      acc = acc + (((w >> (j & 31)) & 1u) ? -s : s);
    }
    float mean = acc * msgs.inv_n;
    return res ? mean + res[g.part_base(p) + j] : mean;
  }
};

// Delta from n dithering messages; a 16-entry table per worker holds the decoded value of
// every nibble, computed with the decode formula (nu * level) / s.
struct DitherMsgSource {
  WorkerMsgs msgs;
  const float *res;
  uint64_t stride;
  uint32_t levels;
  bool natural;
  static constexpr int kLdsFloats = kMaxWorkers * 16;
  __device__ void begin(const Geo &, uint32_t p, float *lds) const {
    for (int e = threadIdx.x; e < msgs.n * 16; e += blockDim.x) {
      int i = e >> 4, nib = e & 15;
      float nu = *reinterpret_cast<const float *>(msgs.ptr[i] + (uint64_t)p * stride);
      float mag = dither_mag(nu, nib & 7, levels, natural);
      lds[e] = (nib & 8) ? -mag : mag;
    }
    __syncthreads();
  }
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *lds) const {
    float acc = 0.0f;
    for (int i = 0; i < msgs.n; ++i) {
      const uint32_t *nibs = reinterpret_cast<const uint32_t *>(msgs.ptr[i] + (uint64_t)p * stride + kHeaderBytes);
      uint32_t nib = (nibs[j >> 3] >> (4 * (j & 7))) & 15u;
      acc = acc + lds[i * 16 + nib];
    }
    float mean = acc * msgs.inv_n;
    return res ? mean + res[g.part_base(p) + j] : mean;
  }
};

// The same for linear dithering with bit planes (more than 7 levels): a table per worker of
// the decoded magnitudes (nu_i * level) / s of its levels 0..s (at most 64).
struct DitherWideMsgSource {
  WorkerMsgs msgs;
  const float *res;
  uint64_t stride;
  uint32_t levels;
  static constexpr int kLdsFloats = kMaxWorkers * 64;
  __device__ void begin(const Geo &, uint32_t p, float *lds) const {
    for (int e = threadIdx.x; e < msgs.n * 64; e += blockDim.x) {
      const int i = e >> 6;
      const uint32_t level = e & 63;
      const float nu = *reinterpret_cast<const float *>(msgs.ptr[i] + (uint64_t)p * stride);
      lds[e] = level <= levels ? dither_mag(nu, level, levels, false) : 0.0f;
    }
    __syncthreads();
  }
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *lds) const {
    const uint32_t planes = dither_planes(levels);
    const uint64_t plane0 = dither_plane0(g.part_elems), plane_bytes = dither_plane_bytes(g.part_elems);
    float acc = 0.0f;
    for (int i = 0; i < msgs.n; ++i) {
      const uint8_t *rec = msgs.ptr[i] + (uint64_t)p * stride;
      const uint32_t nib = (reinterpret_cast<const uint32_t *>(rec + kHeaderBytes)[j >> 3] >> (4 * (j & 7))) & 15u;
      uint32_t level = nib & 7u;
      for (uint32_t t = 0; t < planes; ++t)
        level |= ((reinterpret_cast<const uint32_t *>(rec + plane0 + t * plane_bytes)[j >> 5] >> (j & 31)) & 1u) << (3 + t);
      const float mag = lds[i * 64 + level];
      acc = acc + ((nib & 8u) ? -mag : mag);
    }
    float mean = acc * msgs.inv_n;
    return res ? mean + res[g.part_base(p) + j] : mean;
  }
  // Elements j0 .. j0+7 (j0 a multiple of 8) at once: one nibble word and one byte per plane
  // and worker instead of eight of each.  Same sums in the same order as at().
  __device__ void at8(const Geo &g, uint32_t p, uint32_t j0, uint32_t d, const float *lds, float out[8]) const {
    const uint32_t planes = dither_planes(levels);
    const uint64_t plane0 = dither_plane0(g.part_elems), plane_bytes = dither_plane_bytes(g.part_elems);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    for (int i = 0; i < msgs.n; ++i) {
      const uint8_t *rec = msgs.ptr[i] + (uint64_t)p * stride;
      const uint32_t word = reinterpret_cast<const uint32_t *>(rec + kHeaderBytes)[j0 >> 3];
      uint32_t hi[3] = {0, 0, 0};
      for (uint32_t t = 0; t < planes; ++t) hi[t] = rec[plane0 + t * plane_bytes + (j0 >> 3)];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t nib = (word >> (4 * e)) & 15u;
        const uint32_t level = (nib & 7u) | (((hi[0] >> e) & 1u) << 3) | (((hi[1] >> e) & 1u) << 4) | (((hi[2] >> e) & 1u) << 5);
        const float mag = lds[i * 64 + level];
        acc[e] = acc[e] + ((nib & 8u) ? -mag : mag);
      }
    }
    const uint64_t base = g.part_base(p);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float mean = acc[e] * msgs.inv_n;
      out[e] = j0 + e < d ? (res ? mean + res[base + j0 + e] : mean) : 0.0f;
    }
  }
};

// Eight consecutive elements of a source: its own at8() if it has one, else eight at() calls;
// elements at or past d are 0.
template <class SRC, class = void>
struct has_at8 : std::false_type {};
template <class SRC>
struct has_at8<SRC, std::void_t<decltype(&SRC::at8)>> : std::true_type {};
template <class SRC>
__device__ inline void source_at8(const SRC &src, const Geo &g, uint32_t p, uint32_t j0, uint32_t d, const float *lds,
                                  float out[8]) {
  if constexpr (has_at8<SRC>::value) {
    src.at8(g, p, j0, d, lds, out);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = j0 + e < d ? src.at(g, p, j0 + e, lds) : 0.0f;
  }
}

// Delta for the sparse kinds: the decoded messages were summed into a dense f32 buffer first.
struct DenseSumSource {
  const float *sum;
  const float *res;
  float inv_n;
  static constexpr int kLdsFloats = 1;
  __device__ void begin(const Geo &, uint32_t, float *) const {}
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *) const {
    uint64_t i = g.part_base(p) + j;
    float mean = sum[i] * inv_n;
    return res ? mean + res[i] : mean;
  }
  __device__ void at8(const Geo &g, uint32_t p, uint32_t j0, uint32_t d, const float *, float out[8]) const {
    const uint64_t i0 = g.part_base(p) + j0;
    if (j0 + 8 <= d) {
      float x[8];
      load8_aligned(sum + i0, x);
      float r[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
      if (res) load8_aligned(res + i0, r);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float mean = x[e] * inv_n;
        out[e] = res ? mean + r[e] : mean;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = j0 + e < d ? at(g, p, j0 + e, nullptr) : 0.0f;
    }
  }
};

// Run `fn(source)` with the source that matches `src` (worker f32 / f16 gradient, or the
// server source built by `make_server`).
template <class MakeServer, class Fn>
inline hipError_t with_source(const Source &src, MakeServer make_server, Fn fn) {
  if (src.grad) {
    if (src.dtype == BPC_F16) return fn(GradSource<__half>{(const __half *)src.grad, src.residual});
    return fn(GradSource<float>{(const float *)src.grad, src.residual});
  }
  return fn(make_server());
}

}  // namespace bpc
