// "Sources": device functors that produce the vector a compressor is applied to.
//   worker side:  q_j     = g_j + e_j                          (Algorithm 4, worker lines)
//   server side:  Delta_j = (sum_i decode(delta_i)_j)/n + e~_j (Algorithm 4, server lines)
// Each kernel that needs the vector a second time (after the partition-wide norm is known)
// calls the same functor again, so both passes see identical bits.
#pragma once
#include "device_utils.hpp"
#include "kernels.hpp"

namespace bpc {

// q = g + e, or g alone without error feedback (Algorithm 3).
template <class T>
struct GradSource {
  const T *grad;
  const float *res;
  static constexpr int kLdsFloats = 1;
  __device__ void begin(const Geo &, uint32_t, float *) const {}
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *) const {
    uint64_t i = g.part_base(p) + j;
    float x = load_grad(grad, i);
    return res ? x + res[i] : x;
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

// Delta from n identity messages (plain averaging, Algorithm 1).
struct IdentityMsgSource {
  WorkerMsgs msgs;
  const float *res;
  uint64_t stride;
  static constexpr int kLdsFloats = 1;
  __device__ void begin(const Geo &, uint32_t, float *) const {}
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *) const {
    float acc = 0.0f;
    for (int i = 0; i < msgs.n; ++i) {
      const float *vals = reinterpret_cast<const float *>(msgs.ptr[i] + (uint64_t)p * stride + kHeaderBytes);
      acc = acc + vals[j];
    }
    float mean = acc * msgs.inv_n;
    return res ? mean + res[g.part_base(p) + j] : mean;
  }
};

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
