// Random-k compressor (Section 3.2: k randomly chosen entries of the gradient travel): k indices
// drawn uniformly with replacement from a Philox stream that sender and receiver share, so
// only the k values travel.  The decode multiplies by `value_scale` (d/k makes the operator
// unbiased, Definition 1; 1 gives the plain zero-fill residual of Section 4.2).  Residual
// update as in Algorithm 4: residual = v - decode(message).
//   store  : v_j from the source -> dense buffer (the residual buffer under error feedback)
//   gather : val_t = v[idx_t] -> message
//   fixup  : residual[idx_t] -= scale * val_t   (atomic: an index may repeat)
#include "sources.hpp"

namespace bpc {

__device__ inline uint32_t randk_index(const Philox &rng, uint32_t t, uint32_t d) {
  return (uint32_t)(((uint64_t)rng.word(t) * d) >> 32);
}

template <class SRC>
__global__ __launch_bounds__(kThreads) void randk_store_kernel(Geo g, SRC src, float *buf) {
  __shared__ float lds[SRC::kLdsFloats];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  src.begin(g, p, lds);
  const uint64_t base = g.part_base(p);
#pragma unroll
  for (int c = 0; c < kTile / kThreads; ++c) {
    uint32_t j = tile * kTile + c * kThreads + threadIdx.x;
    if (j < d) buf[base + j] = src.at(g, p, j, lds);
  }
}

__device__ inline void randk_header(const Geo &g, uint32_t p, uint32_t k, uint8_t *payload) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride);
    hdr[0] = k; hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
  }
}

// val_t = buf[idx_t]
__global__ __launch_bounds__(kThreads) void randk_gather_kernel(Geo g, const float *buf, uint8_t *payload,
                                                                uint64_t seed, uint64_t stream_id) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint32_t k = (uint32_t)k_of_device(g, p);
  randk_header(g, p, k, payload);
  float *val = reinterpret_cast<float *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
  const uint64_t base = g.part_base(p);
  const Philox rng(seed, stream_id, p);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads)
    val[t] = buf[base + randk_index(rng, t, d)];
}

// Same, reading the worker's gradient directly (no error feedback: nothing dense is written).
template <class SRC>
__global__ __launch_bounds__(kThreads) void randk_gather_src_kernel(Geo g, SRC src, uint8_t *payload,
                                                                    uint64_t seed, uint64_t stream_id) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint32_t k = (uint32_t)k_of_device(g, p);
  randk_header(g, p, k, payload);
  float *val = reinterpret_cast<float *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
  const Philox rng(seed, stream_id, p);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads)
    val[t] = src.at(g, p, randk_index(rng, t, d), nullptr);
}

__global__ __launch_bounds__(kThreads) void randk_fixup_kernel(Geo g, float *buf, const uint8_t *payload,
                                                               float value_scale, uint64_t seed,
                                                               uint64_t stream_id) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint32_t k = (uint32_t)k_of_device(g, p);
  const float *val = reinterpret_cast<const float *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
  const float scale = value_scale >= 0.0f ? value_scale : (float)d / (float)k;
  const uint64_t base = g.part_base(p);
  const Philox rng(seed, stream_id, p);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads)
    atomicAdd(buf + base + randk_index(rng, t, d), -(scale * val[t]));
}

hipError_t randk_encode(const Geo &g, const bpc_params_t &prm, const bpc_params_t *in_prm, const Source &src,
                        uint8_t *payload, const Workspace &ws, hipStream_t stream) {
  float *dense = ws.at<float>(ws.lay.dense);
  float *buf = src.residual ? src.residual : dense;
  dim3 grid((uint32_t)cdiv(g.k_cap, kThreads), g.P);
  if (src.grad) {
    if (!src.residual) {
      if (src.dtype == BPC_F16)
        randk_gather_src_kernel<<<grid, kThreads, 0, stream>>>(g, GradSource<__half>{(const __half *)src.grad, nullptr},
                                                               payload, prm.seed, prm.stream_id);
      else
        randk_gather_src_kernel<<<grid, kThreads, 0, stream>>>(g, GradSource<float>{(const float *)src.grad, nullptr},
                                                               payload, prm.seed, prm.stream_id);
      return hipGetLastError();
    }
    if (src.dtype == BPC_F16)
      randk_store_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, GradSource<__half>{(const __half *)src.grad, src.residual}, buf);
    else
      randk_store_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, GradSource<float>{(const float *)src.grad, src.residual}, buf);
  } else {
    hipError_t e = fill_zero(dense, sizeof(float) * g.D, stream);
    if (e != hipSuccess) return e;
    // workers that drew from one stream sent values for the same indices
    bool shared = src.msgs.n > 1;
    for (int i = 1; i < src.msgs.n; ++i)
      shared = shared && in_prm[i].seed == in_prm[0].seed && in_prm[i].stream_id == in_prm[0].stream_id &&
               in_prm[i].value_scale == in_prm[0].value_scale;
    if (shared) {
      e = scatter_add_randk_shared(g, in_prm[0], src.msgs, dense, stream);
      if (e != hipSuccess) return e;
    } else {
      for (int i = 0; i < src.msgs.n; ++i) {
        e = scatter_add_sparse(g, in_prm[i], src.msgs.ptr[i], dense, stream);
        if (e != hipSuccess) return e;
      }
    }
    randk_store_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, DenseSumSource{dense, src.residual, src.msgs.inv_n}, buf);
  }
  randk_gather_kernel<<<grid, kThreads, 0, stream>>>(g, buf, payload, prm.seed, prm.stream_id);
  if (src.residual)
    randk_fixup_kernel<<<grid, kThreads, 0, stream>>>(g, buf, payload, prm.value_scale, prm.seed, prm.stream_id);
  return hipGetLastError();
}

}  // namespace bpc
