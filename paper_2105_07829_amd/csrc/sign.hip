// Scaled-sign compressor, C(v) = ||v||_1/d * sign(v) (Section 3.3, example after Definition 2),
// with the residual update of Algorithm 4.  Three launches per call:
//   reduce : v_j from the source, sign bits by wave ballot, per-tile partial of sum |v_j| in f64
//   finish : sigma = (f32)(sum / d) per partition, written to the record header
//   apply  : residual_j = v_j - (bit ? -sigma : sigma)
#include "cluster.hpp"
#include "sources.hpp"

namespace bpc {

// One workgroup = one tile of kTile elements of one partition.  Lane l of a wave owns element
// 64*c + l of chunk c, so a ballot over (v < 0) is two consecutive words of the message.
template <class SRC>
__global__ __launch_bounds__(kThreads) void sign_reduce_kernel(Geo g, SRC src, uint8_t *payload,
                                                               double *partials, int want_sum) {
  __shared__ float lds[SRC::kLdsFloats];
  __shared__ double red[kThreads / 64];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  src.begin(g, p, lds);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  constexpr int kChunks = kTile / kThreads;  // 64-element chunks per wave
  const uint32_t wave_base = tile * kTile + wave * (kChunks * 64);
  uint64_t my_mask = 0;
  double acc = 0.0;
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    uint32_t j = wave_base + c * 64 + lane;
    float v = j < d ? src.at(g, p, j, lds) : 0.0f;
    uint64_t mask = __ballot(v < 0.0f);
    if (lane == c) my_mask = mask;
    acc += (double)fabsf(v);
  }
  uint32_t *bits = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
  const uint32_t n_words = (uint32_t)ru4(cdiv(d, 32));
  if (lane < kChunks) {
    uint32_t word = (wave_base + lane * 64) >> 5;
    if (word < n_words) *reinterpret_cast<uint64_t *>(bits + word) = my_mask;
  }
  if (want_sum) {
    double s = block_sum<kThreads>(acc, red);
    if (threadIdx.x == 0) partials[blockIdx.x] = s;
  }
}

// One wave per partition: sum the tile partials in a fixed order and write the header.
__global__ __launch_bounds__(64) void sign_finish_kernel(Geo g, const double *partials, const float *override,
                                                         uint8_t *payload, uint32_t *status) {
  // (status: NULL when a single-pass kernel of the same call may have set the word)
  if (status && blockIdx.x == 0 && threadIdx.x == 0) status[0] = 0;
  const uint32_t p = blockIdx.x;
  const uint32_t d = g.part_size(p);
  const uint32_t n_tiles = (uint32_t)cdiv(d, kTile);
  float sigma;
  if (override) {
    sigma = override[p];
  } else {
    double s = 0.0;
    for (uint32_t t = threadIdx.x; t < n_tiles; t += 64) s += partials[(uint64_t)p * g.tiles_per_part + t];
    s = wave_sum(s);
    sigma = (float)(s / (double)d);
  }
  if (threadIdx.x == 0) {
    uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride);
    hdr[0] = __float_as_uint(sigma);
    hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
  }
}

template <class SRC>
__global__ __launch_bounds__(kThreads) void sign_apply_kernel(Geo g, SRC src, const uint8_t *payload,
                                                              float *residual) {
  __shared__ float lds[SRC::kLdsFloats];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  src.begin(g, p, lds);
  const float sigma = *reinterpret_cast<const float *>(payload + (uint64_t)p * g.stride);
  const uint64_t base = g.part_base(p);
#pragma unroll
  for (int c = 0; c < kTile / kThreads; ++c) {
    uint32_t j = tile * kTile + c * kThreads + threadIdx.x;
    if (j < d) {
      float v = src.at(g, p, j, lds);
      residual[base + j] = v - (v < 0.0f ? -sigma : sigma);
    }
  }
}

hipError_t sign_encode(const Geo &g_in, const bpc_params_t &prm_in, const Source &src_in, uint8_t *payload,
                       const Workspace &ws, hipStream_t stream) {
  // Full partitions that are a whole number of register tiles go to the single-pass kernel,
  // a ragged last partition (or everything, if the shape does not fit) to the passes below.
  // The single-pass kernels bound a shorter last partition through their buffer descriptors
  // (dword granularity, so an odd number of f16 gradient elements is left to the passes below).
  const bool ragged_ok = !(src_in.grad && src_in.dtype == BPC_F16 && (g_in.D & 1));
  const SplitGeo sp = split_geo(g_in, src_in.grad ? kWTile : kSTile, ragged_ok);
  Geo g = g_in;
  Source src = src_in;
  bpc_params_t prm = prm_in;
  uint32_t *status = ws.status();
  if (sp.single_pass && sp.head.P > 0) {
    bool used = false;
    hipError_t e = src.grad ? sign_worker_single_pass(sp.head, prm, src, payload, ws, stream, &used)
                            : sign_server_single_pass(sp.head, prm, src, payload, ws, stream, &used);
    if (e != hipSuccess) return e;
    if (used) {
      if (sp.tail.D == 0) return hipSuccess;
      advance_to_tail(sp.head.P, g_in, &src, &payload, &prm);
      g = sp.tail;
      status = nullptr;
    }
  }
  double *partials = ws.at<double>(ws.lay.partials);
  auto make_server = [&] { return SignMsgSource{src.msgs, src.residual, g.stride}; };
  return with_source(src, make_server, [&](auto s) -> hipError_t {
    using S = decltype(s);
    sign_reduce_kernel<S><<<g.n_tiles, kThreads, 0, stream>>>(g, s, payload, partials, prm.norm_override == nullptr);
    sign_finish_kernel<<<g.P, 64, 0, stream>>>(g, partials, prm.norm_override, payload, status);
    if (src.residual) sign_apply_kernel<S><<<g.n_tiles, kThreads, 0, stream>>>(g, s, payload, src.residual);
    return hipGetLastError();
  });
}

}  // namespace bpc
