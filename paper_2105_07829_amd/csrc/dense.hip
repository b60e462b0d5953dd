// The dense decode of every message kind, and a zero-fill kernel.
#include "sources.hpp"

namespace bpc {

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(uint32_t *ptr, size_t n_words) {
  size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t step = (size_t)gridDim.x * kThreads;
  const size_t n16 = n_words / 4;
  uint4 *p16 = reinterpret_cast<uint4 *>(ptr);
  for (size_t q = i; q < n16; q += step) p16[q] = make_uint4(0, 0, 0, 0);
  for (size_t w = n16 * 4 + i; w < n_words; w += step) ptr[w] = 0;
}

// `ptr` 16-byte aligned, `bytes` a multiple of 4; nothing past ptr + bytes is written.
hipError_t fill_zero(void *ptr, size_t bytes, hipStream_t stream) {
  size_t n_words = bytes / 4;
  if (n_words == 0) return hipSuccess;
  size_t blocks = cdiv(cdiv(n_words, 4), kThreads);
  if (blocks > 4096) blocks = 4096;
  fill_zero_kernel<<<(uint32_t)blocks, kThreads, 0, stream>>>((uint32_t *)ptr, n_words);
  return hipGetLastError();
}

// Decode of the bit-packed kinds and of the identity record.  A thread owns 4 consecutive
// elements per row of 1024, so the 16-byte stores of a wave cover whole cache lines and can be
// non-temporal; the output goes through a descriptor that ends with the partition (stores
// past it are dropped).  The records are padded to a full partition, so reads stay inside.
template <int KIND>
__global__ __launch_bounds__(kThreads) void decode_packed_kernel(Geo g, uint32_t levels, bool natural, const uint8_t *payload, float *out) {
  constexpr int kRow = kThreads * 4, kRows = kTile / kRow;
  const uint32_t p = __builtin_amdgcn_readfirstlane(blockIdx.x / g.tiles_per_part);
  const uint32_t tile = __builtin_amdgcn_readfirstlane(blockIdx.x % g.tiles_per_part);
  const uint32_t d = g.part_size(p);
  const uint8_t *rec = payload + (uint64_t)p * g.stride;
  const float scale = *reinterpret_cast<const float *>(rec);
  const uint8_t *body = rec + kHeaderBytes;
  const uint32_t valid = d - tile * kTile < (uint32_t)kTile ? d - tile * kTile : (uint32_t)kTile;
  float *tile_out = out + g.part_base(p) + (uint64_t)tile * kTile;
  float lut[8];   // dithering: the decoded magnitudes of the levels
  if (KIND == BPC_DITHER) {
#pragma unroll
    for (int l = 0; l < 8; ++l) lut[l] = (uint32_t)l <= levels ? dither_mag(scale, l, levels, natural) : 0.0f;
  }
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    const uint32_t j = tile * kTile + u * kRow + threadIdx.x * 4;   // partition-local, a multiple of 4
    float v[4];
    if (KIND == BPC_SIGN) {
      const uint32_t nib = body[j >> 3] >> (j & 4);
#pragma unroll
      for (int c = 0; c < 4; ++c) v[c] = ((nib >> c) & 1u) ? -scale : scale;
    } else if (KIND == BPC_DITHER) {
      const uint32_t half = reinterpret_cast<const uint16_t *>(body)[j >> 2];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t nib = (half >> (4 * c)) & 15u;
        const uint32_t l = nib & 7u;
        // select from the eight values held in registers (no indexed array)
        float mag = lut[0];
#pragma unroll
        for (int q = 1; q < 8; ++q) mag = l == (uint32_t)q ? lut[q] : mag;
        v[c] = (nib & 8u) ? -mag : mag;
      }
    } else if (KIND == BPC_FP16) {
      const uint2 h = reinterpret_cast<const uint2 *>(body)[j >> 2];
      const float2 a = __half22float2(*reinterpret_cast<const __half2 *>(&h.x));
      const float2 b = __half22float2(*reinterpret_cast<const __half2 *>(&h.y));
      v[0] = a.x; v[1] = a.y; v[2] = b.x; v[3] = b.y;
    } else {
      const float4 q = reinterpret_cast<const float4 *>(body)[j >> 2];
      v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    row_buf(tile_out, valid, u * kRow, kRow).store16<kNonTemporal>(as_u32x4(v[0], v[1], v[2], v[3]), threadIdx.x * 16);
  }
}

// Linear dithering with bit planes (more than 7 levels): 4 consecutive elements a thread as
// above; the level is the nibble's low three bits plus one bit from each plane, the value
// (nu * level) / s as the format defines it.
__global__ __launch_bounds__(kThreads) void decode_dither_wide_kernel(Geo g, uint32_t levels, const uint8_t *payload, float *out) {
  constexpr int kRow = kThreads * 4, kRows = kTile / kRow;
  const uint32_t p = __builtin_amdgcn_readfirstlane(blockIdx.x / g.tiles_per_part);
  const uint32_t tile = __builtin_amdgcn_readfirstlane(blockIdx.x % g.tiles_per_part);
  const uint32_t d = g.part_size(p);
  const uint8_t *rec = payload + (uint64_t)p * g.stride;
  const float nu = *reinterpret_cast<const float *>(rec);
  const uint8_t *body = rec + kHeaderBytes;
  const uint32_t planes = dither_planes(levels);
  const uint8_t *plane0 = rec + dither_plane0(g.part_elems);
  const uint64_t plane_bytes = dither_plane_bytes(g.part_elems);
  const uint32_t valid = d - tile * kTile < (uint32_t)kTile ? d - tile * kTile : (uint32_t)kTile;
  float *tile_out = out + g.part_base(p) + (uint64_t)tile * kTile;
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    const uint32_t j = tile * kTile + u * kRow + threadIdx.x * 4;   // partition-local, a multiple of 4
    const uint32_t half = reinterpret_cast<const uint16_t *>(body)[j >> 2];
    uint32_t hi[4] = {0, 0, 0, 0};
    for (uint32_t t = 0; t < planes; ++t) {
      const uint32_t bits = plane0[t * plane_bytes + (j >> 3)] >> (j & 4);
#pragma unroll
      for (int c = 0; c < 4; ++c) hi[c] |= ((bits >> c) & 1u) << (3 + t);
    }
    float v[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t nib = (half >> (4 * c)) & 15u;
      const float mag = dither_mag(nu, (nib & 7u) | hi[c], levels, false);
      v[c] = (nib & 8u) ? -mag : mag;
    }
    row_buf(tile_out, valid, u * kRow, kRow).store16<kNonTemporal>(as_u32x4(v[0], v[1], v[2], v[3]), threadIdx.x * 16);
  }
}

// Top-k: out[idx_t] = val_t.  `out` was zero-filled before.  HALF: the values are halves.
template <bool HALF>
__global__ __launch_bounds__(kThreads) void decode_topk_kernel(Geo g, const uint8_t *payload, float *out) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint8_t *rec = payload + (uint64_t)p * g.stride;
  uint32_t k = *reinterpret_cast<const uint32_t *>(rec);
  k = k > g.k_cap ? g.k_cap : k;
  const uint32_t *idx = reinterpret_cast<const uint32_t *>(rec + kHeaderBytes);
  const float *val = reinterpret_cast<const float *>(rec + kHeaderBytes + 4 * ru4(g.k_cap));
  const uint64_t base = g.part_base(p);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads) {
    uint32_t j = idx[t];
    if (j < d) out[base + j] = HALF ? __half2float(reinterpret_cast<const __half *>(val)[t]) : val[t];
  }
}

// Random-k: out[idx_t] += scale * val_t with idx_t regenerated from the Philox stream.
// Repeated indices add equal values, so the order of the atomic adds does not matter.
__global__ __launch_bounds__(kThreads) void decode_randk_kernel(Geo g, const uint8_t *payload, float *out,
                                                                float value_scale, uint64_t seed,
                                                                uint64_t stream_id) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint8_t *rec = payload + (uint64_t)p * g.stride;
  uint32_t k = *reinterpret_cast<const uint32_t *>(rec);
  k = k > g.k_cap ? g.k_cap : k;
  const float *val = reinterpret_cast<const float *>(rec + kHeaderBytes);
  const float scale = value_scale >= 0.0f ? value_scale : (float)d / (float)k;
  const uint64_t base = g.part_base(p);
  const Philox rng(seed, stream_id, p + g.part0);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads) {
    uint32_t j = (uint32_t)(((uint64_t)rng.word(t) * d) >> 32);
    atomicAdd(out + base + j, scale * val[t]);
  }
}

// Random-k messages that share one index stream (same seed and stream id at every worker): the
// n values of draw t are summed in worker order first, then added at idx_t once, i.e. one
// random access per draw instead of n.
__global__ __launch_bounds__(kThreads) void decode_randk_shared_kernel(Geo g, WorkerMsgs msgs, float *out,
                                                                       float value_scale, uint64_t seed,
                                                                       uint64_t stream_id) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  uint32_t k = *reinterpret_cast<const uint32_t *>(msgs.ptr[0] + (uint64_t)p * g.stride);
  k = k > g.k_cap ? g.k_cap : k;
  const float scale = value_scale >= 0.0f ? value_scale : (float)d / (float)k;
  const uint64_t base = g.part_base(p);
  const Philox rng(seed, stream_id, p + g.part0);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads) {
    float s = 0.0f;
    for (int i = 0; i < msgs.n; ++i)
      s = s + scale * reinterpret_cast<const float *>(msgs.ptr[i] + (uint64_t)p * g.stride + kHeaderBytes)[t];
    const uint32_t j = (uint32_t)(((uint64_t)rng.word(t) * d) >> 32);
    atomicAdd(out + base + j, s);
  }
}

hipError_t scatter_add_randk_shared(const Geo &g, const bpc_params_t &prm, const WorkerMsgs &msgs, float *out,
                                    hipStream_t stream) {
  dim3 grid((uint32_t)cdiv(g.k_cap, kThreads), g.P);
  decode_randk_shared_kernel<<<grid, kThreads, 0, stream>>>(g, msgs, out, prm.value_scale, prm.seed, prm.stream_id);
  return hipGetLastError();
}

hipError_t scatter_add_sparse(const Geo &g, const bpc_params_t &prm, const uint8_t *payload, float *out,
                              hipStream_t stream) {
  dim3 grid((uint32_t)cdiv(g.k_cap, kThreads), g.P);
  if (prm.kind == BPC_TOPK)
    decode_topk_kernel<false><<<grid, kThreads, 0, stream>>>(g, payload, out);
  else if (prm.kind == BPC_TOPK16)
    decode_topk_kernel<true><<<grid, kThreads, 0, stream>>>(g, payload, out);
  else
    decode_randk_kernel<<<grid, kThreads, 0, stream>>>(g, payload, out, prm.value_scale, prm.seed, prm.stream_id);
  return hipGetLastError();
}

hipError_t decode_dense(const Geo &g, const bpc_params_t &prm, const uint8_t *payload, float *out,
                        hipStream_t stream) {
  if (prm.kind == BPC_TOPK || prm.kind == BPC_TOPK16 || prm.kind == BPC_RANDK) {
    hipError_t e = fill_zero(out, sizeof(float) * g.D, stream);
    if (e != hipSuccess) return e;
    return scatter_add_sparse(g, prm, payload, out, stream);
  }
  const bool natural = prm.kind == BPC_NATDITHER;
  if (prm.kind == BPC_SIGN) decode_packed_kernel<BPC_SIGN><<<g.n_tiles, kThreads, 0, stream>>>(g, prm.levels, false, payload, out);
  else if (prm.kind == BPC_DITHER && dither_planes(prm.levels) > 0)
    decode_dither_wide_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, prm.levels, payload, out);
  else if (prm.kind == BPC_DITHER || natural)
    decode_packed_kernel<BPC_DITHER><<<g.n_tiles, kThreads, 0, stream>>>(g, prm.levels, natural, payload, out);
  else if (prm.kind == BPC_FP16) decode_packed_kernel<BPC_FP16><<<g.n_tiles, kThreads, 0, stream>>>(g, prm.levels, false, payload, out);
  else decode_packed_kernel<BPC_IDENTITY><<<g.n_tiles, kThreads, 0, stream>>>(g, prm.levels, false, payload, out);
  return hipGetLastError();
}

}  // namespace bpc
