// FP32 -> FP16 conversion as a compressor (Section 4.1: the data type conversion used where
// anything heavier would not pay; Section 5.1 lists the half-precision method): every element of
// q = g + e (worker) or Delta (server) is rounded to the nearest half, ties to even, and the
// residual is what the rounding dropped (Algorithm 4).  No partition-wide quantity is needed,
// so one streaming launch does it: 8 consecutive elements a thread and row, one 16-byte store
// of halves and two of the residual.
#include "sources.hpp"

namespace bpc {

template <class SRC>
__global__ __launch_bounds__(kThreads) void fp16_encode_kernel(Geo g, SRC src, uint8_t *payload, float *residual,
                                                               uint32_t *status) {
  if (blockIdx.x == 0 && threadIdx.x == 0) status[0] = 0;   // no wait in this call: the word reads "none gave up"
  __shared__ float lds[SRC::kLdsFloats];
  constexpr int kRowElems = kThreads * 8, kRows = kTile / kRowElems;
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  src.begin(g, p, lds);
  uint8_t *rec = payload + (uint64_t)p * g.stride;
  if (tile == 0 && threadIdx.x < 4) reinterpret_cast<uint32_t *>(rec)[threadIdx.x] = 0;
  uint4 *chunks = reinterpret_cast<uint4 *>(rec + kHeaderBytes);
  const uint32_t n_chunks = (uint32_t)(ru4(cdiv(d, 2)) / 4);   // the record's half-words, zero past d
  const uint64_t base = g.part_base(p);
#pragma unroll
  for (int row = 0; row < kRows; ++row) {
    const uint32_t j0 = tile * kTile + row * kRowElems + threadIdx.x * 8;
    if ((j0 >> 3) >= n_chunks) continue;
    float v[8];
    source_at8(src, g, p, j0, d, lds, v);
    uint32_t packed[4];
    float r[8];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const __half lo = __float2half_rn(v[e]), hi = __float2half_rn(v[e + 1]);
      packed[e / 2] = (uint32_t)__half_as_ushort(lo) | ((uint32_t)__half_as_ushort(hi) << 16);
      r[e] = v[e] - __half2float(lo);
      r[e + 1] = v[e + 1] - __half2float(hi);
    }
    chunks[j0 >> 3] = make_uint4(packed[0], packed[1], packed[2], packed[3]);
    if (residual) {
      if (j0 + 8 <= d) {
        float4 *out = reinterpret_cast<float4 *>(residual + base + j0);
        out[0] = make_float4(r[0], r[1], r[2], r[3]);
        out[1] = make_float4(r[4], r[5], r[6], r[7]);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (j0 + e < d) residual[base + j0 + e] = r[e];
      }
    }
  }
}

hipError_t fp16_encode(const Geo &g, const bpc_params_t &, const Source &src, uint8_t *payload, const Workspace &ws,
                       hipStream_t stream) {
  auto make_server = [&] { return Fp16MsgSource{src.msgs, src.residual, g.stride}; };
  return with_source(src, make_server, [&](auto s) -> hipError_t {
    fp16_encode_kernel<decltype(s)><<<g.n_tiles, kThreads, 0, stream>>>(g, s, payload, src.residual, ws.status());
    return hipGetLastError();
  });
}

}  // namespace bpc
