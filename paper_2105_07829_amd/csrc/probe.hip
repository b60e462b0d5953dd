// Plain streaming kernels with the memory traffic of the hot-path stages and none of their
// arithmetic: what the memory system gives this access pattern on the device at hand, to be
// read beside the vendor's peak bandwidth.  Same access shape as the worker and update kernels:
// a thread owns 4 consecutive elements per row of a tile, so each 16-byte access of a wave
// covers whole cache lines; all loads of a tile are requested before the first use; data is
// touched once, so loads and stores are non-temporal; the end of the arrays is handled by the
// buffer descriptors (reads past it return 0, writes are dropped).
#include "device_utils.hpp"
#include "geometry.hpp"
#include <hip/hip_runtime.h>

namespace bpc {

constexpr int kPRows = kTile / (kThreads * 4);   // rows of 1024 elements per tile

__device__ inline TileBuf probe_rows(const void *base, uint64_t tile, uint64_t n, uint32_t elem_bytes) {
  const uint64_t first = tile * kTile;
  const uint64_t left = n - first;
  const uint32_t valid = left < (uint64_t)kTile ? (uint32_t)left : (uint32_t)kTile;
  return TileBuf(static_cast<const uint8_t *>(base) + uniform_off(first * elem_bytes), valid * elem_bytes);
}

// c = a (f32): 4 B read + 4 B written per element
__global__ __launch_bounds__(kThreads) void probe_copy_kernel(const float *a, float *c, uint64_t n) {
  const uint64_t tile = blockIdx.x;
  const TileBuf in = probe_rows(a, tile, n, 4);
  u32x4 v[kPRows];
#pragma unroll
  for (int r = 0; r < kPRows; ++r) v[r] = in.load16<kNonTemporal>(threadIdx.x * 16, r * kThreads * 16);
#pragma unroll
  for (int r = 0; r < kPRows; ++r) {
    const uint64_t row0 = tile * kTile + (uint64_t)r * kThreads * 4;
    if (row0 >= n) break;
    const uint64_t left = n - row0;
    const TileBuf out(c + uniform_off(row0), (uint32_t)(left < kThreads * 4 ? left : kThreads * 4) * 4);
    out.store16<kNonTemporal>(v[r], threadIdx.x * 16);
  }
}

// c = widen(a) + b: 2 B (f16) + 4 B (f32) read, 4 B written per element -- the worker's mix of
// gradient, residual in and residual out, without its packed message
__global__ __launch_bounds__(kThreads) void probe_worker_mix_kernel(const __half *a, const float *b, float *c, uint64_t n) {
  const uint64_t tile = blockIdx.x;
  const TileBuf ga = probe_rows(a, tile, n, 2), gb = probe_rows(b, tile, n, 4);
  u32x2 h[kPRows];
  u32x4 e[kPRows];
#pragma unroll
  for (int r = 0; r < kPRows; ++r) {
    h[r] = ga.load8<kNonTemporal>(threadIdx.x * 8, r * kThreads * 8);
    e[r] = gb.load16<kNonTemporal>(threadIdx.x * 16, r * kThreads * 16);
  }
#pragma unroll
  for (int r = 0; r < kPRows; ++r) {
    const uint64_t row0 = tile * kTile + (uint64_t)r * kThreads * 4;
    if (row0 >= n) break;
    const uint64_t left = n - row0;
    const TileBuf out(c + uniform_off(row0), (uint32_t)(left < kThreads * 4 ? left : kThreads * 4) * 4);
    uint32_t lo = h[r].x, hi = h[r].y;
    const float2 p = __half22float2(*reinterpret_cast<const __half2 *>(&lo));
    const float2 q = __half22float2(*reinterpret_cast<const __half2 *>(&hi));
    out.store16<kNonTemporal>(as_u32x4(p.x + __uint_as_float(e[r].x), p.y + __uint_as_float(e[r].y),
                                       q.x + __uint_as_float(e[r].z), q.y + __uint_as_float(e[r].w)),
                              threadIdx.x * 16);
  }
}

// a, b, c each read and written in place (f32): 12 B read + 12 B written per element -- the
// update's mix of moments and parameters
__global__ __launch_bounds__(kThreads) void probe_update_mix_kernel(float *a, float *b, float *c, uint64_t n) {
  const uint64_t tile = blockIdx.x;
  const TileBuf ga = probe_rows(a, tile, n, 4), gb = probe_rows(b, tile, n, 4), gc = probe_rows(c, tile, n, 4);
  u32x4 va[kPRows], vb[kPRows], vc[kPRows];
#pragma unroll
  for (int r = 0; r < kPRows; ++r) {
    va[r] = ga.load16<kNonTemporal>(threadIdx.x * 16, r * kThreads * 16);
    vb[r] = gb.load16<kNonTemporal>(threadIdx.x * 16, r * kThreads * 16);
    vc[r] = gc.load16<kNonTemporal>(threadIdx.x * 16, r * kThreads * 16);
  }
#pragma unroll
  for (int r = 0; r < kPRows; ++r) {
    const uint64_t row0 = tile * kTile + (uint64_t)r * kThreads * 4;
    if (row0 >= n) break;
    const uint64_t left = n - row0;
    const uint32_t bytes = (uint32_t)(left < kThreads * 4 ? left : kThreads * 4) * 4;
    const TileBuf oa(a + uniform_off(row0), bytes), ob(b + uniform_off(row0), bytes), oc(c + uniform_off(row0), bytes);
    // rotate the three streams so that every store depends on a load of another array
    oa.store16<kNonTemporal>(vb[r], threadIdx.x * 16);
    ob.store16<kNonTemporal>(vc[r], threadIdx.x * 16);
    oc.store16<kNonTemporal>(va[r], threadIdx.x * 16);
  }
}

hipError_t stream_probe(int mix, const void *a, const void *b, void *c, uint64_t n, hipStream_t stream) {
  const uint32_t grid = (uint32_t)cdiv(n, kTile);
  if (mix == BPC_PROBE_COPY) probe_copy_kernel<<<grid, kThreads, 0, stream>>>((const float *)a, (float *)c, n);
  else if (mix == BPC_PROBE_WORKER_MIX)
    probe_worker_mix_kernel<<<grid, kThreads, 0, stream>>>((const __half *)a, (const float *)b, (float *)c, n);
  else probe_update_mix_kernel<<<grid, kThreads, 0, stream>>>((float *)const_cast<void *>(a), (float *)const_cast<void *>(b), (float *)c, n);
  return hipGetLastError();
}

}  // namespace bpc
