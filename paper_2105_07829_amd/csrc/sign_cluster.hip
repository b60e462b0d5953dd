// Scaled-sign worker, single pass (Algorithm 4 worker lines with C(v) = ||v||_1/d sign(v)):
// each workgroup reads a 65536-element tile of g and e once, keeps q = g + e in registers,
// writes the sign bits, publishes its part of ||q||_1, waits for the partition's sum and then
// writes e' = q -+ sigma.  HBM traffic is the algorithmic minimum: g and e read once, e' and
// the bits written once.
#include "cluster.hpp"
#include "kernels.hpp"

namespace bpc {

constexpr int kRows = kCPerThread / 4;  // 16 rows of 4096 elements; a thread owns 4 consecutive per row

__device__ inline void widen4(const float4 &g, float out[4]) { out[0] = g.x; out[1] = g.y; out[2] = g.z; out[3] = g.w; }
__device__ inline void widen4(const uint2 &g, float out[4]) {
  float2 a = __half22float2(*reinterpret_cast<const __half2 *>(&g.x));
  float2 b = __half22float2(*reinterpret_cast<const __half2 *>(&g.y));
  out[0] = a.x; out[1] = a.y; out[2] = b.x; out[3] = b.y;
}
template <class G> struct Vec4Of;
template <> struct Vec4Of<float> { using type = float4; };
template <> struct Vec4Of<__half> { using type = uint2; };

// Sign bits of a row: every lane holds a nibble for its 4 elements; 8 neighbouring lanes are
// merged into one 32-bit word which lane 8w of the wave ends up holding.
__device__ inline uint32_t merge8(uint32_t nib) {
  nib |= __shfl_down(nib, 1, 64) << 4;
  nib |= __shfl_down(nib, 2, 64) << 8;
  nib |= __shfl_down(nib, 4, 64) << 16;
  return nib;
}

template <class G, bool EF>
__global__ __launch_bounds__(kCThreads) void sign_worker_cluster_kernel(
    Geo g, ClusterGeo cg, const G *__restrict__ grad, float *__restrict__ res, uint8_t *__restrict__ payload,
    double *slots, uint32_t *status, const float *__restrict__ override) {
  using GV = typename Vec4Of<G>::type;
  __shared__ double red[kCThreads / 64];
  __shared__ float sigma_sh;
  const uint32_t t = threadIdx.x;
  for (uint32_t item = blockIdx.x; item < cg.n_items; item += gridDim.x) {
    const uint32_t p = item / cg.tiles_per_part;
    const uint32_t tile = item % cg.tiles_per_part;
    const uint32_t d = g.part_size(p);
    const uint32_t tile_off = tile * kCTile;
    const uint32_t n_here = d - tile_off < (uint32_t)kCTile ? d - tile_off : (uint32_t)kCTile;
    const uint64_t base = g.part_base(p) + tile_off;
    const bool full = n_here == (uint32_t)kCTile;
    float q[kCPerThread];
    // ---- phase 1: q = g + e
    if (full) {
      const GV *g4 = reinterpret_cast<const GV *>(grad + base);
      const float4 *e4 = reinterpret_cast<const float4 *>(res + base);
      GV gr[kRows];
#pragma unroll
      for (int u = 0; u < kRows; ++u) gr[u] = g4[u * kCThreads + t];
      if (EF) {
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
          float4 e = e4[u * kCThreads + t];
          q[4 * u] = e.x; q[4 * u + 1] = e.y; q[4 * u + 2] = e.z; q[4 * u + 3] = e.w;
        }
      }
#pragma unroll
      for (int u = 0; u < kRows; ++u) {
        float w[4];
        widen4(gr[u], w);
#pragma unroll
        for (int c = 0; c < 4; ++c) q[4 * u + c] = EF ? w[c] + q[4 * u + c] : w[c];
      }
    }
    // ---- sign bits and the tile's share of ||q||_1
    uint32_t *bits = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
    const uint32_t n_words = (uint32_t)ru4(cdiv(d, 32));
    double acc = 0.0;
    if (full) {
#pragma unroll
      for (int u = 0; u < kRows; ++u) {
        uint32_t nib = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          nib |= (q[4 * u + c] < 0.0f ? 1u : 0u) << c;
          acc += (double)fabsf(q[4 * u + c]);
        }
        uint32_t word = merge8(nib);
        uint32_t widx = (tile_off >> 5) + u * (kCThreads * 4 / 32) + (t >> 3);
        if ((t & 7) == 0) bits[widx] = word;
      }
    } else {
      // ragged last tile of a partition: lane-strided and rolled, nothing kept in registers;
      // phase 2 reads g and e again (one tile per call at most)
      const uint32_t lane = t & 63;
      for (uint32_t c0 = (t >> 6) * 64; c0 < (uint32_t)kCTile; c0 += kCThreads) {
        uint32_t j = c0 + lane;
        uint32_t word = (tile_off + c0) >> 5;
        if (word >= n_words) break;
        float v = 0.0f;
        if (j < n_here) {
          v = load_grad(grad, base + j);
          if (EF) v = v + res[base + j];
        }
        uint64_t mask = __ballot(v < 0.0f);
        if (lane == 0) *reinterpret_cast<uint64_t *>(bits + word) = mask;
        acc += (double)fabsf(v);
      }
    }
    float sigma;
    if (override) {
      sigma = override[p];
    } else {
      double part = cluster_block_reduce<false>(acc, red);
      if (t < 64) {
        const uint32_t first = p * cg.tiles_per_part;
        if (t == 0) slot_publish(slots + item, part);
        double total = slots_collect<false>(slots + first, (uint32_t)cdiv(d, kCTile), status);
        if (t == 0) sigma_sh = (float)(total / (double)d);
      }
      __syncthreads();
      sigma = sigma_sh;
    }
    if (tile == 0 && t == 0) {
      uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride);
      hdr[0] = __float_as_uint(sigma);
      hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
    }
    // ---- phase 2: e' = q - C(q)
    if (EF) {
      if (full) {
        float4 *o4 = reinterpret_cast<float4 *>(res + base);
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
          float4 o;
          o.x = q[4 * u] - (q[4 * u] < 0.0f ? -sigma : sigma);
          o.y = q[4 * u + 1] - (q[4 * u + 1] < 0.0f ? -sigma : sigma);
          o.z = q[4 * u + 2] - (q[4 * u + 2] < 0.0f ? -sigma : sigma);
          o.w = q[4 * u + 3] - (q[4 * u + 3] < 0.0f ? -sigma : sigma);
          o4[u * kCThreads + t] = o;
        }
      } else {
        for (uint32_t j = t; j < n_here; j += kCThreads) {
          float v = load_grad(grad, base + j) + res[base + j];
          res[base + j] = v - (v < 0.0f ? -sigma : sigma);
        }
      }
    }
    __syncthreads();  // red / sigma_sh are reused by the next item
  }
}

__global__ void slots_reset_kernel(double *slots, uint32_t n, uint32_t *status) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) slots[i] = -1.0;
  if (i == 0) *status = 0;
}

// Number of workgroups of `kernel` that can be resident at once on the current device.
static int resident_capacity(const void *kernel) {
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kCThreads, 0) != hipSuccess) return 0;
  return cus * per_cu;
}

template <class G, bool EF>
static hipError_t launch_sign_worker(const Geo &g, const ClusterGeo &cg, const void *grad, float *res,
                                     uint8_t *payload, double *slots, uint32_t *status, const float *override,
                                     hipStream_t stream, bool *used) {
  const void *fn = reinterpret_cast<const void *>(&sign_worker_cluster_kernel<G, EF>);
  static int capacity = 0;  // per kernel instantiation; a property of the device and the code object
  if (capacity == 0) capacity = resident_capacity(fn);
  *used = false;
  if (capacity <= 0) return hipSuccess;
  uint32_t grid = cg.n_items < (uint32_t)capacity ? cg.n_items : (uint32_t)capacity;
  if (cg.tiles_per_part > grid) return hipSuccess;  // a partition must fit in the resident grid
  slots_reset_kernel<<<(uint32_t)cdiv(cg.n_items, 256), 256, 0, stream>>>(slots, cg.n_items, status);
  Geo g_ = g;
  ClusterGeo cg_ = cg;
  const G *grad_ = (const G *)grad;
  void *args[] = {&g_, &cg_, &grad_, &res, &payload, &slots, &status, &override};
  *used = true;
  return hipLaunchCooperativeKernel(fn, dim3(grid), dim3(kCThreads), args, 0, stream);
}

// Returns hipSuccess with *used = false when the single-pass kernel cannot run this shape
// (the caller then takes the multi-pass path).
hipError_t sign_worker_single_pass(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                                   const Workspace &ws, hipStream_t stream, bool *used) {
  ClusterGeo cg = make_cluster_geo(g);
  double *slots = ws.at<double>(ws.lay.slots);
  uint32_t *status = ws.at<uint32_t>(ws.lay.status);
  const bool f16 = src.dtype == BPC_F16;
  if (src.residual) {
    return f16 ? launch_sign_worker<__half, true>(g, cg, src.grad, src.residual, payload, slots, status,
                                                  prm.norm_override, stream, used)
               : launch_sign_worker<float, true>(g, cg, src.grad, src.residual, payload, slots, status,
                                                 prm.norm_override, stream, used);
  }
  return f16 ? launch_sign_worker<__half, false>(g, cg, src.grad, nullptr, payload, slots, status,
                                                 prm.norm_override, stream, used)
             : launch_sign_worker<float, false>(g, cg, src.grad, nullptr, payload, slots, status,
                                                prm.norm_override, stream, used);
}

}  // namespace bpc
