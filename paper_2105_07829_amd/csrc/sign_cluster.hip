// Scaled-sign worker, single pass (Algorithm 4 worker lines with C(v) = ||v||_1/d sign(v)):
// each workgroup reads a tile (8192 elements) of g and e once, keeps q = g + e in registers,
// writes the sign bits, publishes its part of ||q||_1, waits for the partition's sum and then
// writes e' = q -+ sigma.  HBM traffic is the algorithmic minimum: g and e read once, e' and
// the bits written once.
#include "tile_rows.hpp"

namespace bpc {

// 512 threads (two workgroups a CU) and 16 elements a thread: q of two tiles (the current one
// and the one awaiting its total) and the loads of a third fit the registers.  (One workgroup of
// 1024 threads a CU took as long at 336 M f16 elements and 2-6 % longer at 110 M and with f32
// gradients.)
constexpr int kSWThreads = 512;
constexpr int kSWPer = 16;
constexpr int kSWTile = kSWThreads * kSWPer;
constexpr int kRows = kSWPer / 4;  // rows of kSWThreads * 4 elements; a thread owns 4 consecutive per row

template <class G, bool EF>
struct SignWorkerOp {
  using GV = typename Vec4Of<G>::type;
  struct Raw { GV g[kRows]; u32x4 e[kRows]; };
  struct Held { float q[kSWPer]; };
  static constexpr bool kMax = false;
  static constexpr int kRowsPerTile = kRows;
  static constexpr int kTableFloats = 1;
  static constexpr size_t kMaxDynLds = 0;
  static constexpr int kThreads = kSWThreads;
  static constexpr bool kPersistent = true;
  struct Ctx { float sigma; };

  Geo g;
  ClusterGeo cg;
  const G *__restrict__ grad;
  float *__restrict__ res;
  uint8_t *__restrict__ payload;
  const float *__restrict__ override;

  __device__ uint32_t n_items() const { return cg.n_items; }
  __device__ bool needs_total() const { return override == nullptr; }
  __device__ uint32_t part_of(uint32_t item) const { return __builtin_amdgcn_readfirstlane(item / cg.tiles_per_part); }
  __device__ uint32_t tile_off(uint32_t item) const { return __builtin_amdgcn_readfirstlane((item % cg.tiles_per_part) * kSWTile); }
  __device__ uint64_t base(uint32_t item) const { return uniform_off(g.part_base(part_of(item)) + tile_off(item)); }
  __device__ void slots_of(uint32_t item, uint32_t *first, uint32_t *count) const {
    uint32_t p = part_of(item);
    *first = p * cg.tiles_per_part;
    *count = (uint32_t)cdiv(g.part_size(p), kSWTile);
  }
  // Elements of the tile that lie inside its partition.  Every tile access goes through a
  // buffer descriptor of exactly that many elements: loads past it return 0 (q = 0 there:
  // nothing for the norm, a clear sign bit) and stores past it are dropped.
  __device__ uint32_t valid_of(uint32_t item) const {
    const uint32_t left = g.part_size(part_of(item)) - tile_off(item);
    return __builtin_amdgcn_readfirstlane(left < (uint32_t)kSWTile ? left : (uint32_t)kSWTile);
  }
  __device__ uint32_t *bits_of(uint32_t p) const {
    return reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
  }

  __device__ void issue_row(uint32_t item, int u, Raw &raw) const {
    const TileBuf gb(grad + base(item), valid_of(item) * sizeof(G));
    raw.g[u] = tile_load4(gb, threadIdx.x * (4 * sizeof(G)), u * (kSWThreads * 4 * sizeof(G)), grad);
    if (EF) {
      const TileBuf eb(res + base(item), valid_of(item) * 4);
      raw.e[u] = eb.load16<kNonTemporal>(threadIdx.x * 16, u * (kSWThreads * 16));
    }
  }

  __device__ double phase1(uint32_t, Raw &raw, Held &h, float *) const {
    double acc = 0.0;
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      float w[4];
      widen4(raw.g[u], w);
      float e[4];
      widen4(raw.e[u], e);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float q = EF ? w[c] + e[c] : w[c];
        h.q[4 * u + c] = q;
        acc += (double)fabsf(q);
      }
    }
    return acc;
  }

  __device__ void early(uint32_t item, Held &h) const {
    const TileBuf bb(bits_of(part_of(item)) + (tile_off(item) >> 5), kSWTile / 8);
    const uint32_t t = threadIdx.x;
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      uint32_t nib = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) nib |= (h.q[4 * u + c] < 0.0f ? 1u : 0u) << c;
      uint32_t word = merge8(nib);
      // (a plain store: marked non-temporal, stores this small -- 32 bytes a wave -- slow the
      // kernel down, 0.587 against 0.575 ms at 336 M elements)
      if ((t & 7) == 0) bb.store4(word, (t >> 3) * 4, u * (kSWThreads * 4 / 8));
    }
  }

  __device__ float sigma_of(uint32_t p, double total) const {
    if (override) return uniform_load(override + p);
    return (float)(total / (double)g.part_size(p));
  }
  __device__ void header(uint32_t item, float sigma) const {
    if (tile_off(item) == 0 && threadIdx.x == 0) {
      uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)part_of(item) * g.stride);
      hdr[0] = __float_as_uint(sigma);
      hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
    }
  }

  __device__ float scale_of(uint32_t item, double total) const { return sigma_of(part_of(item), total); }
  __device__ Ctx begin2(uint32_t item, float sigma, float *) const {
    header(item, sigma);
    return Ctx{sigma};
  }
  __device__ void row2(uint32_t item, int u, Held &h, const Ctx &ctx) const {
    if (!EF) return;
    const float sigma = ctx.sigma;
    const TileBuf ob = row_buf(res + base(item), valid_of(item), u * (kSWThreads * 4), kSWThreads * 4);
    float o[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) o[c] = h.q[4 * u + c] - (h.q[4 * u + c] < 0.0f ? -sigma : sigma);
    ob.store16<kNonTemporal>(as_u32x4(o[0], o[1], o[2], o[3]), threadIdx.x * 16);
  }

};

// Returns hipSuccess with *used = false when the single-pass kernel cannot run this shape
// (the caller then takes the multi-pass path).
hipError_t sign_worker_single_pass(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                                   const Workspace &ws, hipStream_t stream, bool *used) {
  ClusterGeo cg = make_cluster_geo(g, kSWTile);
  double *slots = ws.at<double>(ws.lay.slots);
  uint32_t *status = ws.status();
  uint32_t *tickets = ws.tickets();
  const bool f16 = src.dtype == BPC_F16;
  if (src.residual) {
    if (f16)
      return launch_cluster(SignWorkerOp<__half, true>{g, cg, (const __half *)src.grad, src.residual, payload, prm.norm_override},
                            cg, slots, status, tickets, stream, used);
    return launch_cluster(SignWorkerOp<float, true>{g, cg, (const float *)src.grad, src.residual, payload, prm.norm_override},
                          cg, slots, status, tickets, stream, used);
  }
  if (f16)
    return launch_cluster(SignWorkerOp<__half, false>{g, cg, (const __half *)src.grad, nullptr, payload, prm.norm_override},
                          cg, slots, status, tickets, stream, used);
  return launch_cluster(SignWorkerOp<float, false>{g, cg, (const float *)src.grad, nullptr, payload, prm.norm_override},
                        cg, slots, status, tickets, stream, used);
}

}  // namespace bpc
