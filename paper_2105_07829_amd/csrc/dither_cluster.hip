// Linear-dithering worker, single pass (Algorithm 4 worker lines with the stochastic
// multi-level quantiser): a workgroup reads a tile (16384 elements) of g and e once, keeps
// q = g + e in registers, publishes its part of ||q||_2^2 (or max |q|), waits for the
// partition's norm, then draws the levels, writes the packed nibbles and e' = q - decode.
#include "dither_common.hpp"

namespace bpc {

// 1024 threads (one workgroup a CU) and 16 elements a thread, as in the scaled-sign worker.
constexpr int kDWThreads = 1024;
constexpr int kDWPer = 16;
constexpr int kDWTile = kDWThreads * kDWPer;
constexpr int kDRows = kDWPer / 8;  // rows of kDWThreads * 8 elements; a thread owns 8 consecutive per row

struct F32x8 { u32x4 a, b; };
template <class G> struct Vec8Of;
template <> struct Vec8Of<float> { using type = F32x8; };
template <> struct Vec8Of<__half> { using type = u32x4; };

__device__ inline void widen8(const F32x8 &g, float out[8]) {
  out[0] = __uint_as_float(g.a.x); out[1] = __uint_as_float(g.a.y); out[2] = __uint_as_float(g.a.z); out[3] = __uint_as_float(g.a.w);
  out[4] = __uint_as_float(g.b.x); out[5] = __uint_as_float(g.b.y); out[6] = __uint_as_float(g.b.z); out[7] = __uint_as_float(g.b.w);
}
__device__ inline void widen8(const u32x4 &g, float out[8]) {
  const uint32_t w[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float2 f = __half22float2(*reinterpret_cast<const __half2 *>(&w[i]));
    out[2 * i] = f.x;
    out[2 * i + 1] = f.y;
  }
}
// 8 consecutive gradient elements of thread t in row u of a tile window
__device__ inline F32x8 tile_load8(const TileBuf &b, int u, const float *) {
  return {b.load16(threadIdx.x * 32, u * (kDWThreads * 32)), b.load16(threadIdx.x * 32 + 16, u * (kDWThreads * 32))};
}
__device__ inline u32x4 tile_load8(const TileBuf &b, int u, const __half *) {
  return b.load16(threadIdx.x * 16, u * (kDWThreads * 16));
}

// WIDE: linear levels beyond 7, whose upper level bits go to the record's bit planes.
template <class G, bool EF, bool LINF, bool NAT, bool WIDE = false>
struct DitherWorkerOp {
  using GV = typename Vec8Of<G>::type;
  struct Raw { GV g[kDRows]; F32x8 e[kDRows]; };
  struct Held { float q[kDWPer]; };
  static constexpr bool kMax = LINF;
  static constexpr int kRowsPerTile = kDRows;
  static constexpr int kTableFloats = 64;   // decoded magnitudes of the levels 0..s
  static constexpr size_t kMaxDynLds = 0;
  static constexpr int kThreads = kDWThreads;
  static constexpr bool kPersistent = true;
  struct Ctx { float nu, top_over_nu; int mode; const float *mag; };

  Geo g;
  ClusterGeo cg;
  const G *__restrict__ grad;
  float *__restrict__ res;
  uint8_t *__restrict__ payload;
  const float *__restrict__ override;
  uint32_t levels;
  uint64_t seed, stream_id;

  __device__ uint32_t n_items() const { return cg.n_items; }
  __device__ bool needs_total() const { return override == nullptr; }
  __device__ uint32_t part_of(uint32_t item) const { return __builtin_amdgcn_readfirstlane(item / cg.tiles_per_part); }
  __device__ uint32_t tile_off(uint32_t item) const { return __builtin_amdgcn_readfirstlane((item % cg.tiles_per_part) * kDWTile); }
  __device__ uint64_t base(uint32_t item) const { return uniform_off(g.part_base(part_of(item)) + tile_off(item)); }
  __device__ void slots_of(uint32_t item, uint32_t *first, uint32_t *count) const {
    uint32_t p = part_of(item);
    *first = p * cg.tiles_per_part;
    *count = (uint32_t)cdiv(g.part_size(p), kDWTile);
  }

  // Elements of the tile that lie inside its partition.  Every tile access goes through a
  // buffer descriptor of exactly that many elements: loads past it return 0 (q = 0 there:
  // nothing for the norm, level 0) and stores past it are dropped.
  __device__ uint32_t valid_of(uint32_t item) const {
    const uint32_t left = g.part_size(part_of(item)) - tile_off(item);
    return __builtin_amdgcn_readfirstlane(left < (uint32_t)kDWTile ? left : (uint32_t)kDWTile);
  }
  __device__ void issue_row(uint32_t item, int u, Raw &raw) const {
    raw.g[u] = tile_load8(TileBuf(grad + base(item), valid_of(item) * sizeof(G)), u, grad);
    if (EF) raw.e[u] = tile_load8(TileBuf(res + base(item), valid_of(item) * 4), u, (const float *)nullptr);
  }

  __device__ double phase1(uint32_t, Raw &raw, Held &h, float *) const {
    double acc = 0.0;
    float mx = 0.0f;
#pragma unroll
    for (int u = 0; u < kDRows; ++u) {
      float w[8];
      widen8(raw.g[u], w);
      float e[8];
      widen8(raw.e[u], e);
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float q = EF ? w[c] + e[c] : w[c];
        h.q[8 * u + c] = q;
        if (LINF) mx = fmaxf(mx, fabsf(q));
        else acc = fma((double)q, (double)q, acc);
      }
    }
    return LINF ? (double)mx : acc;
  }
  __device__ void early(uint32_t, Held &) const {}

  __device__ float nu_of(uint32_t p, double total) const {
    if (override) return uniform_load(override + p);
    return LINF ? (float)total : (float)sqrt(total);
  }
  __device__ void header(uint32_t item, float nu) const {
    if (tile_off(item) == 0 && threadIdx.x == 0) {
      uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)part_of(item) * g.stride);
      hdr[0] = __float_as_uint(nu);
      hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
    }
  }

  __device__ float scale_of(uint32_t item, double total) const { return nu_of(part_of(item), total); }
  __device__ Ctx begin2(uint32_t item, float nu, float *mag) const {
    header(item, nu);
    dither_fill_table(nu, levels, NAT, mag);
    const float top_over_nu = dither_top(levels, NAT) / nu;
    return Ctx{nu, top_over_nu, dither_mode(nu, top_over_nu), mag};
  }
  __device__ void row2(uint32_t item, int u, Held &h, const Ctx &ctx) const {
    if (ctx.mode == 1) row2_body<1>(item, u, h, ctx);
    else if (ctx.mode == 2) row2_body<2>(item, u, h, ctx);
    else row2_body<0>(item, u, h, ctx);
  }

  template <int MODE>
  __device__ void row2_body(uint32_t item, int u, Held &h, const Ctx &ctx) const {
    const float nu = ctx.nu, top_over_nu = ctx.top_over_nu, top = dither_top(levels, NAT);
    const float *mag = ctx.mag;
    const uint32_t p = part_of(item);
    const Philox rng(seed, stream_id, p + g.part0);
    const uint64_t b = base(item);
    uint32_t *nibs = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
    const uint32_t off = (u * kDWThreads + threadIdx.x) * 8;  // within the tile
    const uint32_t j0 = tile_off(item) + off;                // within the partition
    uint32_t word = 0, hi[3] = {0, 0, 0};
    float r[8];
    if (MODE == 0) {
#pragma unroll
      for (int c = 0; c < 8; ++c) r[c] = h.q[8 * u + c];
    } else {
      uint32_t rnd[8];
      rng.block(j0 >> 2, rnd);
      rng.block((j0 >> 2) + 1, rnd + 4);
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const uint32_t code = dither_quantise<MODE == 2, NAT, WIDE>(h.q[8 * u + c], nu, top_over_nu, top, levels, rnd[c], mag, &r[c]);
        if (WIDE) {
          word |= (((code >> 6) << 3) | (code & 7u)) << (4 * c);
#pragma unroll
          for (int t = 0; t < 3; ++t) hi[t] |= ((code >> (3 + t)) & 1u) << c;
        } else {
          word |= code << (4 * c);
        }
      }
    }
    TileBuf(nibs + (tile_off(item) >> 3), kDWTile / 2).store4(word, threadIdx.x * 4, u * (kDWThreads * 4));
    if (WIDE) {
      // one byte per thread and plane: bit c = bit 3 + t of the level of the thread's element c
      const uint8_t *rec = payload + (uint64_t)p * g.stride;
      const uint32_t planes = dither_planes(levels);
      for (uint32_t t = 0; t < planes; ++t)
        TileBuf(rec + dither_plane0(g.part_elems) + t * dither_plane_bytes(g.part_elems) + (tile_off(item) >> 3), kDWTile / 8)
            .store1(hi[t], threadIdx.x, u * kDWThreads);
    }
    if (EF) {
      const TileBuf ob = row_buf(res + b, valid_of(item), u * (kDWThreads * 8), kDWThreads * 8);
      ob.store16(as_u32x4(r[0], r[1], r[2], r[3]), threadIdx.x * 32);
      ob.store16(as_u32x4(r[4], r[5], r[6], r[7]), threadIdx.x * 32 + 16);
    }
  }

};

template <class G, bool EF>
static hipError_t launch_dither(const Geo &g, const ClusterGeo &cg, const bpc_params_t &prm, const Source &src,
                                uint8_t *payload, double *slots, uint32_t *status, uint32_t *tickets, hipStream_t stream,
                                bool *used) {
#define BPC_DW(LINF, NAT)                                                                                  \
  return launch_cluster(DitherWorkerOp<G, EF, LINF, NAT>{g, cg, (const G *)src.grad, src.residual, payload, \
                                                         prm.norm_override, prm.levels, prm.seed, prm.stream_id}, \
                        cg, slots, status, tickets, stream, used)
  const bool nat = prm.kind == BPC_NATDITHER;
  if (!nat && dither_planes(prm.levels) > 0) {
#define BPC_DWW(LINF)                                                                                             \
  return launch_cluster(DitherWorkerOp<G, EF, LINF, false, true>{g, cg, (const G *)src.grad, src.residual, payload, \
                                                                 prm.norm_override, prm.levels, prm.seed, prm.stream_id}, \
                        cg, slots, status, tickets, stream, used)
    if (prm.norm == BPC_NORM_LINF) BPC_DWW(true);
    BPC_DWW(false);
#undef BPC_DWW
  }
  if (prm.norm == BPC_NORM_LINF) {
    if (nat) BPC_DW(true, true);
    BPC_DW(true, false);
  }
  if (nat) BPC_DW(false, true);
  BPC_DW(false, false);
#undef BPC_DW
}

hipError_t dither_worker_single_pass(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                                     const Workspace &ws, hipStream_t stream, bool *used) {
  ClusterGeo cg = make_cluster_geo(g, kDWTile);
  double *slots = ws.at<double>(ws.lay.slots);
  uint32_t *status = ws.status();
  uint32_t *tickets = ws.tickets();
  const bool f16 = src.dtype == BPC_F16;
  if (src.residual)
    return f16 ? launch_dither<__half, true>(g, cg, prm, src, payload, slots, status, tickets, stream, used)
               : launch_dither<float, true>(g, cg, prm, src, payload, slots, status, tickets, stream, used);
  return f16 ? launch_dither<__half, false>(g, cg, prm, src, payload, slots, status, tickets, stream, used)
             : launch_dither<float, false>(g, cg, prm, src, payload, slots, status, tickets, stream, used);
}

}  // namespace bpc
