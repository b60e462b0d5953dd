// Linear-dithering worker, single pass (Algorithm 4 worker lines with the stochastic
// multi-level quantiser): a workgroup reads a tile (8192 elements) of g and e once, keeps
// q = g + e in registers, publishes its part of ||q||_2^2 (or max |q|), waits for the
// partition's norm, then draws the levels, writes the packed nibbles and e' = q - decode.
#include "dither_common.hpp"
#include "tile_rows.hpp"

namespace bpc {

// 512 threads (two workgroups a CU) and 16 elements a thread, laid out as in the scaled-sign
// worker: 4 rows of 2048 elements, a thread owns 4 consecutive elements per row -- one Philox
// block -- so every 16-byte access of a wave covers whole cache lines and is marked
// non-temporal.  The four nibbles of a thread and row are two bytes of the record, which every
// lane stores for itself with a plain store (small stores with the non-temporal hint slow the
// whole kernel down).  With one workgroup of 1024 threads a CU the quantiser (2.7 us of vector
// instructions a tile) ran between the workgroup's memory phases; two workgroups run it under
// each other's (336 M f16 elements: 0.712 -> 0.668 ms; with 8 consecutive elements a thread,
// i.e. two 16-byte halves per 32 bytes, the access pattern set the time: 0.69 ms with or
// without the arithmetic).
constexpr int kDWThreads = 512;
constexpr int kDWPer = 16;
constexpr int kDWTile = kDWThreads * kDWPer;
constexpr int kDRows = kDWPer / 4;  // rows of kDWThreads * 4 elements; a thread owns 4 consecutive per row

// WIDE: linear levels beyond 7, whose upper level bits go to the record's bit planes.
template <class G, bool EF, bool LINF, bool NAT, bool WIDE = false>
struct DitherWorkerOp {
  using GV = typename Vec4Of<G>::type;
  struct Raw { GV g[kDRows]; u32x4 e[kDRows]; };
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
    const TileBuf gb(grad + base(item), valid_of(item) * sizeof(G));
    raw.g[u] = tile_load4(gb, threadIdx.x * (4 * sizeof(G)), u * (kDWThreads * 4 * sizeof(G)), grad);
    if (EF) {
      const TileBuf eb(res + base(item), valid_of(item) * 4);
      raw.e[u] = eb.load16<kNonTemporal>(threadIdx.x * 16, u * (kDWThreads * 16));
    }
  }

  __device__ double phase1(uint32_t, Raw &raw, Held &h, float *) const {
    double acc = 0.0;
    float mx = 0.0f;
#pragma unroll
    for (int u = 0; u < kDRows; ++u) {
      float w[4];
      widen4(raw.g[u], w);
      float e[4];
      widen4(raw.e[u], e);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float q = EF ? w[c] + e[c] : w[c];
        h.q[4 * u + c] = q;
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
    const uint32_t t = threadIdx.x;
    const uint32_t j0 = tile_off(item) + (u * kDWThreads + t) * 4;   // within the partition: one Philox block
    uint32_t nibs = 0, hi[3] = {0, 0, 0};
    const uint32_t planes = WIDE ? dither_planes(levels) : 0u;
    float r[4];
    if (MODE == 0) {
#pragma unroll
      for (int c = 0; c < 4; ++c) r[c] = h.q[4 * u + c];
    } else {
      uint32_t rnd[4], code[4];
      rng.block(j0 >> 2, rnd);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        code[c] = dither_quantise<MODE == 2, NAT, WIDE>(h.q[4 * u + c], nu, top_over_nu, top, levels, rnd[c], mag, &r[c]);
        if (WIDE) nibs |= (((code[c] >> 6) << 3) | (code[c] & 7u)) << (4 * c);
        else nibs |= code[c] << (4 * c);
      }
      if (WIDE) {
        // bit 3 + k of the levels goes to plane k; most records have one plane (up to 15 levels)
#pragma unroll
        for (int c = 0; c < 4; ++c) hi[0] |= ((code[c] >> 3) & 1u) << c;
        if (planes > 1) {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            hi[1] |= ((code[c] >> 4) & 1u) << c;
            hi[2] |= ((code[c] >> 5) & 1u) << c;
          }
        }
      }
    }
    // the four nibbles of this lane: two bytes of the record (a plain store: marked non-temporal,
    // stores this small slow the whole kernel down)
    uint8_t *rec = payload + (uint64_t)p * g.stride;
    const TileBuf nb(rec + kHeaderBytes + (tile_off(item) >> 1), kDWTile / 2);
    nb.store2(nibs, t * 2, u * (kDWThreads * 2));
    if (WIDE) {
      // a plane holds one bit per element: eight lanes make a word, which lane 8w stores
      for (uint32_t k = 0; k < planes; ++k) {
        const uint32_t pw = merge8(hi[k]);
        const TileBuf pb(rec + dither_plane0(g.part_elems) + k * dither_plane_bytes(g.part_elems) + (tile_off(item) >> 3), kDWTile / 8);
        if ((t & 7) == 0) pb.store4(pw, (t >> 3) * 4, u * (kDWThreads * 4 / 8));
      }
    }
    if (EF) {
      const TileBuf ob = row_buf(res + base(item), valid_of(item), u * (kDWThreads * 4), kDWThreads * 4);
      ob.store16<kNonTemporal>(as_u32x4(r[0], r[1], r[2], r[3]), t * 16);
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
