// Linear-dithering server, single pass (Algorithm 4 server lines): Delta = mean of the n
// decoded worker messages + e~, p = C(Delta) with fresh stochastic levels, e~' = Delta - p.
// A workgroup reads a tile (8192 elements) of e~ and the matching nibbles of the n messages
// once, keeps Delta in registers, exchanges its part of ||Delta||_2^2 (or max |Delta|) and
// then writes the packed levels and e~'.
//
// A thread owns 8 consecutive elements per row, i.e. one 32-bit word of every worker's nibbles
// per row.  A nibble indexes a 16-entry LDS table per worker that holds the decoded values
// +-(nu_i * level) / s (16 consecutive floats: lanes never conflict on a bank).  With the
// number of workers known at compile time the workgroup has 512 threads and two rows, so that
// all its words of all workers are requested at once and still fit the register file next to
// e~ and the sums; otherwise 256 threads, four rows and a rolled loop over the workers.
#include "dither_common.hpp"
#include "sources.hpp"

namespace bpc {

struct DMsgPtrs {
  const uint8_t *ptr[kMaxWorkers];
  int n;
  float inv_n;
};
inline DMsgPtrs dmsg_ptrs(const WorkerMsgs &m) {
  DMsgPtrs r;
  for (int i = 0; i < kMaxWorkers; ++i) r.ptr[i] = i < m.n ? m.ptr[i] : nullptr;
  r.n = m.n;
  r.inv_n = m.inv_n;
  return r;
}

// Byte B of `x`, and-ed with `mask`, in one instruction (the byte is picked by the operand's
// sub-dword select instead of a shift).
template <int B>
__device__ inline uint32_t byte_and(uint32_t x, uint32_t mask) {
  uint32_t r;
  if (B == 0) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(mask), "v"(x));
  else if (B == 1) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(mask), "v"(x));
  else if (B == 2) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(mask), "v"(x));
  else asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(mask), "v"(x));
  return r;
}

// NW > 0: number of workers known at compile time (unrolled); NW == 0: rolled loop.
// WIDE: linear levels 8..15 (the 5-bit form): one bit plane beside the nibbles, on the way in
// and on the way out; a worker's table then has 32 entries, index = plane bit << 4 | nibble,
// and the workers come in groups of four so that their words and plane bytes fit the registers.
template <bool EF, bool LINF, int NW, bool NAT, bool WIDE = false>
struct DitherServerOp {
  static constexpr int kThreads = NW > 0 ? 512 : kSThreads;
  static constexpr int kDSRows = kSTile / (kThreads * 8);   // 2 or 4
  static constexpr int kPerThread = 8 * kDSRows;
  struct Raw { u32x4 e[2 * kDSRows]; };
  struct Held { float delta[kPerThread]; };
  struct Ctx { float nu, top_over_nu; int mode; const float *mag; };
  static constexpr bool kMax = LINF;
  static constexpr int kRowsPerTile = kDSRows;
  static constexpr int kLutStride = WIDE ? 32 : 16;
  // decode tables (at most 1024 floats), the output magnitudes, and (WIDE) the spread table:
  // for each value of a plane byte, its even bits at bit 6 of the four bytes of one word and its
  // odd bits likewise in a second word, i.e. where the "plane bit << 4" of a table index falls
  // once a word's nibbles sit at bits 2..5 of its bytes
  static constexpr int kSpreadAt = kMaxWorkers * 16 + 16;
  static constexpr int kTableFloats = kSpreadAt + (WIDE ? 512 : 0);
  static_assert(!WIDE || (NW > 0 && NW * 32 <= kMaxWorkers * 16), "tables of the wide form must fit");
  static constexpr size_t kMaxDynLds = 0;
  static constexpr bool kPersistent = false;
  static constexpr int kWavesPerSimd = (NW > 8 && !WIDE) ? 6 : 4;

  Geo g;
  ClusterGeo cg;
  DMsgPtrs msgs;
  float *__restrict__ res;
  uint8_t *__restrict__ payload;
  const float *__restrict__ override;
  uint32_t levels;
  uint64_t seed, stream_id;

  __device__ uint32_t n_items() const { return cg.n_items; }
  __device__ bool needs_total() const { return override == nullptr; }
  __device__ uint32_t part_of(uint32_t item) const { return __builtin_amdgcn_readfirstlane(item / cg.tiles_per_part); }
  __device__ uint32_t tile_off(uint32_t item) const { return __builtin_amdgcn_readfirstlane((item % cg.tiles_per_part) * kSTile); }
  __device__ uint64_t base(uint32_t item) const { return uniform_off(g.part_base(part_of(item)) + tile_off(item)); }
  __device__ void slots_of(uint32_t item, uint32_t *first, uint32_t *count) const {
    uint32_t p = part_of(item);
    *first = p * cg.tiles_per_part;
    *count = (uint32_t)cdiv(g.part_size(p), kSTile);
  }

  // Elements of the tile that lie inside its partition (fewer than a tile's only at the end of
  // a shorter last partition).  e~ is read and written through descriptors of that many
  // elements; the messages are read from their padded records and what they decode to past
  // the partition's end is cleared, so those elements add nothing to the norm and encode as
  // zero bits.
  __device__ uint32_t valid_of(uint32_t item) const {
    const uint32_t left = g.part_size(part_of(item)) - tile_off(item);
    return __builtin_amdgcn_readfirstlane(left < (uint32_t)kSTile ? left : (uint32_t)kSTile);
  }
  __device__ void issue_row(uint32_t item, int u, Raw &raw) const {
    if (!EF) return;
    const TileBuf eb = row_buf(res + base(item), valid_of(item), u * (kThreads * 8), kThreads * 8);
    raw.e[2 * u] = eb.load16(threadIdx.x * 32, 0);
    raw.e[2 * u + 1] = eb.load16(threadIdx.x * 32 + 16, 0);
  }

  // Decode tables of all workers for partition p: lut[i*16 + nibble], or (WIDE)
  // lut[i*32 + (plane bit << 4 | nibble)].
  __device__ void fill_luts(uint32_t p, float *lut) const {
    __syncthreads();
    for (int e = threadIdx.x; e < msgs.n * kLutStride; e += kThreads) {
      const int i = e / kLutStride, code = e % kLutStride;
      const float nu = *reinterpret_cast<const float *>(msgs.ptr[i] + (uint64_t)p * g.stride);
      const uint32_t level = (code & 7) | ((code >> 4) << 3);
      const float mag = level <= levels ? dither_mag(nu, level, levels, NAT) : 0.0f;
      lut[e] = (code & 8) ? -mag : mag;
    }
    __syncthreads();
  }

  // The word of worker i's nibbles that covers this thread's 8 elements of each row.
  __device__ void load_words(uint32_t item, int i, uint32_t out[kDSRows]) const {
    const uint32_t *nibs = reinterpret_cast<const uint32_t *>(
        msgs.ptr[i] + uniform_off((uint64_t)part_of(item) * g.stride + kHeaderBytes + (tile_off(item) >> 1)));
#pragma unroll
    for (int u = 0; u < kDSRows; ++u) out[u] = nibs[u * kThreads + threadIdx.x];
  }

  // The byte of worker i's bit plane that covers this thread's 8 elements of each row.
  __device__ void load_planes(uint32_t item, int i, uint32_t out[kDSRows]) const {
    const uint8_t *plane = msgs.ptr[i] + uniform_off((uint64_t)part_of(item) * g.stride + dither_plane0(g.part_elems) + (tile_off(item) >> 3));
#pragma unroll
    for (int u = 0; u < kDSRows; ++u) out[u] = plane[u * kThreads + threadIdx.x];
  }
  // WIDE, once per workgroup: the spread table.
  template <bool W = WIDE, std::enable_if_t<W, int> = 0>
  __device__ void init(float *table) const {
    if (threadIdx.x < 256) {
      uint32_t even = 0, odd = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        even |= ((threadIdx.x >> (2 * k)) & 1u) << (8 * k + 6);
        odd |= ((threadIdx.x >> (2 * k + 1)) & 1u) << (8 * k + 6);
      }
      u32x2 e;
      e.x = even; e.y = odd;
      reinterpret_cast<u32x2 *>(table + kSpreadAt)[threadIdx.x] = e;
    }
  }
  // WIDE: table offset = (plane bit << 4 | nibble) * 4: the nibbles at bits 2..5 of the bytes of
  // two words as in add_worker, the plane bits or-ed in at bit 6 through the spread table.
  __device__ static void add_worker_wide(const uint32_t word[kDSRows], const uint32_t pb[kDSRows], const float *lut_i,
                                         const float *table, float acc[kPerThread]) {
    const char *lut_b = reinterpret_cast<const char *>(lut_i);
    const u32x2 *spread = reinterpret_cast<const u32x2 *>(table + kSpreadAt);
#pragma unroll
    for (int u = 0; u < kDSRows; ++u) {
      const u32x2 bits = spread[pb[u]];
      const uint32_t even = ((word[u] << 2) & 0x3c3c3c3cu) | bits.x, odd = ((word[u] >> 2) & 0x3c3c3c3cu) | bits.y;
      float v[8];
      v[0] = *reinterpret_cast<const float *>(lut_b + byte_and<0>(even, 0x7cu));
      v[1] = *reinterpret_cast<const float *>(lut_b + byte_and<0>(odd, 0x7cu));
      v[2] = *reinterpret_cast<const float *>(lut_b + byte_and<1>(even, 0x7cu));
      v[3] = *reinterpret_cast<const float *>(lut_b + byte_and<1>(odd, 0x7cu));
      v[4] = *reinterpret_cast<const float *>(lut_b + byte_and<2>(even, 0x7cu));
      v[5] = *reinterpret_cast<const float *>(lut_b + byte_and<2>(odd, 0x7cu));
      v[6] = *reinterpret_cast<const float *>(lut_b + byte_and<3>(even, 0x7cu));
      v[7] = *reinterpret_cast<const float *>(lut_b + byte_and<3>(odd, 0x7cu));
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[8 * u + c] = acc[8 * u + c] + v[c];
    }
  }

  // The byte offsets nibble*4 of a word's eight nibbles into a worker's table: after a shift
  // by two either way, every nibble sits at bits 2..5 of a byte.
  __device__ static void add_worker(const uint32_t word[kDSRows], const float *lut_i, float acc[kPerThread]) {
    const char *lut_b = reinterpret_cast<const char *>(lut_i);
#pragma unroll
    for (int u = 0; u < kDSRows; ++u) {
      const uint32_t even = word[u] << 2, odd = word[u] >> 2;
      float v[8];
      v[0] = *reinterpret_cast<const float *>(lut_b + byte_and<0>(even, 0x3cu));
      v[1] = *reinterpret_cast<const float *>(lut_b + byte_and<0>(odd, 0x3cu));
      v[2] = *reinterpret_cast<const float *>(lut_b + byte_and<1>(even, 0x3cu));
      v[3] = *reinterpret_cast<const float *>(lut_b + byte_and<1>(odd, 0x3cu));
      v[4] = *reinterpret_cast<const float *>(lut_b + byte_and<2>(even, 0x3cu));
      v[5] = *reinterpret_cast<const float *>(lut_b + byte_and<2>(odd, 0x3cu));
      v[6] = *reinterpret_cast<const float *>(lut_b + byte_and<3>(even, 0x3cu));
      v[7] = *reinterpret_cast<const float *>(lut_b + byte_and<3>(odd, 0x3cu));
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[8 * u + c] = acc[8 * u + c] + v[c];
    }
  }

  __device__ double phase1(uint32_t item, Raw &raw, Held &h, float *table) const {
    const uint32_t p = part_of(item);
#pragma unroll
    for (int u = 0; u < kDSRows; ++u) issue_row(item, u, raw);
    float acc[kPerThread];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) acc[k] = 0.0f;
    if (WIDE) {
      // groups of four workers, each requested in one go (more in flight would not fit the
      // registers next to the tile of the older partition)
      constexpr int kGroup = NW > 4 ? 4 : (NW > 0 ? NW : 1);
#pragma unroll 1   // (unrolled, the loads of all groups are hoisted to the front)
      for (int i0 = 0; i0 < NW; i0 += kGroup) {
        uint32_t word[kGroup][kDSRows], pb[kGroup][kDSRows];
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
          load_words(item, i0 + k, word[k]);
          load_planes(item, i0 + k, pb[k]);
        }
        if (i0 == 0) fill_luts(p, table);
#pragma unroll
        for (int k = 0; k < kGroup; ++k) add_worker_wide(word[k], pb[k], table + (i0 + k) * 32, table, acc);
      }
    } else if (NW > 8) {
      // many workers: groups of four, so that a lane stays within 80 registers and three
      // workgroups share a CU (n = 16: 1.31 -> 1.18 ms at 336 M elements; with 4 or 8 workers
      // everything in one go, below, was as fast or faster)
      constexpr int kGroup = 4;
#pragma unroll 1   // (unrolled, the loads of all groups are hoisted to the front)
      for (int i0 = 0; i0 < NW; i0 += kGroup) {
        uint32_t word[kGroup][kDSRows];
#pragma unroll
        for (int k = 0; k < kGroup; ++k) load_words(item, i0 + k, word[k]);
        if (i0 == 0) fill_luts(p, table);
#pragma unroll
        for (int k = 0; k < kGroup; ++k) add_worker(word[k], table + (i0 + k) * 16, acc);
      }
    } else if (NW > 0) {
      // every word of every worker is requested before the tables are built
      uint32_t word[NW > 0 ? NW : 1][kDSRows];
#pragma unroll
      for (int i = 0; i < NW; ++i) load_words(item, i, word[i]);
      fill_luts(p, table);
#pragma unroll
      for (int i = 0; i < NW; ++i) add_worker(word[i], table + i * 16, acc);
    } else {
      fill_luts(p, table);
      for (int i = 0; i < msgs.n; ++i) {
        uint32_t word[kDSRows];
        load_words(item, i, word);
        add_worker(word, table + i * 16, acc);
      }
    }
    const uint32_t valid = valid_of(item);
    double sum = 0.0;
    float mx = 0.0f;
#pragma unroll
    for (int u = 0; u < kDSRows; ++u) {
      const u32x4 ea = raw.e[2 * u], eb = raw.e[2 * u + 1];
      const float e[8] = {__uint_as_float(ea.x), __uint_as_float(ea.y), __uint_as_float(ea.z), __uint_as_float(ea.w),
                          __uint_as_float(eb.x), __uint_as_float(eb.y), __uint_as_float(eb.z), __uint_as_float(eb.w)};
      // elements of this thread's row segment that exist
      const uint32_t seg0 = (u * kThreads + threadIdx.x) * 8;
      const uint32_t have = valid > seg0 ? valid - seg0 : 0u;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float mean = acc[8 * u + c] * msgs.inv_n;
        float d = EF ? mean + e[c] : mean;
        d = (uint32_t)c < have ? d : 0.0f;
        h.delta[8 * u + c] = d;
        if (LINF) mx = fmaxf(mx, fabsf(d));
        else sum = fma((double)d, (double)d, sum);
      }
    }
    return LINF ? (double)mx : sum;
  }
  __device__ void early(uint32_t, Held &) const {}

  __device__ float nu_of(uint32_t p, double total) const {
    if (override) return uniform_load(override + p);
    return LINF ? (float)total : (float)sqrt(total);
  }
  __device__ float scale_of(uint32_t item, double total) const { return nu_of(part_of(item), total); }
  __device__ Ctx begin2(uint32_t item, float nu, float *table) const {
    const uint32_t p = part_of(item);
    if (tile_off(item) == 0 && threadIdx.x == 0) {
      uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride);
      hdr[0] = __float_as_uint(nu);
      hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
    }
    float *mag = table + kMaxWorkers * 16;
    dither_fill_table(nu, levels, NAT, mag);
    const float top_over_nu = dither_top(levels, NAT) / nu;
    return Ctx{nu, top_over_nu, dither_mode(nu, top_over_nu), mag};
  }

  template <int MODE>
  __device__ void row2_body(uint32_t item, int u, Held &h, const Ctx &ctx) const {
    const uint32_t p = part_of(item);
    const Philox rng(seed, stream_id, p + g.part0);
    const uint32_t j0 = tile_off(item) + (u * kThreads + threadIdx.x) * 8;
    float r[8];
    uint32_t hi = 0;
    const uint32_t word = dither_row<MODE, NAT, WIDE>(&h.delta[8 * u], ctx.nu, ctx.top_over_nu, dither_top(levels, NAT), levels, rng, j0, ctx.mag, r, &hi);
    uint32_t *nibs = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
    (nibs + uniform_off((tile_off(item) + u * (kThreads * 8)) >> 3))[threadIdx.x] = word;
    if (WIDE) {
      uint8_t *plane = payload + (uint64_t)p * g.stride + dither_plane0(g.part_elems);
      (plane + uniform_off((tile_off(item) + u * (kThreads * 8)) >> 3))[threadIdx.x] = (uint8_t)hi;
    }
    if (EF) {
      const TileBuf ob = row_buf(res + base(item), valid_of(item), u * (kThreads * 8), kThreads * 8);
      ob.store16(as_u32x4(r[0], r[1], r[2], r[3]), threadIdx.x * 32);
      ob.store16(as_u32x4(r[4], r[5], r[6], r[7]), threadIdx.x * 32 + 16);
    }
  }
  __device__ void row2(uint32_t item, int u, Held &h, const Ctx &ctx) const {
    if (ctx.mode == 1) row2_body<1>(item, u, h, ctx);
    else if (ctx.mode == 2) row2_body<2>(item, u, h, ctx);
    else row2_body<0>(item, u, h, ctx);
  }

};

template <bool EF, bool LINF, bool NAT, bool WIDE>
static hipError_t launch_dither_server(const Geo &g, const ClusterGeo &cg, const bpc_params_t &prm,
                                       const Source &src, uint8_t *payload, double *slots, uint32_t *status, uint32_t *tickets,
                                       hipStream_t stream, bool *used) {
  const DMsgPtrs mp = dmsg_ptrs(src.msgs);
  float *res = src.residual;
#define BPC_DS(NW)                                                                                          \
  return launch_cluster(DitherServerOp<EF, LINF, NW, NAT, WIDE>{g, cg, mp, res, payload, prm.norm_override, prm.levels, \
                                                           prm.seed, prm.stream_id},                        \
                        cg, slots, status, tickets, stream, used)
  switch (mp.n) {
    case 4: BPC_DS(4);
    case 8: BPC_DS(8);
    case 16: BPC_DS(16);
    default:
      if constexpr (WIDE) {
        *used = false;   // the wide form is built for 4, 8 and 16 workers; others take the passes
        return hipSuccess;
      } else {
        BPC_DS(0);
      }
  }
#undef BPC_DS
}

hipError_t dither_server_single_pass(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                                     const Workspace &ws, hipStream_t stream, bool *used) {
  ClusterGeo cg = make_cluster_geo(g, kSTile);
  double *slots = ws.at<double>(ws.lay.slots);
  uint32_t *status = ws.status();
  uint32_t *tickets = ws.tickets();
  const bool linf = prm.norm == BPC_NORM_LINF, nat = prm.kind == BPC_NATDITHER;
  const uint32_t planes = nat ? 0u : dither_planes(prm.levels);
  if (planes > 1) {   // 6 and 7 bits: the multi-pass kernels
    *used = false;
    return hipSuccess;
  }
#define BPC_DSL(EF)                                                                                              \
  do {                                                                                                           \
    if (planes == 1 && linf) return launch_dither_server<EF, true, false, true>(g, cg, prm, src, payload, slots, status, tickets, stream, used);  \
    if (planes == 1) return launch_dither_server<EF, false, false, true>(g, cg, prm, src, payload, slots, status, tickets, stream, used);         \
    if (linf && nat) return launch_dither_server<EF, true, true, false>(g, cg, prm, src, payload, slots, status, tickets, stream, used);   \
    if (linf) return launch_dither_server<EF, true, false, false>(g, cg, prm, src, payload, slots, status, tickets, stream, used);         \
    if (nat) return launch_dither_server<EF, false, true, false>(g, cg, prm, src, payload, slots, status, tickets, stream, used);          \
    return launch_dither_server<EF, false, false, false>(g, cg, prm, src, payload, slots, status, tickets, stream, used);                  \
  } while (0)
  if (src.residual) BPC_DSL(true);
  BPC_DSL(false);
#undef BPC_DSL
}

}  // namespace bpc
