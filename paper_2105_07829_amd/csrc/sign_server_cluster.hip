// Scaled-sign server, single pass (Algorithm 4 server lines): Delta = mean of the n decoded
// worker messages + e~, p = C(Delta), e~' = Delta - p.  A workgroup reads an 8192-element
// tile of e~ and the matching bits of the n messages once, keeps Delta in registers, writes
// the sign bits of Delta, exchanges its part of ||Delta||_1 and writes e~' = Delta -+ sigma.
//
// A thread owns 8 elements per row (2 rows of 4096 elements per tile, 512 threads): a wave takes
// 512 consecutive elements of a row, lane l the four elements from 4 l and the four from
// 256 + 4 l, so that every 16-byte access of a wave to e~ covers whole cache lines and is marked
// non-temporal.  Its share of a worker's sign bits is then two nibbles 32 bytes apart; when the
// tile's bits are staged in LDS they are interleaved (4 instructions per 8 bytes) so that the two
// nibbles of a thread are one byte again.  With the number of workers fixed at compile time that
// byte indexes a 256-row LDS table whose row holds, as eight halves, -1 where the byte's bit is
// set and +1 where it is clear, and the sum advances by one mixed-precision fused multiply-add
// per element and worker: fma(+-1, sigma_i, acc) rounds once, and the product is exact, so it
// is acc +- sigma_i to the bit, the f32 addition in worker order (for any sigma_i, negative ones
// included).  The n scales of a partition sit in the first n lanes of every wave and reach the
// multiply-add through a scalar register.  Three workgroups a CU overlap each other's loads,
// sums and stores.
#include "tile_rows.hpp"
#include "sources.hpp"

namespace bpc {

constexpr int kSSThreads = 512;
constexpr int kSSTile = 8192;
constexpr int kSSWaves = kSSThreads / 64;
constexpr int kSRows = kSSTile / (kSSThreads * 8);   // 2
constexpr int kSPerThread = 8 * kSRows;

// Just the message pointers (the random-stream fields of WorkerMsgs are not needed here).
struct MsgPtrs {
  const uint8_t *ptr[kMaxWorkers];
  int n;
  float inv_n;
};
inline MsgPtrs msg_ptrs(const WorkerMsgs &m) {
  MsgPtrs r;
  for (int i = 0; i < kMaxWorkers; ++i) r.ptr[i] = i < m.n ? m.ptr[i] : nullptr;
  r.n = m.n;
  r.inv_n = m.inv_n;
  return r;
}

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// -|sigma| if bit C of `byte` is set, else +|sigma|: the bit is shifted to the sign position
// and the magnitude takes its sign from there (one shift and one bit-field insert).
template <int C>
__device__ inline float pick_sign(uint32_t byte, uint32_t mag) {
  return __builtin_copysignf(__uint_as_float(mag), __uint_as_float(byte << (31 - C)));
}

// The n-term sum of +-sigma_i can be had from bit counts when every worker sent the SAME
// scale and that scale is short: with the low six bits of its significand clear (and the scale
// positive, normal and far from overflow) every partial sum m * sigma, |m| <= 64, is exactly
// representable, so the f32 sum in worker order is exact and equals sigma * (n - 2 c), c = the
// number of workers whose bit is set -- bit for bit the same result, without the n additions.
// (Workers get such a scale by agreeing on one, e.g. through bpc_params_t::norm_override.)
__device__ inline bool scale_is_short(uint32_t bits) {
  const uint32_t ex = bits >> 23;   // (a set sign bit makes this 256 or more)
  return (bits & 0x3fu) == 0u && ex >= 1u && ex <= 240u;
}

// NW > 0: the number of workers is known at compile time: the tile's sign bits of all workers are
// requested in one round trip with e~, staged through LDS and summed by table look-up and
// multiply-add (above); NW == 0: any number, a rolled loop over the workers that loads a
// worker's bytes and forms +-sigma_i with a shift and a bit-field insert.
// COUNT: the caller stated that the workers share a scale array; the counting form is compiled in
// and taken for the partitions where it is exact.
template <bool EF, int NW, bool COUNT = false>
struct SignServerOp {
  // loads of a tile: its rows of e~, this wave's share of the workers' bits, a worker's scale
  struct Raw {
    u32x4 e[2 * kSRows];
    u32x4 fetched[NW > 0 ? (NW * (kSSTile / 8192) + kSSWaves - 1) / kSSWaves : 1];
    float my_sigma;
  };
  struct Held { float delta[kSPerThread]; };
  static constexpr bool kMax = false;
  static constexpr int kRowsPerTile = kSRows;
  // LDS: the n scales (NW == 0), then (NW > 0) the tile's sign bits of every worker, 1 KiB each,
  // then the tables that init() fills once per workgroup
  static constexpr int kBitsPerWorker = kSSTile / 8;   // bytes
  static constexpr int kSpreadWords = COUNT ? 512 : 0;   // byte -> its 8 bits as 8 bytes (the counting form of the sum)
  static constexpr int kUnitWords = NW > 0 ? 256 * 4 : 0;   // byte -> 8 halves: -1 where its bit is set, +1 where clear
  static constexpr int kTableFloats = kMaxWorkers + (NW > 0 ? NW * kBitsPerWorker / 4 : 0) + kSpreadWords + kUnitWords;
  static constexpr int kThreads = kSSThreads;
  static constexpr int kWavesPerSimd = 6;   // 80 registers a lane, three workgroups a CU
  static constexpr bool kPersistent = false;
  static constexpr size_t kMaxDynLds = 0;
  struct Ctx { float sigma; };

  Geo g;
  ClusterGeo cg;
  MsgPtrs msgs;
  float *__restrict__ res;
  uint8_t *__restrict__ payload;
  const float *__restrict__ override;

  __device__ uint32_t n_items() const { return cg.n_items; }
  __device__ bool needs_total() const { return override == nullptr; }
  __device__ uint32_t part_of(uint32_t item) const { return __builtin_amdgcn_readfirstlane(item / cg.tiles_per_part); }
  __device__ uint32_t tile_off(uint32_t item) const { return __builtin_amdgcn_readfirstlane((item % cg.tiles_per_part) * kSSTile); }
  __device__ uint64_t base(uint32_t item) const { return uniform_off(g.part_base(part_of(item)) + tile_off(item)); }
  __device__ void slots_of(uint32_t item, uint32_t *first, uint32_t *count) const {
    uint32_t p = part_of(item);
    *first = p * cg.tiles_per_part;
    *count = (uint32_t)cdiv(g.part_size(p), kSSTile);
  }
  __device__ static uint32_t lane() { return threadIdx.x & 63; }

  // Elements of the tile that lie inside its partition (fewer than a tile's only at the end of
  // a shorter last partition).  e~ is read and written through descriptors of that many
  // elements; the messages are read from their padded records and what they decode to past
  // the partition's end is cleared, so those elements add nothing to the norm and encode as
  // zero bits.
  __device__ uint32_t valid_of(uint32_t item) const {
    const uint32_t left = g.part_size(part_of(item)) - tile_off(item);
    return __builtin_amdgcn_readfirstlane(left < (uint32_t)kSSTile ? left : (uint32_t)kSSTile);
  }
  // Within a row: byte offset in e~ of the thread's first four elements (the other four lie
  // 1024 bytes on), and the elements' numbers.
  __device__ static uint32_t first_byte() { return (threadIdx.x >> 6) * 2048 + (threadIdx.x & 63) * 16; }
  __device__ static uint32_t element_of(int u, int c) {
    return u * (kSSThreads * 8) + (threadIdx.x >> 6) * 512 + (threadIdx.x & 63) * 4 + (c < 4 ? c : 252 + c);
  }
  // A worker's bits of a tile are fetched in pieces of 1 KiB (16 bytes a lane, 8192 elements);
  // piece j = (worker j / kPieces, part j % kPieces) is fetched by wave j % kSSWaves.
  static constexpr int kPieces = kSSTile / 8192;
  static_assert(!COUNT || NW > 0, "the counting form is built for fixed numbers of workers");
  static_assert(kSSTile % 8192 == 0, "tile must be whole pieces");
  // Row u of e~; with row 0 also the workers' scales (lane i of every wave: worker i) and
  // (NW > 0) the tile's sign bits, all in one round trip.
  __device__ void issue_row(uint32_t item, int u, Raw &raw) const {
    if (EF) {
      const TileBuf eb = row_buf(res + base(item), valid_of(item), u * (kSSThreads * 8), kSSThreads * 8);
      raw.e[2 * u] = eb.load16<kNonTemporal>(first_byte(), 0);
      raw.e[2 * u + 1] = eb.load16<kNonTemporal>(first_byte() + 1024, 0);
    }
    if (u != 0) return;
    const uint32_t p = part_of(item);
    raw.my_sigma = 0.0f;
    if ((int)(threadIdx.x & 63) < msgs.n)
      raw.my_sigma = *reinterpret_cast<const float *>(msgs.ptr[threadIdx.x & 63] + (uint64_t)p * g.stride);
    if (NW > 0) {
      const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
      const uint64_t rec_off = uniform_off((uint64_t)p * g.stride + kHeaderBytes + (tile_off(item) >> 3));
#pragma unroll
      for (int j = 0; j < NW * kPieces; ++j)
        if ((uint32_t)(j % kSSWaves) == wave) {
          const TileBuf mb(msgs.ptr[j / kPieces] + rec_off + (j % kPieces) * 1024, 1024);
          raw.fetched[j / kSSWaves] = mb.load16(lane * 16, 0);
        }
    }
  }

  // Once per workgroup: the tables that do not depend on the tile.
  __device__ u32x2 *spread_of(float *sig) const { return reinterpret_cast<u32x2 *>(sig + kMaxWorkers + NW * kBitsPerWorker / 4); }
  __device__ u32x4 *unit_of(float *sig) const { return reinterpret_cast<u32x4 *>(sig + kMaxWorkers + NW * kBitsPerWorker / 4 + kSpreadWords); }
  __device__ void init(float *sig) const {
    if (NW > 0 && threadIdx.x < 256u) {
      const uint32_t b = threadIdx.x;
      if (COUNT) {   // bit c of the byte value -> byte c
        u32x2 sp;
        sp.x = (b & 1u) | ((b & 2u) << 7) | ((b & 4u) << 14) | ((b & 8u) << 21);
        sp.y = ((b >> 4) & 1u) | ((b & 32u) << 3) | ((b & 64u) << 10) | ((b & 128u) << 17);
        spread_of(sig)[b] = sp;
      }
      // bit c of the byte value -> half c: 0x3C00 is 1.0, the sign bit makes it -1.0
      u32x4 *unit = unit_of(sig);
      u32x4 row;
      row.x = 0x3C003C00u | ((b & 1u) << 15) | ((b & 2u) << 30);
      row.y = 0x3C003C00u | ((b & 4u) << 13) | ((b & 8u) << 28);
      row.z = 0x3C003C00u | ((b & 16u) << 11) | ((b & 32u) << 26);
      row.w = 0x3C003C00u | ((b & 64u) << 9) | ((b & 128u) << 24);
      unit[b] = row;
    }
  }

  // The two nibbles of worker i's sign bits that cover this thread's 4 + 4 elements of each row,
  // as one byte.
  __device__ void load_bytes(uint32_t item, int i, uint32_t out[kSRows]) const {
    const uint8_t *bits = msgs.ptr[i] + uniform_off((uint64_t)part_of(item) * g.stride + kHeaderBytes + (tile_off(item) >> 3));
    const uint32_t at = (threadIdx.x >> 6) * 64 + ((threadIdx.x & 63) >> 1), shift = (threadIdx.x & 1u) * 4u;
#pragma unroll
    for (int u = 0; u < kSRows; ++u) {
      const uint32_t a = bits[u * kSSThreads + at], b = bits[u * kSSThreads + at + 32];
      out[u] = ((a >> shift) & 0xfu) | (((b >> shift) & 0xfu) << 4);
    }
  }

  __device__ void add_worker(const uint32_t byte[kSRows], float sigma_i, float acc[kSPerThread]) const {
    // decode is bit ? -sigma : sigma.  With |sigma| and, for a negative sigma, inverted bits
    // this is bit' ? -|sigma| : |sigma| for every finite sigma.
    const uint32_t raw_sigma = __float_as_uint(sigma_i);
    const uint32_t mag = raw_sigma & 0x7fffffffu;
    const uint32_t flip = (raw_sigma >> 31) ? 0xffu : 0u;
#pragma unroll
    for (int u = 0; u < kSRows; ++u) {
      const uint32_t b = byte[u] ^ flip;
      acc[8 * u + 0] = acc[8 * u + 0] + pick_sign<0>(b, mag);
      acc[8 * u + 1] = acc[8 * u + 1] + pick_sign<1>(b, mag);
      acc[8 * u + 2] = acc[8 * u + 2] + pick_sign<2>(b, mag);
      acc[8 * u + 3] = acc[8 * u + 3] + pick_sign<3>(b, mag);
      acc[8 * u + 4] = acc[8 * u + 4] + pick_sign<4>(b, mag);
      acc[8 * u + 5] = acc[8 * u + 5] + pick_sign<5>(b, mag);
      acc[8 * u + 6] = acc[8 * u + 6] + pick_sign<6>(b, mag);
      acc[8 * u + 7] = acc[8 * u + 7] + pick_sign<7>(b, mag);
    }
  }

  __device__ double phase1(uint32_t item, Raw &raw, Held &h, float *sig) const {
#pragma unroll
    for (int u = 0; u < kSRows; ++u) issue_row(item, u, raw);
    float acc[kSPerThread];
#pragma unroll
    for (int k = 0; k < kSPerThread; ++k) acc[k] = 0.0f;
    const float my_sigma = raw.my_sigma;
    if (NW > 0) {
      // the bits are handed out through LDS
      uint8_t *staged = reinterpret_cast<uint8_t *>(sig + kMaxWorkers);
      const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
      const u32x4 *fetched = raw.fetched;
      const u32x2 *spread = spread_of(sig);
      const u32x4 *unit = unit_of(sig);
      // (the staging area is free: every wave has passed the barriers that follow the sums of
      // the tile before)
      // Four lanes hold the 64 bytes of bits of a wave's 512 elements of a row: lanes 0 and 1 of
      // the four the bytes of the lanes' first elements, lanes 2 and 3 those of their second.
      // Nibble k of the first 32 bytes and nibble k of the second become byte k: lanes 0 and 1
      // fetch the words of the lane two up and write 32 bytes each.
#pragma unroll
      for (int j = 0; j < NW * kPieces; ++j)
        if ((uint32_t)(j % kSSWaves) == wave) {
          const u32x4 a = fetched[j / kSSWaves];
          const uint32_t aw[4] = {a.x, a.y, a.z, a.w};
          uint32_t out[8];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const uint32_t b = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)aw[k], 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
            const uint32_t lo = (aw[k] & 0x0F0F0F0Fu) | ((b & 0x0F0F0F0Fu) << 4);
            const uint32_t hi = ((aw[k] >> 4) & 0x0F0F0F0Fu) | (b & 0xF0F0F0F0u);
            out[2 * k] = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
            out[2 * k + 1] = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
          }
          if ((lane & 2) == 0) {
            u32x4 *dst = reinterpret_cast<u32x4 *>(staged + (j / kPieces) * kBitsPerWorker + (j % kPieces) * 1024 + (lane >> 2) * 64 + (lane & 1) * 32);
            u32x4 o0, o1;
            o0.x = out[0]; o0.y = out[1]; o0.z = out[2]; o0.w = out[3];
            o1.x = out[4]; o1.y = out[5]; o1.z = out[6]; o1.w = out[7];
            dst[0] = o0;
            dst[1] = o1;
          }
        }
      __syncthreads();
      // every wave for itself: do all workers carry worker 0's scale, and is it short?
      bool counting = false;
      uint32_t first_bits = 0;
      if (COUNT) {
        first_bits = __builtin_amdgcn_readfirstlane(__float_as_uint(my_sigma));
        const bool same = lane >= (uint32_t)NW || __float_as_uint(my_sigma) == first_bits;
        counting = __all(same) && scale_is_short(first_bits);
      }
      if (COUNT && counting) {
        // counting form: a byte's bits spread to bytes, added up over the workers as integers
        // (at most 16 a byte), then c -> sigma (n - 2 c) as fma(c, -2 sigma, n sigma): every term exact
        uint32_t cnt[kSRows][2];
#pragma unroll
        for (int u = 0; u < kSRows; ++u) cnt[u][0] = cnt[u][1] = 0;
#pragma unroll 4
        for (int i = 0; i < NW; ++i)
#pragma unroll
          for (int u = 0; u < kSRows; ++u) {
            const u32x2 sp = spread[staged[i * kBitsPerWorker + u * kSSThreads + threadIdx.x]];
            cnt[u][0] += sp.x;
            cnt[u][1] += sp.y;
          }
        const float sigma = __uint_as_float(first_bits);
        const float all_clear = (float)NW * sigma, per_bit = -2.0f * sigma;
#pragma unroll
        for (int u = 0; u < kSRows; ++u)
#pragma unroll
          for (int c = 0; c < 8; ++c)
            acc[8 * u + c] = __builtin_fmaf((float)((cnt[u][c / 4] >> (8 * (c % 4))) & 0xffu), per_bit, all_clear);
      } else {
        // four workers per trip: unrolled further, the LDS reads of all workers would be in
        // flight at once and cost more registers than a lane has at this occupancy
#pragma unroll 4
        for (int i = 0; i < NW; ++i) {
          uint32_t byte[kSRows];
#pragma unroll
          for (int u = 0; u < kSRows; ++u) byte[u] = staged[i * kBitsPerWorker + u * kSSThreads + threadIdx.x];
          // acc +- sigma_i as fma(+-1, sigma_i, acc): the compiler folds the widening of the half
          // into the multiply-add (v_fma_mix_f32)
          const float sigma_i = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_sigma), i));
#pragma unroll
          for (int u = 0; u < kSRows; ++u) {
            const u32x4 row = unit[byte[u]];
            const uint32_t w[4] = {row.x, row.y, row.z, row.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const half2_t pm = __builtin_bit_cast(half2_t, w[c]);
              acc[8 * u + 2 * c] = __builtin_fmaf((float)pm.x, sigma_i, acc[8 * u + 2 * c]);
              acc[8 * u + 2 * c + 1] = __builtin_fmaf((float)pm.y, sigma_i, acc[8 * u + 2 * c + 1]);
            }
          }
        }
      }
    } else {
      __syncthreads();
      if ((int)threadIdx.x < msgs.n) sig[threadIdx.x] = my_sigma;
      __syncthreads();
      for (int i = 0; i < msgs.n; ++i) {
        uint32_t byte[kSRows];
        load_bytes(item, i, byte);
        add_worker(byte, sig[i], acc);
      }
    }
    const uint32_t valid = valid_of(item);
    double sum = 0.0;
#pragma unroll
    for (int u = 0; u < kSRows; ++u) {
      const u32x4 ea = raw.e[2 * u], eb = raw.e[2 * u + 1];
      const float e[8] = {__uint_as_float(ea.x), __uint_as_float(ea.y), __uint_as_float(ea.z), __uint_as_float(ea.w),
                          __uint_as_float(eb.x), __uint_as_float(eb.y), __uint_as_float(eb.z), __uint_as_float(eb.w)};
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float mean = acc[8 * u + c] * msgs.inv_n;
        float d = EF ? mean + e[c] : mean;
        d = element_of(u, c) < valid ? d : 0.0f;   // (elements past a shorter last partition)
        h.delta[8 * u + c] = d;
        sum += (double)fabsf(d);
      }
    }
    return sum;
  }

  // Sign bits of Delta: two nibbles per thread and row, each merged with those of the seven lanes
  // above into a word (32 consecutive elements); the words of the second nibbles lie 8 words on.
  __device__ void early(uint32_t item, Held &h) const {
    uint32_t *bits = reinterpret_cast<uint32_t *>(payload + (uint64_t)part_of(item) * g.stride + kHeaderBytes);
#pragma unroll
    for (int u = 0; u < kSRows; ++u) {
      uint32_t na = 0, nb = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        na |= (h.delta[8 * u + c] < 0.0f ? 1u : 0u) << c;
        nb |= (h.delta[8 * u + 4 + c] < 0.0f ? 1u : 0u) << c;
      }
      const uint32_t wa = merge8(na), wb = merge8(nb);
      uint32_t *row_words = bits + uniform_off((tile_off(item) >> 5) + u * (kSSThreads * 8 / 32));
      if ((threadIdx.x & 7) == 0) {
        const uint32_t at = (threadIdx.x >> 6) * 16 + ((threadIdx.x & 63) >> 3);
        row_words[at] = wa;
        row_words[at + 8] = wb;
      }
    }
  }

  __device__ float sigma_of(uint32_t p, double total) const {
    if (override) return uniform_load(override + p);
    return (float)(total / (double)g.part_size(p));
  }
  __device__ void header(uint32_t item, float s) const {
    if (tile_off(item) == 0 && threadIdx.x == 0) {
      uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)part_of(item) * g.stride);
      hdr[0] = __float_as_uint(s);
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
    const TileBuf ob = row_buf(res + base(item), valid_of(item), u * (kSSThreads * 8), kSSThreads * 8);
    float r[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) r[c] = h.delta[8 * u + c] - (h.delta[8 * u + c] < 0.0f ? -sigma : sigma);
    ob.store16<kNonTemporal>(as_u32x4(r[0], r[1], r[2], r[3]), first_byte());
    ob.store16<kNonTemporal>(as_u32x4(r[4], r[5], r[6], r[7]), first_byte() + 1024);
  }

};

template <bool EF>
static hipError_t launch_sign_server(const Geo &g, const ClusterGeo &cg, const bpc_params_t &prm, const Source &src,
                                     uint8_t *payload, double *slots, uint32_t *status, uint32_t *tickets, hipStream_t stream,
                                     bool *used) {
  const MsgPtrs mp = msg_ptrs(src.msgs);
  float *res = src.residual;
  // The counting form is taken at 16 workers, where it is as fast as the sum (110 M elements:
  // 0.241-0.248 ms against 0.248-0.253 ms; both are bound by the memory system there) and does
  // not depend on the order of the workers; it is not instantiated for fewer.
  if (src.msgs.shared_scale && mp.n == 16)
    return launch_cluster(SignServerOp<EF, 16, true>{g, cg, mp, res, payload, prm.norm_override}, cg, slots, status, tickets, stream, used);
  switch (mp.n) {
    case 4: return launch_cluster(SignServerOp<EF, 4>{g, cg, mp, res, payload, prm.norm_override}, cg, slots, status, tickets, stream, used);
    case 8: return launch_cluster(SignServerOp<EF, 8>{g, cg, mp, res, payload, prm.norm_override}, cg, slots, status, tickets, stream, used);
    case 16: return launch_cluster(SignServerOp<EF, 16>{g, cg, mp, res, payload, prm.norm_override}, cg, slots, status, tickets, stream, used);
    default: return launch_cluster(SignServerOp<EF, 0>{g, cg, mp, res, payload, prm.norm_override}, cg, slots, status, tickets, stream, used);
  }
}

hipError_t sign_server_single_pass(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                                   const Workspace &ws, hipStream_t stream, bool *used) {
  ClusterGeo cg = make_cluster_geo(g, kSSTile);
  double *slots = ws.at<double>(ws.lay.slots);
  uint32_t *status = ws.status();
  uint32_t *tickets = ws.tickets();
  if (src.residual) return launch_sign_server<true>(g, cg, prm, src, payload, slots, status, tickets, stream, used);
  return launch_sign_server<false>(g, cg, prm, src, payload, slots, status, tickets, stream, used);
}

}  // namespace bpc
