// Host+device description of how a flat gradient is cut into partitions and
// how a call's device workspace is carved up.  Record format: include/bpc.h.
#pragma once
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#include "../../include/bpc.h"

#if defined(__HIPCC__)
#define BPC_HD __host__ __device__
#else
#define BPC_HD
#endif

namespace bpc {

constexpr int kMaxWorkers = 64;      // most worker messages one aggregate call accepts
constexpr int kTile = 4096;          // elements one workgroup handles in the streaming kernels
constexpr int kThreads = 256;        // workgroup size of the streaming kernels
constexpr int kSThreads = 256;       // workgroup size of the server-side kernels when the number of workers is not one they are compiled for
constexpr int kWTile = 8192;         // tile of the worker-side single-pass kernels (512 threads x 16 elements)
constexpr int kSTile = 8192;         // tile of the server-side single-pass kernels and of single-pass LANS
constexpr uint32_t kHeaderBytes = 16;
constexpr int kTicketClasses = 16;   // counters the ticketed single-pass kernels draw their tiles from (workgroup w uses counter w % 16)
constexpr int kTicketStride = 4096;  // bytes between two of them, so that they lie in different memory channels
constexpr int kMaxRuns = 64;         // most runs of partitions of one class (compressed / carried as they are) a call accepts
constexpr uint32_t kTopkListCap = 32768;  // entries of a partition's top-k short list
constexpr uint32_t kTopkHistWords = 2048 + 1024 + 1024;  // top-k radix histograms of a partition

BPC_HD inline uint64_t ru4(uint64_t x) { return (x + 3) / 4 * 4; }
BPC_HD inline uint64_t cdiv(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// Everything a kernel needs to find partition p and its record.
// k = max(1, floor(ratio*d)), never above d; exact in f64 for d < 2^31.
BPC_HD inline uint64_t k_rule(double ratio, uint64_t d) {
  if (d == 0) return 0;
  uint64_t k = (uint64_t)floor(ratio * (double)d);
  if (k < 1) k = 1;
  if (k > d) k = d;
  return k;
}

struct Geo {
  uint64_t D;            // elements of the flat gradient
  uint64_t part_elems;   // elements of a full partition
  uint32_t P;            // number of partitions
  uint32_t tiles_per_part;  // kTile-sized tiles of a full partition
  uint32_t n_tiles;      // tiles over all partitions (last partition may have fewer)
  uint32_t k_cap;        // kept elements of a full partition (TOPK/RANDK), else 0
  uint64_t stride;       // bytes between records
  double k_ratio;
  uint32_t part0;        // partition number of partition 0 of this view (non-zero when a call
                         // hands the tail of a gradient to a different set of kernels)

  BPC_HD uint64_t part_base(uint32_t p) const { return (uint64_t)p * part_elems; }
  BPC_HD uint32_t part_size(uint32_t p) const {
    uint64_t rest = D - (uint64_t)p * part_elems;
    return (uint32_t)(rest < part_elems ? rest : part_elems);
  }
};

inline bool params_valid(const bpc_params_t *p) {
  if (!p) return false;
  // (2^28 elements at most: byte offsets inside a partition's record and arrays fit 32 bits everywhere)
  if (p->part_elems == 0 || p->part_elems % 1024 != 0 || p->part_elems > (1ull << 28)) return false;
  switch (p->kind) {
    case BPC_IDENTITY: case BPC_SIGN: case BPC_FP16: return true;
    case BPC_TOPK: case BPC_TOPK16: case BPC_RANDK: return p->k_ratio > 0.0 && p->k_ratio <= 1.0;
    case BPC_DITHER:
      return p->levels >= 1 && p->levels <= 63 && (p->norm == BPC_NORM_L2 || p->norm == BPC_NORM_LINF);
    case BPC_NATDITHER:
      return p->levels >= 1 && p->levels <= 7 && (p->norm == BPC_NORM_L2 || p->norm == BPC_NORM_LINF);
    default: return false;
  }
}

// Bit planes that follow the nibbles of a linear-dithering record: level bits 3, 4, 5.
BPC_HD inline uint32_t dither_planes(uint32_t levels) {
  uint32_t planes = 0;
  while ((levels >> (3 + planes)) != 0) ++planes;
  return planes;
}
// Byte offset of plane 0 in a record, and bytes from one plane to the next.
BPC_HD inline uint64_t dither_plane0(uint64_t part_elems) { return kHeaderBytes + 4 * ru4(cdiv(part_elems, 8)); }
BPC_HD inline uint64_t dither_plane_bytes(uint64_t part_elems) { return 4 * ru4(cdiv(part_elems, 32)); }

inline size_t stride_of(const bpc_params_t *p) {
  uint64_t d = p->part_elems, words = 0;
  switch (p->kind) {
    case BPC_IDENTITY: words = ru4(d); break;
    case BPC_SIGN:     words = ru4(cdiv(d, 32)); break;
    case BPC_DITHER:   words = ru4(cdiv(d, 8)) + dither_planes(p->levels) * ru4(cdiv(d, 32)); break;
    case BPC_NATDITHER: words = ru4(cdiv(d, 8)); break;
    case BPC_TOPK:     words = 2 * ru4(k_rule(p->k_ratio, d)); break;
    case BPC_TOPK16:   words = ru4(k_rule(p->k_ratio, d)) + ru4(cdiv(k_rule(p->k_ratio, d), 2)); break;
    case BPC_RANDK:    words = ru4(k_rule(p->k_ratio, d)); break;
    case BPC_FP16:     words = ru4(cdiv(d, 2)); break;
  }
  return (size_t)(kHeaderBytes + 4 * words);
}

inline Geo make_geo(const bpc_params_t *p, uint64_t D) {
  Geo g;
  g.D = D;
  g.part_elems = p->part_elems;
  g.P = (uint32_t)cdiv(D, p->part_elems);
  g.tiles_per_part = (uint32_t)cdiv(p->part_elems, kTile);
  uint64_t last = D - (uint64_t)(g.P ? g.P - 1 : 0) * p->part_elems;
  g.n_tiles = g.P ? (g.P - 1) * g.tiles_per_part + (uint32_t)cdiv(last, kTile) : 0;
  g.k_cap = (p->kind == BPC_TOPK || p->kind == BPC_TOPK16 || p->kind == BPC_RANDK) ? (uint32_t)k_rule(p->k_ratio, p->part_elems) : 0;
  g.stride = stride_of(p);
  g.k_ratio = p->k_ratio;
  g.part0 = 0;
  return g;
}

// Device workspace of one call.  Offsets in bytes from the workspace base, each
// a multiple of 256.  Regions a kind does not use have size 0.
struct WsLayout {
  size_t status;     // u32[4 * kMaxRuns], at offset 0 whatever the shape: one slot of four words for every run of
                     // partitions a call is split into (one run unless partitions bypass compression).  Word 0 of a
                     // slot is non-zero if a single-pass kernel of that run gave up waiting
  size_t tickets;    // u32 at every kTicketStride bytes, kTicketClasses of them: the ticket counters of the
                     // ticketed single-pass kernels
  size_t partials;   // double[n_tiles]: per-tile partial norms
  size_t dense;      // float[D]: q / Delta / decoded message when no caller buffer can hold it
  size_t hist;       // u32[P*kTopkHistWords]: top-k radix histograms (2048 + 1024 + 1024 bins)
  size_t state;      // u32[P*8 + 8]: top-k selection state; a barrier counter
  size_t guess;      // u32[P]: top-k key from which elements go to a partition's short list
  size_t starts;     // u32[kMaxWorkers * P * (groups of 8192 elements per partition + 1)]: where each group's
                     // entries start in each worker's top-k message (server side)
  size_t samp;       // f32[P * 4096]: sums of the sampled chunks of Delta (top-k, server side)
  size_t cand;       // u32[P * kTopkListCap] indices, then as many value bits: top-k short lists of the partitions
  size_t tilecnt;    // u32[2*n_tiles]: per-tile (greater, equal) counts, then offsets
  size_t slots;      // double[3 * tiles of kSTile]: partition-wide reductions of the single-pass kernels
                     // (one per tile; three for the LANS block norms)
  size_t norms;      // double[3*P]: LANS block norms when blocks are the partitions
  size_t total;
};

inline WsLayout ws_layout(const bpc_params_t *p, uint64_t D) {
  Geo g = make_geo(p, D);
  WsLayout w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
  // kinds whose update reads a dense decode of the message from the workspace
  const bool topk = p->kind == BPC_TOPK || p->kind == BPC_TOPK16;
  bool sparse = topk || p->kind == BPC_RANDK || (p->kind == BPC_DITHER && dither_planes(p->levels) > 0);
  w.status = take(16 * kMaxRuns);
  w.tickets = take((size_t)kTicketClasses * kTicketStride);
  w.partials = take(sizeof(double) * (size_t)g.n_tiles);
  w.dense = take(sparse ? sizeof(float) * (size_t)D : 0);
  w.hist = take(topk ? sizeof(uint32_t) * kTopkHistWords * (size_t)g.P : 0);
  w.state = take(topk ? sizeof(uint32_t) * (8 * (size_t)g.P + 8) : 0);
  w.guess = take(topk ? sizeof(uint32_t) * (size_t)g.P : 0);
  w.starts = take(topk ? sizeof(uint32_t) * kMaxWorkers * (size_t)g.P * (cdiv(p->part_elems, 8192) + 1) : 0);
  w.samp = take(topk ? sizeof(float) * 4096 * (size_t)g.P : 0);
  w.cand = take(topk ? 8 * (size_t)kTopkListCap * (size_t)g.P : 0);
  w.tilecnt = take(topk ? sizeof(uint32_t) * 2 * (size_t)g.n_tiles : 0);
  w.slots = take(sizeof(double) * 3 * ((size_t)g.P * cdiv(g.part_elems, kSTile)));
  w.norms = take(sizeof(double) * 3 * (size_t)g.P);
  w.total = off;
  return w;
}

// Extra workspace of LANS with caller-defined blocks (update.hip), placed where the block norms
// of the default blocks go (WsLayout::norms).  `tiles` = tiles of kSTile elements.
struct BlockWs {
  uint32_t *tot;      // [4 * n_blocks]: bits of phi, w_r, w_c of every block that reaches beyond a tile
  uint32_t *cnt;      // [n_blocks]: tiles of the block that have published their share
  double *tslots;     // [6 * tiles]: slots A and B of every tile, three sums each
  uint32_t *first;    // [tiles]: the block that holds the first element of the tile
  uint32_t *list;     // [1 + tiles]: number of deferred tiles, then their numbers
  size_t bytes;       // of all of the above
};
inline BlockWs block_ws(uint8_t *base, uint64_t n_blocks, uint64_t tiles) {
  BlockWs w;
  size_t off = 0;
  const uintptr_t at = reinterpret_cast<uintptr_t>(base);   // (base may be NULL when only the size is asked for)
  auto take = [&](size_t bytes) { uintptr_t q = at + off; off += (bytes + 255) / 256 * 256; return q; };
  w.tot = reinterpret_cast<uint32_t *>(take(16 * (size_t)n_blocks));
  w.cnt = reinterpret_cast<uint32_t *>(take(4 * (size_t)n_blocks));
  w.tslots = reinterpret_cast<double *>(take(48 * (size_t)tiles));
  w.first = reinterpret_cast<uint32_t *>(take(4 * (size_t)tiles));
  w.list = reinterpret_cast<uint32_t *>(take(4 * ((size_t)tiles + 1)));
  w.bytes = off;
  return w;
}

BPC_HD inline uint64_t k_of_device(const Geo &g, uint32_t p) { return k_rule(g.k_ratio, g.part_size(p)); }

}  // namespace bpc
