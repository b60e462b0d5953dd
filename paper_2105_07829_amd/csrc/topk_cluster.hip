// Top-k in a single pass over the data (Section 3.2; residual in the fused form of Section
// 4.2: the vector itself with the k sent slots zeroed).  A workgroup (512 threads) reads a tile
// (8192 elements) of its sources once, keeps v = g + e (worker) or v = mean + e~ (server) in
// registers and takes part in four partition-wide exchanges through global memory:
//
//   1-3  three-level radix select on the 31-bit magnitude key (11 + 10 + 10 bits): every tile
//        adds its LDS histogram of the current digit into the partition's histogram with
//        device-scope atomics, signs off on a counter, waits until all tiles of the
//        partition have, and reads the finished histogram; every tile then finds the bucket
//        of the k-th largest key for itself.  The result is the threshold key T and the
//        number r of keys equal to T that are kept;
//   4    tiles publish how many keys above / equal to T they hold and wait for the tiles
//        before them, which gives each tile its position in the index-ordered output (keys
//        equal to T are admitted lowest index first).
//
// Tiles are handed out by ticket in start order, so (as for the ticketed driver of
// cluster.hpp) every tile a workgroup waits for is running or about to, provided a partition
// has no more tiles than the device holds workgroups; all waits are bounded and report
// through the status word.  Traffic is the algorithmic minimum: sources read once, residual
// and message written once.
#include "cluster_launch.hpp"

namespace bpc {

constexpr int kTkThreads = 512;
constexpr int kTkPer = 16;                        // elements a thread keeps: few, so that 8 waves fit a SIMD
constexpr int kTkTile = kTkThreads * kTkPer;      // 8192
constexpr int kTkRows = kTkPer / 4;               // 4 rows of 2048; a thread owns 4 consecutive per row
constexpr int kTkRow = kTkThreads * 4;
static_assert(kTkTile == kSTile, "the workspace is laid out for tiles of kSTile elements");
constexpr int kTkBins1 = 2048, kTkBins23 = 1024;
constexpr int kTkHistPerPart = 4096;              // 2048 + 1024 + 1024 (layout shared with the multi-pass kernels)
constexpr uint64_t kTkPublished = 1ull << 63;
// Tiles of a partition add into kTkCopies copies of its histogram (tile number modulo the
// count): atomics on one cache line are performed one after the other, and a partition's
// tiles all hit the same few lines.
constexpr int kTkCopies = 2;

__device__ inline uint32_t tk_key(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// Where a tile's 16 values per thread come from.
template <class G, bool EF>
struct TkWorkerSrc {
  const G *grad;
  const float *res;
  __device__ void load(uint64_t tile_base, uint32_t valid, float v[kTkPer]) const {
    const TileBuf gb(grad + tile_base, valid * sizeof(G));
    const TileBuf eb(res + tile_base, EF ? valid * 4 : 0);
    u32x4 gr[kTkRows], er[kTkRows];
#pragma unroll
    for (int u = 0; u < kTkRows; ++u) {
      if (sizeof(G) == 4) {
        gr[u] = gb.load16<kNonTemporal>(threadIdx.x * 16, u * (kTkRow * 4));
      } else {
        const u32x2 h = gb.load8<kNonTemporal>(threadIdx.x * 8, u * (kTkRow * 2));
        gr[u].x = h.x; gr[u].y = h.y; gr[u].z = 0; gr[u].w = 0;
      }
      if (EF) er[u] = eb.load16<kNonTemporal>(threadIdx.x * 16, u * (kTkRow * 4));
    }
#pragma unroll
    for (int u = 0; u < kTkRows; ++u) {
      float w[4];
      if (sizeof(G) == 4) {
        w[0] = __uint_as_float(gr[u].x); w[1] = __uint_as_float(gr[u].y);
        w[2] = __uint_as_float(gr[u].z); w[3] = __uint_as_float(gr[u].w);
      } else {
        const uint32_t lo = gr[u].x, hi = gr[u].y;
        const float2 a = __half22float2(*reinterpret_cast<const __half2 *>(&lo));
        const float2 b = __half22float2(*reinterpret_cast<const __half2 *>(&hi));
        w[0] = a.x; w[1] = a.y; w[2] = b.x; w[3] = b.y;
      }
      const float e[4] = {__uint_as_float(er[u].x), __uint_as_float(er[u].y), __uint_as_float(er[u].z), __uint_as_float(er[u].w)};
#pragma unroll
      for (int c = 0; c < 4; ++c) v[4 * u + c] = EF ? w[c] + e[c] : w[c];
    }
  }
};
// Server: Delta = sum * (1/n) + e~ from the dense sum of the decoded worker messages.
template <bool EF>
struct TkServerSrc {
  const float *sum;
  const float *res;
  float inv_n;
  __device__ void load(uint64_t tile_base, uint32_t valid, float v[kTkPer]) const {
    const TileBuf sb(sum + tile_base, valid * 4);
    const TileBuf eb(res + tile_base, EF ? valid * 4 : 0);
    u32x4 sr[kTkRows], er[kTkRows];
#pragma unroll
    for (int u = 0; u < kTkRows; ++u) {
      sr[u] = sb.load16<kNonTemporal>(threadIdx.x * 16, u * (kTkRow * 4));
      if (EF) er[u] = eb.load16<kNonTemporal>(threadIdx.x * 16, u * (kTkRow * 4));
    }
#pragma unroll
    for (int u = 0; u < kTkRows; ++u) {
      const float s[4] = {__uint_as_float(sr[u].x), __uint_as_float(sr[u].y), __uint_as_float(sr[u].z), __uint_as_float(sr[u].w)};
      const float e[4] = {__uint_as_float(er[u].x), __uint_as_float(er[u].y), __uint_as_float(er[u].z), __uint_as_float(er[u].w)};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float mean = s[c] * inv_n;
        v[4 * u + c] = EF ? mean + e[c] : mean;
      }
    }
  }
};

struct TkArgs {
  Geo g;
  ClusterGeo cg;
  float *res_out;       // residual written in place (NULL: no error feedback)
  uint8_t *payload;
  uint32_t *hist;       // [P][kTkCopies][4096], zeroed
  uint32_t *flags;      // [3][P * tiles_per_part]: tile has added its level-1..3 histogram; zeroed
  uint64_t *tilecnt;    // [n_items]: published (equal << 32 | greater) counts; zeroed
  uint32_t *status;     // word 0: a wait gave up; word 1: ticket counter; both zeroed
};

// Waits (first wave) until the `count` flags from `flags` on are all set; bounded.  Every tile
// has a flag of its own: polling one shared counter would queue the polls of a whole
// partition, and the sign-offs behind them, on a single address.
__device__ inline void tk_wait_flags(const uint32_t *flags, uint32_t count, uint32_t *status) {
  if (threadIdx.x < 64) {
    int spins = 0;
    for (;;) {
      bool ok = true;
      for (uint32_t s = threadIdx.x; s < count; s += 64)
        ok = ok && __hip_atomic_load(flags + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
      if (__all(ok)) break;
      if (++spins > kSpinLimit) {
        if (threadIdx.x == 0) atomicOr(status, 1u);
        break;
      }
      __builtin_amdgcn_s_sleep(16);
    }
  }
  __syncthreads();
}

// One level of the select.  `in_play(key)` says whether a key still competes and `digit(key)`
// is its bucket; on return *prefix_io / *k_rem_io describe the next level.
template <int BINS, int LEVEL>
__device__ inline void tk_level(const TkArgs &a, uint32_t p, uint32_t copy, uint32_t tiles_in_part, const uint32_t key_of[kTkPer],
                                uint32_t *h /*LDS, BINS*/, uint32_t *scan /*LDS, threads*/, uint32_t *sh /*LDS, 2*/,
                                uint32_t *prefix_io, uint32_t *k_rem_io) {
  const uint32_t prefix = *prefix_io, k_rem = *k_rem_io;
  constexpr int kHiShift = LEVEL == 1 ? 31 : LEVEL == 2 ? 20 : 10;   // level 1: every key competes (key >> 31 == 0)
  constexpr int kLoShift = LEVEL == 1 ? 20 : LEVEL == 2 ? 10 : 0;
  for (int b = threadIdx.x; b < BINS; b += kTkThreads) h[b] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kTkPer; ++i) {
    const uint32_t key = key_of[i];
    if ((key >> kHiShift) == prefix) atomicAdd(&h[(key >> kLoShift) & (BINS - 1)], 1u);
  }
  __syncthreads();
  uint32_t *gh = a.hist + (uint64_t)p * (kTkCopies * kTkHistPerPart) + (LEVEL == 1 ? 0 : LEVEL == 2 ? kTkBins1 : kTkBins1 + kTkBins23);
  uint32_t *mine = gh + (copy % kTkCopies) * kTkHistPerPart;
  for (int b = threadIdx.x; b < BINS; b += kTkThreads)
    if (h[b]) __hip_atomic_fetch_add(&mine[b], h[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  // the adds have been performed once the vector-memory counter has drained; only then sign off
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  uint32_t *flags = a.flags + (uint64_t)(LEVEL - 1) * a.g.P * a.cg.tiles_per_part + (uint64_t)p * a.cg.tiles_per_part;
  if (threadIdx.x == 0) __hip_atomic_store(flags + copy, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  tk_wait_flags(flags, tiles_in_part, a.status);
  // bucket b with  count(buckets above b) < k_rem <= count(buckets above b) + count(b);
  // thread t owns buckets BINS-1 - t*PER - (PER-1) .. BINS-1 - t*PER, highest first
  constexpr int kPer = BINS / kTkThreads;
  uint32_t cnt[kPer];
  uint32_t local = 0;
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    // the histogram is final by now and was not read before: plain loads
    uint32_t c = 0;
#pragma unroll
    for (int q = 0; q < kTkCopies; ++q) c += gh[q * kTkHistPerPart + BINS - 1 - (threadIdx.x * kPer + i)];
    cnt[i] = c;
    local += c;
  }
  uint32_t total;
  const uint32_t above = block_exclusive_scan<kTkThreads>(local, scan, &total);
  if (above < k_rem && k_rem <= above + local) {
    uint32_t run = above;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      if (run < k_rem && k_rem <= run + cnt[i]) {
        const uint32_t bin = BINS - 1 - (threadIdx.x * kPer + i);
        sh[0] = LEVEL == 1 ? bin : ((prefix << 10) | bin);
        sh[1] = k_rem - run;
      }
      run += cnt[i];
    }
  }
  __syncthreads();
  *prefix_io = __builtin_amdgcn_readfirstlane(sh[0]);
  *k_rem_io = __builtin_amdgcn_readfirstlane(sh[1]);
  __syncthreads();
}

template <class SRC>
__global__ __launch_bounds__(kTkThreads, 5) void topk_single_kernel(const TkArgs a, const SRC src) {
  __shared__ uint32_t h[kTkBins1];
  __shared__ uint32_t scan[kTkThreads];
  __shared__ uint32_t sh[4];
  __shared__ uint32_t wave_cnt[2][kTkRows][kTkThreads / 64];
  if (threadIdx.x == 0) sh[2] = atomicAdd(a.status + 1, 1u);
  __syncthreads();
  const uint32_t item = __builtin_amdgcn_readfirstlane(sh[2]);
  if (item >= a.cg.n_items) return;
  const Geo &g = a.g;
  const uint32_t p = __builtin_amdgcn_readfirstlane(item / a.cg.tiles_per_part);
  const uint32_t tile = __builtin_amdgcn_readfirstlane(item % a.cg.tiles_per_part);
  const uint32_t d = g.part_size(p);
  const uint32_t tiles_in_part = (uint32_t)cdiv(d, kTkTile);
  const uint32_t tile_off = tile * kTkTile;
  const uint32_t valid = d - tile_off < (uint32_t)kTkTile ? d - tile_off : (uint32_t)kTkTile;
  const uint64_t tile_base = g.part_base(p) + tile_off;
  const uint32_t k = (uint32_t)k_of_device(g, p);

  // elements past the partition's end read as 0: key 0 and the highest indices, so with
  // k <= d they are never among the kept
  // the values are kept as magnitude keys plus one word of sign bits
  uint32_t key[kTkPer];
  uint32_t neg_bits = 0;
  {
    float v[kTkPer];
    src.load(tile_base, valid, v);
#pragma unroll
    for (int i = 0; i < kTkPer; ++i) {
      key[i] = tk_key(v[i]);
      neg_bits |= (__float_as_uint(v[i]) >> 31) << i;
    }
  }
  // from here on the keys and the sign word are all there is (without this the compiler keeps
  // the values, and everything it derives from the keys, in registers of their own)
#pragma unroll
  for (int i = 0; i < kTkPer; ++i) asm volatile("" : "+v"(key[i]));
  asm volatile("" : "+v"(neg_bits));

  uint32_t prefix = 0, k_rem = k;
  tk_level<kTkBins1, 1>(a, p, tile, tiles_in_part, key, h, scan, sh, &prefix, &k_rem);
  tk_level<kTkBins23, 2>(a, p, tile, tiles_in_part, key, h, scan, sh, &prefix, &k_rem);
  tk_level<kTkBins23, 3>(a, p, tile, tiles_in_part, key, h, scan, sh, &prefix, &k_rem);
  const uint32_t T = prefix, r = k_rem;

  // Index order inside the tile is (row, wave, lane, component).  For both classes (key > T,
  // key == T): elements of lower lanes of the same wave and row from ballots, whole waves and
  // rows before from a table in LDS.
  const uint32_t wave = threadIdx.x >> 6;
  // bit i: element i of this thread lies inside the partition and its key is above T / equals T
  uint32_t gt_bits = 0, eq_bits = 0;
#pragma unroll
  for (int i = 0; i < kTkPer; ++i) {
    const bool in = (uint32_t)((i >> 2) * kTkRow) + threadIdx.x * 4 + (i & 3) < valid;
    gt_bits |= (in && key[i] > T ? 1u : 0u) << i;
    eq_bits |= (in && key[i] == T ? 1u : 0u) << i;
  }
  // keep the two words as the only record of the classes (otherwise the compiler carries
  // the 64 individual predicates along in registers of their own)
  asm volatile("" : "+v"(gt_bits), "+v"(eq_bits));
  uint32_t start_gt[kTkRows], start_eq[kTkRows];   // of the class, in the tile, before this thread's row segment
#pragma unroll
  for (int u = 0; u < kTkRows; ++u) {
    // this thread's greater keys (low half) and ties (high half) of the row
    const uint32_t mine = __popc((gt_bits >> (4 * u)) & 15u) + (__popc((eq_bits >> (4 * u)) & 15u) << 16);
    const uint32_t incl = wave_inclusive_scan_u32(mine);   // at most 256 per half: no carry between them
    const uint32_t excl = incl - mine;
    start_gt[u] = excl & 0xffffu;
    start_eq[u] = excl >> 16;
    if ((threadIdx.x & 63) == 63) {
      wave_cnt[0][u][wave] = incl & 0xffffu;
      wave_cnt[1][u][wave] = incl >> 16;
    }
  }
  __syncthreads();
  // add what whole waves and rows before contribute: a walk over the (row, wave) table
  uint32_t tile_gt = 0, tile_eq = 0;
#pragma unroll
  for (int u = 0; u < kTkRows; ++u) {
    uint32_t part_gt = 0, part_eq = 0, row_gt = 0, row_eq = 0;
#pragma unroll
    for (int w = 0; w < kTkThreads / 64; ++w) {
      const uint32_t cg = wave_cnt[0][u][w], ce = wave_cnt[1][u][w];
      part_gt += (uint32_t)w < wave ? cg : 0u;
      part_eq += (uint32_t)w < wave ? ce : 0u;
      row_gt += cg;
      row_eq += ce;
    }
    start_gt[u] += tile_gt + part_gt;
    start_eq[u] += tile_eq + part_eq;
    tile_gt += row_gt;
    tile_eq += row_eq;
  }
  // exchange 4: counts of the tiles before this one
  uint64_t *slots = a.tilecnt + (uint64_t)p * a.cg.tiles_per_part;
  if (threadIdx.x == 0)
    __hip_atomic_store(slots + tile, kTkPublished | ((uint64_t)tile_eq << 32) | tile_gt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (threadIdx.x < 64) {
    uint64_t acc_gt = 0, acc_eq = 0;
    int spins = 0;
    for (;;) {
      bool ok = true;
      acc_gt = 0; acc_eq = 0;
      for (uint32_t s = threadIdx.x; s < tile; s += 64) {
        const uint64_t x = __hip_atomic_load(slots + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = ok && (x & kTkPublished);
        acc_gt += (uint32_t)x;
        acc_eq += (uint32_t)((x & ~kTkPublished) >> 32);
      }
      if (__all(ok)) break;
      if (++spins > kSpinLimit) {
        if (threadIdx.x == 0) atomicOr(a.status, 1u);
        break;
      }
      __builtin_amdgcn_s_sleep(8);
    }
    uint32_t s_gt = (uint32_t)acc_gt, s_eq = (uint32_t)acc_eq;
    s_gt = wave_sum_u32(s_gt);
    s_eq = wave_sum_u32(s_eq);
    if (threadIdx.x == 0) { sh[0] = s_gt; sh[1] = s_eq; }
  }
  __syncthreads();
  const uint32_t gt_before = sh[0], eq_before = sh[1];

  uint8_t *rec = a.payload + (uint64_t)p * g.stride;
  if (tile == 0 && threadIdx.x == 0) {
    uint32_t *hdr = reinterpret_cast<uint32_t *>(rec);
    hdr[0] = k;
    hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
  }
  // the record's index and value arrays, k entries each
  const TileBuf idx(rec + kHeaderBytes, k * 4);
  const TileBuf val(rec + kHeaderBytes + 4 * ru4(g.k_cap), k * 4);
  const uint32_t ties_tile = eq_before < r ? eq_before : r;   // ties admitted before this tile
#pragma unroll
  for (int u = 0; u < kTkRows; ++u) {
    uint32_t n_gt = start_gt[u];                  // greater keys of the tile before this element
    uint32_t eq_rank = eq_before + start_eq[u];   // rank of this element among the partition's ties, if it is one
    float out[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float x = __uint_as_float(key[4 * u + c] | (((neg_bits >> (4 * u + c)) & 1u) << 31));
      const bool gt = (gt_bits >> (4 * u + c)) & 1u, tie = (eq_bits >> (4 * u + c)) & 1u;
      const bool take = gt || (tie && eq_rank < r);
      if (take) {
        const uint32_t ties_here = (eq_rank < r ? eq_rank : r) - ties_tile;   // ties admitted in this tile before this element
        const uint32_t pos = gt_before + ties_tile + n_gt + ties_here;
        idx.store4(tile_off + (uint32_t)(u * kTkRow) + threadIdx.x * 4 + c, pos * 4, 0);
        val.store4(__float_as_uint(x), pos * 4, 0);
      }
      n_gt += gt ? 1u : 0u;
      eq_rank += tie ? 1u : 0u;
      out[c] = take ? 0.0f : x;
    }
    if (a.res_out) {
      const TileBuf ob = row_buf(a.res_out + tile_base, valid, u * kTkRow, kTkRow);
      ob.store16<kNonTemporal>(as_u32x4(out[0], out[1], out[2], out[3]), threadIdx.x * 16);
    }
    __builtin_amdgcn_sched_barrier(0);   // one row at a time: interleaving rows costs registers
  }
}

// zeroes the histograms, the sign-off counters, the published counts and the status words
__global__ __launch_bounds__(256) void topk_reset_kernel(uint32_t *hist, size_t hist_words, uint32_t *flags, size_t flag_words,
                                                         uint64_t *tilecnt, size_t n_items, uint32_t *status) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, st = (size_t)gridDim.x * 256;
  for (size_t k = i; k < hist_words; k += st) hist[k] = 0;
  for (size_t k = i; k < flag_words; k += st) flags[k] = 0;
  for (size_t k = i; k < n_items; k += st) tilecnt[k] = 0;
  if (i < 2) status[i] = 0;
}

template <class SRC>
static hipError_t launch_topk_single(const TkArgs &a, const SRC &src, const Workspace &ws, hipStream_t stream, bool *used) {
  const void *fn = reinterpret_cast<const void *>(&topk_single_kernel<SRC>);
  static int capacity = 0;
  if (capacity == 0) capacity = cluster_capacity(fn, kTkThreads, 0);
  *used = false;
  if (capacity <= 0 || a.cg.tiles_per_part > (uint32_t)capacity) return hipSuccess;
  *used = true;
  hipError_t e = cluster_launch_begin(stream);
  if (e != hipSuccess) return e;
  const size_t hist_words = (size_t)kTkCopies * kTkHistPerPart * a.g.P, flag_words = (size_t)3 * a.g.P * a.cg.tiles_per_part;
  topk_reset_kernel<<<256, 256, 0, stream>>>(a.hist, hist_words, a.flags, flag_words, a.tilecnt, a.cg.n_items, a.status);
  topk_single_kernel<SRC><<<a.cg.n_items, kTkThreads, 0, stream>>>(a, src);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  (void)ws;
  return cluster_launch_end(stream);
}

// `dense_sum`: server only, the sum of the decoded worker messages.  *used = false when the
// shape cannot take this kernel (the caller then runs the multi-pass kernels).
hipError_t topk_single_pass(const Geo &g, const Source &src, const float *dense_sum, uint8_t *payload,
                            const Workspace &ws, hipStream_t stream, bool *used) {
  *used = false;
  if (g.part_elems % kTkTile != 0) return hipSuccess;
  if (src.grad && src.dtype == BPC_F16 && (g.D & 1)) return hipSuccess;   // descriptors bound at dword granularity
  TkArgs a;
  a.g = g;
  a.cg = make_cluster_geo(g, kTkTile);
  a.res_out = src.residual;
  a.payload = payload;
  a.hist = ws.at<uint32_t>(ws.lay.hist);
  a.flags = ws.at<uint32_t>(ws.lay.partials);   // 16 bytes a tile there, 12 needed
  a.tilecnt = ws.at<uint64_t>(ws.lay.tilecnt);
  a.status = ws.at<uint32_t>(ws.lay.status);
  const bool ef = src.residual != nullptr;
  if (src.grad) {
    if (src.dtype == BPC_F16) {
      if (ef) return launch_topk_single(a, TkWorkerSrc<__half, true>{(const __half *)src.grad, src.residual}, ws, stream, used);
      return launch_topk_single(a, TkWorkerSrc<__half, false>{(const __half *)src.grad, nullptr}, ws, stream, used);
    }
    if (ef) return launch_topk_single(a, TkWorkerSrc<float, true>{(const float *)src.grad, src.residual}, ws, stream, used);
    return launch_topk_single(a, TkWorkerSrc<float, false>{(const float *)src.grad, nullptr}, ws, stream, used);
  }
  if (ef) return launch_topk_single(a, TkServerSrc<true>{dense_sum, src.residual, src.msgs.inv_n}, ws, stream, used);
  return launch_topk_single(a, TkServerSrc<false>{dense_sum, nullptr, src.msgs.inv_n}, ws, stream, used);
}

}  // namespace bpc
