// Top-k compressor (Section 3.2: of a gradient only its k entries of largest magnitude travel)
// with the residual update of Algorithm 4 in its fused form (Section 4.2, operator fusion: the
// residual is the vector itself with the k sent slots set to zero).
//
// Selection is exact: a three-level radix select on the 31-bit magnitude key
// bits(v) & 0x7fffffff (11 + 10 + 10 bits); elements equal to the threshold key are admitted
// lowest index first, and the record lists its entries by ascending index.
//
// Short-list form (k of a full partition at most half of kTopkListCap): one pass over the data.
//   sample     : 4096 elements of each partition (512 evenly spread chunks of eight); the key G
//                at a rank of the sample chosen so that, but for rare cases, at least k and
//                at most about 2 k elements of the partition have keys >= G
//   load+hist1 : v_j from the source -> dense buffer; the elements with key >= G go to the
//                partition's short list and into the histogram of key >> 20
//   select     : one workgroup per partition runs the radix select on the short list alone
//                and writes the record; kept slots of the buffer zeroed
// The sample only decides how much work the selection is, never its result: a partition whose
// short list came out shorter than k or longer than kTopkListCap (the sample misled, or a
// great many equal magnitudes, or fewer than k non-zeros) is taken by the long form below
// instead: one more kernel, enqueued behind, which returns at once if no partition needs it
// and else runs the long form's passes for those partitions (the rest of their level-1
// histogram first) with its resident grid meeting between the passes.
//
// Long form (a k too large for a short list), five passes over the dense buffer:
//   load+hist1 : as above, every element counted
//   hist2      : bin of level 1 that holds the k-th largest key, histogram inside it
//   hist3      : the same one level down
//   count      : threshold key T and the number r of elements with key == T that are kept;
//                per tile, how many keys are > T and == T
//   emit       : (idx, val) in ascending index order; kept slots of the buffer zeroed
// Each pass works out the selection so far from the histograms of the passes before it (every
// workgroup for itself), so no launches sit between the passes.
//
// Server side the vector is Delta = (sum of the n decoded messages) / n + e~.  It is never
// scattered into a dense buffer (n k read-modify-writes at random places of HBM per partition):
// the messages list their entries by ascending index, so the load pass sums the stretch of each
// message that falls into its group of 8192 elements in LDS, and the sample pass collects the
// sums of the sampled chunks in one sweep over the messages.
#include "cluster.hpp"
#include "sources.hpp"
#include "tile_rows.hpp"

namespace bpc {

constexpr int kBins1 = 2048, kBins23 = 1024;
constexpr int kHist1 = 0, kHist2 = kBins1, kHist3 = kHist2 + kBins23;
static_assert(kHist3 + kBins23 == kTopkHistWords, "histogram words of a partition");
constexpr int kShift1 = 20, kShift2 = 10;
constexpr int kBits1 = 11, kBits23 = 10;
// A workgroup of the histogram / count passes handles a few consecutive tiles of one partition
// (template parameter TPG): its LDS histogram is merged into the partition's with one atomic
// per non-empty bin, so more tiles a workgroup mean fewer of those (an atomic on global memory
// costs some 11 ns of one memory channel's time; they were the larger part of the level-2
// pass), while fewer, longer workgroups hide less latency (8 tiles a workgroup doubled the
// time of the passes that only read).
constexpr int kTpgLoad = 2, kTpgHist2 = 4, kTpgHist3 = 1, kTpgCount = 1;
constexpr int kSelThreads = 1024;                       // workgroup of the select pass
constexpr int kSelPer = kTopkListCap / kSelThreads;     // list entries a thread of it keeps
constexpr uint32_t kGatedGrid = 1024;                   // grid of the long-form kernel behind the short-list form, at most
constexpr int kSamplePer = 16;                          // sampled elements per thread of the sample pass
constexpr uint32_t kSample = kThreads * kSamplePer;     // per partition: 4096
constexpr uint32_t kNoGuess = 0xffffffffu;              // no key reaches it: nothing goes to the short list

__device__ inline uint32_t key_of(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// state words per partition: words 2L, 2L + 1 hold (prefix, rank left) after level L = 1..3;
// word 0 the length of the short list, word 1 non-zero if the partition is left to the long form
enum { kStPrefix = 0, kStKRem = 1 };
enum { kStListLen = 0, kStLong = 1 };

// Whether partition p is left to the long form (uniform over the workgroup).
__device__ inline bool long_form(const uint32_t *state, uint32_t p) {
  return __builtin_amdgcn_readfirstlane(state[p * 8 + kStLong]) != 0;
}

// Group `blk` of TPG consecutive tiles of one partition.
struct GroupOf {
  uint32_t p, tile_lo, tile_hi, d;
};
template <int TPG>
__device__ inline GroupOf group_of(const Geo &g, uint32_t blk) {
  constexpr uint32_t kTilesPerGroup = TPG;
  const uint32_t groups_per_part = (uint32_t)cdiv(g.tiles_per_part, kTilesPerGroup);
  GroupOf r;
  r.p = blk / groups_per_part;
  r.d = g.part_size(r.p);
  const uint32_t n_tiles = (uint32_t)cdiv(r.d, kTile);
  r.tile_lo = (blk % groups_per_part) * kTilesPerGroup;
  r.tile_hi = r.tile_lo + kTilesPerGroup < n_tiles ? r.tile_lo + kTilesPerGroup : n_tiles;
  return r;
}
inline uint32_t group_count(const Geo &g, int tpg) { return g.P * (uint32_t)cdiv(g.tiles_per_part, tpg); }

// All threads of a workgroup of THREADS: walk a histogram `h` of BINS bins (global or LDS)
// from the highest bin down and find the bin b with
//   count(bins above b) < k_rem <= count(bins above b) + count(b).
// sel[0] = (prefix << BITS) | b (the extended prefix), sel[1] = the rank left inside b.
// Every workgroup of the pass that follows a histogram pass does this for itself (a few
// microseconds of L2 reads) instead of a launch of its own in between.
template <int BINS, int BITS, int THREADS>
__device__ inline void pick_bin(const uint32_t *h, uint32_t k_rem, uint32_t prefix, uint32_t *scan, uint32_t *sel) {
  constexpr int kPer = BINS / THREADS > 0 ? BINS / THREADS : 1;
  // thread t owns bins BINS-1 - t*kPer - i, highest first; threads past the bins own none
  uint32_t cnt[kPer];
  uint32_t local = 0;
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    const uint32_t b = threadIdx.x * kPer + i;
    cnt[i] = b < (uint32_t)BINS ? h[BINS - 1 - b] : 0u;
    local += cnt[i];
  }
  uint32_t total;
  const uint32_t above = block_exclusive_scan<THREADS>(local, scan, &total);
  if (above < k_rem && k_rem <= above + local) {
    uint32_t run = above;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      if (run < k_rem && k_rem <= run + cnt[i]) {
        sel[0] = (prefix << BITS) | (BINS - 1 - (threadIdx.x * kPer + i));
        sel[1] = k_rem - run;
      }
      run += cnt[i];
    }
  }
  __syncthreads();
}

// Radix select, inside one workgroup of THREADS, among the keys of the values the threads hold
// in registers (the low 31 bits of bits[i], i < cnt <= rounds, `rounds` the same for all
// threads).  h: LDS, kBins1 words.
// Level 1: the level-1 bin of the key of rank `rank` (1 = the largest) in sel[0], the rank left
// inside it in sel[1].
template <int PER, int THREADS>
__device__ inline void level1_in_registers(const uint32_t (&bits)[PER], uint32_t cnt, uint32_t rounds, uint32_t rank,
                                           uint32_t *h, uint32_t *scan, uint32_t *sel) {
  for (int b = threadIdx.x; b < kBins1; b += THREADS) h[b] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    if ((uint32_t)i >= rounds) break;
    if ((uint32_t)i < cnt) atomicAdd(&h[(bits[i] & 0x7fffffffu) >> kShift1], 1u);
  }
  __syncthreads();
  pick_bin<kBins1, kBits1, THREADS>(h, rank, 0, scan, sel);
}
// Levels 2 and 3, given level 1's (b1, k_rem1): the key in sel[0], the rank left among the keys
// equal to it in sel[1].
template <int PER, int THREADS>
__device__ inline void levels23_in_registers(const uint32_t (&bits)[PER], uint32_t cnt, uint32_t rounds, uint32_t b1,
                                             uint32_t k_rem1, uint32_t *h, uint32_t *scan, uint32_t *sel) {
  for (int b = threadIdx.x; b < kBins23; b += THREADS) h[b] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    if ((uint32_t)i >= rounds) break;
    const uint32_t key = bits[i] & 0x7fffffffu;
    if ((uint32_t)i < cnt && (key >> kShift1) == b1) atomicAdd(&h[(key >> kShift2) & (kBins23 - 1)], 1u);
  }
  __syncthreads();
  pick_bin<kBins23, kBits23, THREADS>(h, k_rem1, b1, scan, sel);
  const uint32_t prefix2 = sel[0], k_rem2 = sel[1];
  __syncthreads();
  for (int b = threadIdx.x; b < kBins23; b += THREADS) h[b] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    if ((uint32_t)i >= rounds) break;
    const uint32_t key = bits[i] & 0x7fffffffu;
    if ((uint32_t)i < cnt && (key >> kShift2) == prefix2) atomicAdd(&h[key & (kBins23 - 1)], 1u);
  }
  __syncthreads();
  pick_bin<kBins23, kBits23, THREADS>(h, k_rem2, prefix2, scan, sel);
}

// Chunk (of eight consecutive elements) number c of the sample of a partition sampled every
// `stride` chunks: one of the c-th stretch of `stride` chunks, at a place that moves from
// stretch to stretch (chunks at equal distances of a power of two would all come from the same
// few memory channels).
__device__ inline uint32_t sample_chunk(uint32_t c, uint32_t stride) { return c * stride + (c * 37u) % stride; }

// Sample chunks and their spacing for a partition of d elements.
__device__ inline uint32_t sample_chunks(uint32_t d) { return d / 8 < kSample / 8 ? d / 8 : kSample / 8; }

constexpr uint32_t kGroupElems = kTpgLoad * kTile;   // elements a workgroup of the load pass takes: 8192
static_assert(kGroupElems == 8192, "the workspace is laid out for groups of 8192 elements");

// Server side: Delta = (sum of the n decoded top-k messages) / n + e~ straight from the
// messages.  A message lists its entries by ascending index, so the entries of a group of
// 8192 elements are one stretch of it; `topk_starts_kernel` records where each stretch begins.
struct TopkMsgs {
  WorkerMsgs msgs;
  const float *res;
  const uint32_t *starts;   // [worker][partition][group .. groups_per_part]
  uint32_t groups_per_part, k_cap;
  uint64_t stride;
  int half;
  uint32_t group_shift;     // log2 of the elements of a group (13 for the load pass)
  __device__ const uint8_t *rec(int i, uint32_t p) const { return msgs.ptr[i] + (uint64_t)p * stride; }
  __device__ uint32_t k_of(int i, uint32_t p) const {
    const uint32_t k = *reinterpret_cast<const uint32_t *>(rec(i, p));
    return k > k_cap ? k_cap : k;
  }
  __device__ const uint32_t *idx(int i, uint32_t p) const { return reinterpret_cast<const uint32_t *>(rec(i, p) + kHeaderBytes); }
  __device__ float value(int i, uint32_t p, uint32_t t) const {
    const uint8_t *v = rec(i, p) + kHeaderBytes + 4 * ru4(k_cap);
    return half ? __half2float(reinterpret_cast<const __half *>(v)[t]) : reinterpret_cast<const float *>(v)[t];
  }
  // The residual's eight elements from j0 (zeros without a residual or past the end), and
  // Delta from them and the sums of the decoded messages.
  __device__ void load_res8(const Geo &g, uint32_t p, uint32_t j0, uint32_t d, float r[8]) const {
    const uint64_t i0 = g.part_base(p) + j0;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = 0.0f;
    if (res) {
      if (j0 + 8 <= d) load8_aligned(res + i0, r);
      else
        for (int e = 0; e < 8; ++e) r[e] = j0 + e < d ? res[i0 + e] : 0.0f;
    }
  }
  __device__ void combine8(uint32_t j0, uint32_t d, const float *sum, const float r[8], float out[8]) const {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float mean = sum[e] * msgs.inv_n;
      out[e] = j0 + e < d ? (res ? mean + r[e] : mean) : 0.0f;
    }
  }
  __device__ void finish8(const Geo &g, uint32_t p, uint32_t j0, uint32_t d, const float *sum, float out[8]) const {
    float r[8];
    load_res8(g, p, j0, d, r);
    combine8(j0, d, sum, r, out);
  }
};

// For t = 0 .. k: entry t is the first one of every group after the group of entry t - 1 up to
// its own group (t = k: up to the end).  A message that is not in ascending order leaves
// groups unset; readers clamp what they find to [0, k].
// The same sweep adds the entries that fall into the chunks of the sample pass to `samp`
// (zeroed before; about one entry in 250, so the global atomics do not matter, and the guess
// needs no particular order of the sum); `samp` may be null.
__global__ __launch_bounds__(kThreads) void topk_starts_kernel(Geo g, TopkMsgs m, uint32_t *starts, float *samp) {
  const uint32_t p = blockIdx.y, i = blockIdx.z;
  const uint32_t k = m.k_of(i, p);
  const uint32_t *idx = m.idx(i, p);
  uint32_t *tab = starts + ((uint64_t)i * g.P + p) * (m.groups_per_part + 1);
  auto group = [&](uint32_t j) { const uint32_t q = j >> m.group_shift; return q < m.groups_per_part ? q : m.groups_per_part - 1; };
  const uint32_t d = g.part_size(p);
  const uint32_t chunks = sample_chunks(d), stride = chunks ? (d / 8) / chunks : 1u;
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t <= k; t += gridDim.x * kThreads) {
    const uint32_t first = t == 0 ? 0u : group(idx[t - 1]) + 1;
    const uint32_t last = t == k ? m.groups_per_part : group(idx[t]);
    for (uint32_t q = first; q <= last && q <= m.groups_per_part; ++q) tab[q] = t;
    if (samp && t < k) {
      const uint32_t j = idx[t], cj = j >> 3, c = cj / stride;
      if (c < chunks && cj == sample_chunk(c, stride)) atomicAdd(&samp[(uint64_t)p * kSample + c * 8 + (j & 7u)], m.value(i, p, t));
    }
  }
}

// The load pass's view: the workgroup's group of 8192 elements summed in LDS, worker by worker
// (a barrier in between: the order of the sum is the workers'), a thread's first entry of the
// next worker requested before the adds of this one.
struct TopkMsgsGroupSource : TopkMsgs {
  static constexpr int kLdsFloats = kGroupElems + 5 * kMaxWorkers + 2;   // sums, ranges, counts before, record addresses
  __device__ void begin(const Geo &, uint32_t, float *) const {}
  __device__ void begin_group(const Geo &g, uint32_t p, uint32_t grp, float *lds) const {
    uint32_t *range = reinterpret_cast<uint32_t *>(lds + kGroupElems);
    // (the records' addresses go to LDS: a thread's entries belong to workers it finds at run
    // time, and indexing the kernel arguments by such a number is a memory access of its own)
    const uint8_t **recs = reinterpret_cast<const uint8_t **>(lds + kGroupElems + 3 * kMaxWorkers + 2);
    const uint32_t lo = grp * kGroupElems;
    if (threadIdx.x < (uint32_t)msgs.n) {
      recs[threadIdx.x] = rec(threadIdx.x, p);
      const uint32_t *tab = starts + ((uint64_t)threadIdx.x * g.P + p) * (groups_per_part + 1);
      const uint32_t k = k_of(threadIdx.x, p);
      const uint32_t s = tab[grp] < k ? tab[grp] : k, e = tab[grp + 1] < k ? tab[grp + 1] : k;
      range[2 * threadIdx.x] = s;
      range[2 * threadIdx.x + 1] = e < s ? s : e;
    }
    for (uint32_t q = threadIdx.x; q < kGroupElems / 4; q += kThreads) reinterpret_cast<float4 *>(lds)[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    __syncthreads();
    // entries of the group before worker i's, over all workers
    uint32_t *cum = range + 2 * kMaxWorkers;
    if (threadIdx.x < 64) {
      const uint32_t c = threadIdx.x < (uint32_t)msgs.n ? range[2 * threadIdx.x + 1] - range[2 * threadIdx.x] : 0u;
      const uint32_t incl = wave_inclusive_scan_u32(c);
      cum[threadIdx.x + 1] = incl;
      if (threadIdx.x == 0) cum[0] = 0;
    }
    __syncthreads();
    const uint32_t total = cum[msgs.n];
    constexpr int kMine = 4;   // entries a thread takes
    if (total <= (uint32_t)(kMine * kThreads)) {
      // all the group's entries are requested at once (worker-major, so a thread's entries come
      // in worker order), then added worker by worker with a barrier in between
      uint32_t rel[kMine], who[kMine];
      float val[kMine];
#pragma unroll
      for (int r = 0; r < kMine; ++r) {
        const uint32_t q = r * kThreads + threadIdx.x;
        who[r] = 0xffffffffu;
        rel[r] = 0;
        val[r] = 0.0f;
        if (q < total) {
          uint32_t a = 0, b = msgs.n;   // cum[a] <= q < cum[b]
          while (b - a > 1) {
            const uint32_t mid = (a + b) >> 1;
            if (cum[mid] <= q) a = mid; else b = mid;
          }
          const uint32_t t = range[2 * a] + (q - cum[a]);
          const uint8_t *rc = recs[a];
          who[r] = a;
          rel[r] = reinterpret_cast<const uint32_t *>(rc + kHeaderBytes)[t] - lo;
          const uint8_t *vp = rc + kHeaderBytes + 4 * ru4(k_cap);
          val[r] = half ? __half2float(reinterpret_cast<const __half *>(vp)[t]) : reinterpret_cast<const float *>(vp)[t];
        }
      }
      for (int i = 0; i < msgs.n; ++i) {
        if (cum[i + 1] != cum[i]) {   // (uniform)
#pragma unroll
          for (int r = 0; r < kMine; ++r)
            if (who[r] == (uint32_t)i && rel[r] < kGroupElems) lds[rel[r]] = lds[rel[r]] + val[r];
          __syncthreads();
        }
      }
    } else {
      for (int i = 0; i < msgs.n; ++i) {
        const uint32_t s = range[2 * i], e = range[2 * i + 1];
        for (uint32_t q = s + threadIdx.x; q < e; q += kThreads) {
          const uint32_t r = idx(i, p)[q] - lo;
          if (r < kGroupElems) lds[r] = lds[r] + value(i, p, q);
        }
        __syncthreads();
      }
    }
  }
};

// The sample pass's view of the same: the sums of the sampled chunks, collected by the sweep of
// `topk_starts_kernel`.
struct TopkMsgsSampleSource : TopkMsgs {
  const float *samp;
  static constexpr int kLdsFloats = 1;
  __device__ void begin(const Geo &, uint32_t, float *) const {}
  // j0: the first element of a sampled chunk
  __device__ void at8(const Geo &g, uint32_t p, uint32_t j0, uint32_t d, const float *, float out[8]) const {
    const uint32_t chunks = sample_chunks(d), stride = (d / 8) / chunks;
    float sum[8];
    load8_aligned(samp + (uint64_t)p * kSample + 8 * ((j0 >> 3) / stride), sum);
    finish8(g, p, j0, d, sum, out);
  }
};

// Zeroes the histograms and the state words; with `sample`, workgroup p < P also works out
// partition p's guess G from a sample of 512 chunks of eight consecutive elements (else the
// guess is "none").  Random 64-byte reads cost about as much as 16 times as many sequential
// ones, hence chunks rather than single elements.
template <class SRC>
__global__ __launch_bounds__(kThreads) void topk_sample_kernel(Geo g, SRC src, uint32_t *hist, uint32_t *state,
                                                               uint32_t *guess, int sample, uint32_t *status) {
  __shared__ __align__(16) float lds[SRC::kLdsFloats];
  __shared__ uint32_t h[kBins1];
  if (blockIdx.x == 0 && threadIdx.x == 0) status[0] = 0;   // (set by a wait of the long form that gave up)
  __shared__ uint32_t scan[kThreads];
  __shared__ uint32_t sel[2];
  {
    const size_t i0 = (size_t)blockIdx.x * kThreads + threadIdx.x, step = (size_t)gridDim.x * kThreads;
    uint4 *h16 = reinterpret_cast<uint4 *>(hist);
    for (size_t q = i0; q < (size_t)kTopkHistWords * g.P / 4; q += step) h16[q] = make_uint4(0, 0, 0, 0);
    for (size_t q = i0; q < 8ull * g.P + 8; q += step) state[q] = 0;   // (8 spare words: the long form's barrier counter)
  }
  const uint32_t p = blockIdx.x;
  if (p >= g.P) return;
  if (!sample) {
    if (threadIdx.x == 0) guess[p] = kNoGuess;
    return;
  }
  static_assert(kSamplePer % 8 == 0, "whole chunks");
  constexpr uint32_t kChunksPer = kSamplePer / 8;
  const uint32_t d = g.part_size(p);
  const uint32_t chunks = sample_chunks(d);                   // chunks in the sample (whole chunks of the partition only)
  const uint32_t m = 8 * chunks;                              // elements in the sample
  // rank in the sample: the expected rank of the partition's k-th largest, four standard
  // deviations of a count of twice that size further down (neighbours are not independent),
  // and a little more
  const double expect = (double)k_of_device(g, p) * (double)m / (double)d;
  const uint32_t rank = (uint32_t)(expect + 4.0 * sqrt(2.0 * expect) + 3.0);
  if (rank >= m) {   // (uniform) the whole partition would be listed
    if (threadIdx.x == 0) guess[p] = 0;
    return;
  }
  const uint32_t stride = (d / 8) / chunks;
  src.begin(g, p, lds);
  __syncthreads();
  uint32_t key[kSamplePer];
  uint32_t cnt = 0;
  // (every load is issued, with chunk 0 standing in past the end, so that none is waited for
  // before the last is on its way)
#pragma unroll
  for (uint32_t i = 0; i < kChunksPer; ++i) {
    const uint32_t c = i * kThreads + threadIdx.x;
    float v[8];
    source_at8(src, g, p, 8 * sample_chunk(c < chunks ? c : 0u, stride), d, lds, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) key[8 * i + e] = key_of(v[e]);
    cnt += c < chunks ? 8 : 0;
  }
  level1_in_registers<kSamplePer, kThreads>(key, cnt, kSamplePer, rank, h, scan, sel);
  const uint32_t b1 = sel[0], k_rem1 = sel[1];
  __syncthreads();
  levels23_in_registers<kSamplePer, kThreads>(key, cnt, kSamplePer, b1, k_rem1, h, scan, sel);
  if (threadIdx.x == 0) guess[p] = sel[0];
}

template <class SRC, class = void>
struct has_begin_group : std::false_type {};
template <class SRC>
struct has_begin_group<SRC, std::void_t<decltype(&SRC::begin_group)>> : std::true_type {};

// Load pass.  Besides the buffer: the elements of the workgroup's tiles whose key is at least
// the partition's guess go to its short list, together and in index order, at the place one
// atomic add on the list length hands out; place and count are recorded per group of tiles, so
// the select pass can walk the list in index order whatever order the groups arrived in.
// The level-1 histogram takes those elements only (the bin of the k-th largest key and the rank
// inside it come out the same as long as the list holds k elements; every non-empty bin of every
// workgroup is one atomic on global memory, and with all elements counted those atomics were
// most of this pass on the server side); without a guess it takes all elements.
// LISTED (every partition has a guess): only the listed elements are counted, and their bins
// start at the guess's, so the LDS histogram is kNearBins bins from there (8 KB less LDS a
// workgroup: a fourth workgroup per compute unit on the server side); the rare key beyond them
// goes to the partition's histogram directly.
constexpr int kNearBins = 64;
// The group is taken as 8 rows of 1024 elements, 4 consecutive elements a thread and row: every
// 16-byte access of a wave to the gradient, the residual and the buffer covers whole cache lines
// and is marked non-temporal; everything goes through descriptors of the elements that exist
// (the rest read as zero and are not written).  All loads of the group are requested before the
// first is used.  Index order in the list is row, thread, element: a thread's place in its
// row comes from the wave's ballots, the places of the rows and waves from one scan of their
// 32 counts.
constexpr int kLoadRowElems = kThreads * 4;
constexpr int kLoadRows = kGroupElems / kLoadRowElems;
template <class SRC, bool LISTED>
__global__ __launch_bounds__(kThreads) void topk_load_hist1_kernel(Geo g, SRC src, float *buf, uint32_t *hist, uint32_t *state,
                                                                   const uint32_t *guess, uint32_t *groupcnt,
                                                                   uint32_t *cand_idx, uint32_t *cand_val) {
  __shared__ __align__(16) float lds[SRC::kLdsFloats];
  constexpr int kLocalBins = LISTED ? kNearBins : kBins1;
  constexpr int kWaves = kThreads / 64;
  static_assert(kLoadRows * kWaves <= 64, "one wave scans the counts of all rows and waves");
  __shared__ uint32_t h[kLocalBins];
  __shared__ uint32_t run_cnt[kLoadRows * kWaves];   // listed elements per row and wave, then how many come before them
  __shared__ uint32_t off_sh;
  const GroupOf w = group_of<kTpgLoad>(g, blockIdx.x);
  for (int b = threadIdx.x; b < kLocalBins; b += kThreads) h[b] = 0;
  src.begin(g, w.p, lds);
  __syncthreads();
  if (w.tile_lo >= w.tile_hi) return;  // (uniform) past the end of a shorter last partition
  const uint32_t j_lo = __builtin_amdgcn_readfirstlane(w.tile_lo * kTile);
  const uint32_t left = w.d - j_lo;
  const uint32_t valid = __builtin_amdgcn_readfirstlane(left < kGroupElems ? left : kGroupElems);
  const uint64_t base = uniform_off(g.part_base(w.p) + j_lo);
  const bool ef = src.res != nullptr;
  const TileBuf eb(ef ? src.res + base : nullptr, ef ? valid * 4 : 0);
  float v[kLoadRows][4];
  if constexpr (has_begin_group<SRC>::value) {
    // the residual's elements are requested first, so they are on their way while the group's
    // sum is formed
    u32x4 er[kLoadRows];
#pragma unroll
    for (int u = 0; u < kLoadRows; ++u) er[u] = eb.load16<kNonTemporal>(threadIdx.x * 16, u * kLoadRowElems * 4);
    src.begin_group(g, w.p, w.tile_lo / kTpgLoad, lds);
#pragma unroll
    for (int u = 0; u < kLoadRows; ++u) {
      const float4 sum = reinterpret_cast<const float4 *>(lds)[u * kThreads + threadIdx.x];
      const float sv[4] = {sum.x, sum.y, sum.z, sum.w};
      float e[4];
      widen4(er[u], e);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float mean = sv[c] * src.msgs.inv_n;
        const float delta = ef ? mean + e[c] : mean;
        v[u][c] = (uint32_t)(u * kLoadRowElems + c) + threadIdx.x * 4 < valid ? delta : 0.0f;
      }
    }
  } else {
    using T = typename SRC::Elem;
    const TileBuf gb(src.grad + base, valid * (uint32_t)sizeof(T));
    typename Vec4Of<T>::type gr[kLoadRows];
    u32x4 er[kLoadRows];
#pragma unroll
    for (int u = 0; u < kLoadRows; ++u) {
      gr[u] = tile_load4(gb, threadIdx.x * 4 * (uint32_t)sizeof(T), u * kLoadRowElems * (uint32_t)sizeof(T), (const T *)nullptr);
      er[u] = eb.load16<kNonTemporal>(threadIdx.x * 16, u * kLoadRowElems * 4);
    }
    if constexpr (sizeof(T) == 2) patch_last_half<kLoadRows, kLoadRowElems>(gb, valid, gr);
#pragma unroll
    for (int u = 0; u < kLoadRows; ++u) {
      float x[4], e[4];
      widen4(gr[u], x);
      widen4(er[u], e);
#pragma unroll
      for (int c = 0; c < 4; ++c) v[u][c] = ef ? x[c] + e[c] : x[c];
    }
  }
#pragma unroll
  for (int u = 0; u < kLoadRows; ++u)
    row_buf(buf + base, valid, u * kLoadRowElems, kLoadRowElems).store16<kNonTemporal>(as_u32x4(v[u][0], v[u][1], v[u][2], v[u][3]), threadIdx.x * 16);
  const uint32_t G = guess[w.p];
  uint32_t mask = 0;   // bit 4 u + c: element c of row u goes to the list
#pragma unroll
  for (int u = 0; u < kLoadRows; ++u) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if ((uint32_t)(u * kLoadRowElems + c) + threadIdx.x * 4 < valid) {
        const uint32_t key = key_of(v[u][c]);
        const bool listed = key >= G;
        if (LISTED) {
          if (listed) {
            const uint32_t rel = (key >> kShift1) - (G >> kShift1);
            if (rel < (uint32_t)kNearBins) atomicAdd(&h[rel], 1u);
            else atomicAdd(&hist[(uint64_t)w.p * kTopkHistWords + kHist1 + (key >> kShift1)], 1u);
          }
        } else {
          atomicAdd(&h[key >> kShift1], 1u);
        }
        mask |= (uint32_t)listed << (4 * u + c);
      }
    }
  }
  if (G != kNoGuess) {
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t before[kLoadRows];   // listed elements of the row in the wave's lanes below this one
#pragma unroll
    for (int u = 0; u < kLoadRows; ++u) {
      uint32_t mine = 0, all = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const unsigned long long m = __ballot((mask >> (4 * u + c)) & 1u);
        mine += __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        all += (uint32_t)__popcll(m);
      }
      before[u] = mine;
      if (lane == 0) run_cnt[u * kWaves + wave] = all;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
      const uint32_t x = threadIdx.x < (uint32_t)(kLoadRows * kWaves) ? run_cnt[threadIdx.x] : 0u;
      const uint32_t incl = wave_inclusive_scan_u32(x);
      if (threadIdx.x < (uint32_t)(kLoadRows * kWaves)) run_cnt[threadIdx.x] = incl - x;
      if (threadIdx.x == 63) {
        const uint32_t total = incl;
        const uint32_t off = total ? atomicAdd(&state[w.p * 8 + kStListLen], total) : 0u;
        off_sh = off;
        groupcnt[2 * blockIdx.x] = off;
        groupcnt[2 * blockIdx.x + 1] = total;
      }
    }
    __syncthreads();
    const uint64_t list = (uint64_t)w.p * kTopkListCap;
#pragma unroll
    for (int u = 0; u < kLoadRows; ++u) {
      uint32_t pos = off_sh + run_cnt[u * kWaves + wave] + before[u];
      const uint32_t j0 = j_lo + u * kLoadRowElems + threadIdx.x * 4;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if ((mask >> (4 * u + c)) & 1u) {
          if (pos < kTopkListCap) {
            cand_idx[list + pos] = j0 + c;
            cand_val[list + pos] = __float_as_uint(v[u][c]);
          }
          ++pos;
        }
      }
    }
  }
  __syncthreads();
  uint32_t *gh = hist + (uint64_t)w.p * kTopkHistWords + kHist1 + (LISTED ? (G >> kShift1) : 0u);
  for (int b = threadIdx.x; b < kLocalBins; b += kThreads)
    if (h[b]) atomicAdd(&gh[b], h[b]);   // (LISTED: bins past the last one hold nothing)
}

// The selection state of partition p after `LEVEL` levels in sel[0] (prefix / threshold key)
// and sel[1] (rank left among the keys that match it): level 1 from k, each further level
// from the state the pass before recorded.  The first workgroup of the partition records the
// new state for the next pass.
template <int LEVEL>
__device__ inline void selection_after(const Geo &g, const uint32_t *hist, uint32_t *state, uint32_t p, bool first,
                                       uint32_t *scan, uint32_t *sel) {
  const uint32_t *gh = hist + (uint64_t)p * kTopkHistWords;
  if (LEVEL == 1) pick_bin<kBins1, kBits1, kThreads>(gh + kHist1, (uint32_t)k_of_device(g, p), 0, scan, sel);
  else pick_bin<kBins23, kBits23, kThreads>(gh + (LEVEL == 2 ? kHist2 : kHist3), state[p * 8 + 2 * (LEVEL - 1) + kStKRem],
                                            state[p * 8 + 2 * (LEVEL - 1) + kStPrefix], scan, sel);
  // (state words 2L, 2L+1 hold the selection after level L; nobody reads the words this pass writes)
  if (first && threadIdx.x == 0) {
    state[p * 8 + 2 * LEVEL + kStPrefix] = sel[0];
    state[p * 8 + 2 * LEVEL + kStKRem] = sel[1];
  }
}

// Keys of 4 consecutive elements from j (a multiple of 4) of a partition of d elements;
// *n receives how many of them exist.
__device__ inline void keys4(const float *part, uint32_t j, uint32_t d, uint32_t key[4], uint32_t *n) {
  if (j + 4 <= d) {
    const float4 f = *reinterpret_cast<const float4 *>(part + j);
    key[0] = key_of(f.x); key[1] = key_of(f.y); key[2] = key_of(f.z); key[3] = key_of(f.w);
    *n = 4;
  } else {
    *n = j < d ? d - j : 0u;
#pragma unroll
    for (int c = 0; c < 4; ++c) key[c] = j + c < d ? key_of(part[j + c]) : 0u;
  }
}

// The long-form kernels take their groups of tiles in a loop, so that they can be launched with
// a small grid behind the short-list form (`gated`: only partitions left to the long form).

// LEVEL 2: keys whose top 11 bits equal the prefix, histogram of the next 10 bits.
// LEVEL 3: keys whose top 21 bits equal the prefix, histogram of the last 10 bits.
// LEVEL 1 (long form behind the short-list form only): the keys below the partition's guess,
// which the load pass left out of the level-1 histogram.
template <int LEVEL>
__device__ inline void topk_hist_body(const Geo &g, const float *buf, uint32_t *hist, uint32_t *state, uint32_t n_groups,
                                      int gated, const uint32_t *guess = nullptr) {
  constexpr int kBins = LEVEL == 1 ? kBins1 : kBins23;
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t scan[kThreads];
  __shared__ uint32_t sel[2];
  for (uint32_t blk = blockIdx.x; blk < n_groups; blk += gridDim.x) {
    const GroupOf w = group_of<LEVEL == 2 ? kTpgHist2 : kTpgHist3>(g, blk);
    if (gated && !long_form(state, w.p)) continue;
    for (int b = threadIdx.x; b < kBins; b += kThreads) h[b] = 0;
    if constexpr (LEVEL == 1) {
      const uint32_t G = guess[w.p];
      __syncthreads();
      const float *part1 = buf + g.part_base(w.p);
      for (uint32_t tile = w.tile_lo; tile < w.tile_hi; ++tile) {
#pragma unroll
        for (int c = 0; c < kTile / (kThreads * 4); ++c) {
          uint32_t key[4], n;
          keys4(part1, tile * kTile + c * (kThreads * 4) + threadIdx.x * 4, w.d, key, &n);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if ((uint32_t)e < n && key[e] < G) atomicAdd(&h[key[e] >> kShift1], 1u);
        }
      }
      __syncthreads();
      uint32_t *gh1 = hist + (uint64_t)w.p * kTopkHistWords + kHist1;
      for (int b = threadIdx.x; b < kBins; b += kThreads)
        if (h[b]) atomicAdd(&gh1[b], h[b]);
      __syncthreads();
      continue;
    }
    selection_after<(LEVEL > 1 ? LEVEL - 1 : 1)>(g, hist, state, w.p, w.tile_lo == 0, scan, sel);
    const uint32_t prefix = sel[0];
    constexpr int kHiShift = LEVEL == 2 ? kShift1 : kShift2;
    constexpr int kLoShift = LEVEL == 2 ? kShift2 : 0;
    const float *part = buf + g.part_base(w.p);
    for (uint32_t tile = w.tile_lo; tile < w.tile_hi; ++tile) {
#pragma unroll
      for (int c = 0; c < kTile / (kThreads * 4); ++c) {
        uint32_t key[4], n;
        keys4(part, tile * kTile + c * (kThreads * 4) + threadIdx.x * 4, w.d, key, &n);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if ((uint32_t)e < n && (key[e] >> kHiShift) == prefix) atomicAdd(&h[(key[e] >> kLoShift) & (kBins23 - 1)], 1u);
      }
    }
    __syncthreads();
    uint32_t *gh = hist + (uint64_t)w.p * kTopkHistWords + (LEVEL == 2 ? kHist2 : kHist3);
    for (int b = threadIdx.x; b < kBins23; b += kThreads)
      if (h[b]) atomicAdd(&gh[b], h[b]);
    __syncthreads();
  }
}

template <int LEVEL>
__global__ __launch_bounds__(kThreads) void topk_hist_kernel(Geo g, const float *buf, uint32_t *hist, uint32_t *state,
                                                             uint32_t n_groups) {
  topk_hist_body<LEVEL>(g, buf, hist, state, n_groups, 0);
}

// Per tile: number of keys above the threshold and equal to it.  The first workgroup of a
// partition also records the threshold key T and the number r of keys equal to T that are
// kept, for the compaction.
__device__ inline void topk_count_body(const Geo &g, const float *buf, const uint32_t *hist, uint32_t *state,
                                       uint32_t *tilecnt, uint32_t n_groups, int gated) {
  __shared__ uint32_t red[2][kThreads / 64];
  __shared__ uint32_t scan[kThreads];
  __shared__ uint32_t sel[2];
  for (uint32_t blk = blockIdx.x; blk < n_groups; blk += gridDim.x) {
    const GroupOf w = group_of<kTpgCount>(g, blk);
    if (gated && !long_form(state, w.p)) continue;
    selection_after<3>(g, hist, state, w.p, w.tile_lo == 0, scan, sel);
    const uint32_t T = sel[0];
    const float *part = buf + g.part_base(w.p);
    for (uint32_t tile = w.tile_lo; tile < w.tile_hi; ++tile) {
      uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
      for (int c = 0; c < kTile / (kThreads * 4); ++c) {
        uint32_t key[4], n;
        keys4(part, tile * kTile + c * (kThreads * 4) + threadIdx.x * 4, w.d, key, &n);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          n_gt += (uint32_t)e < n && key[e] > T;
          n_eq += (uint32_t)e < n && key[e] == T;
        }
      }
      n_gt = wave_sum_u32(n_gt);
      n_eq = wave_sum_u32(n_eq);
      __syncthreads();
      if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = n_gt;
        red[1][threadIdx.x >> 6] = n_eq;
      }
      __syncthreads();
      if (threadIdx.x == 0) {
        uint32_t a = 0, b = 0;
        for (int v = 0; v < kThreads / 64; ++v) { a += red[0][v]; b += red[1][v]; }
        const uint64_t t = (uint64_t)w.p * g.tiles_per_part + tile;
        tilecnt[2 * t] = a;
        tilecnt[2 * t + 1] = b;
      }
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(kThreads) void topk_count_kernel(Geo g, const float *buf, const uint32_t *hist,
                                                              uint32_t *state, uint32_t *tilecnt, uint32_t n_groups) {
  topk_count_body(g, buf, hist, state, tilecnt, n_groups, 0);
}

// Header of partition p's record; for the half-value form also the zeros the format wants from
// value k to the end of its last group of four words.
template <bool HALF>
__device__ inline void topk_write_header(const Geo &g, uint32_t p, uint8_t *payload) {
  uint8_t *rec0 = payload + (uint64_t)p * g.stride;
  uint32_t *hdr = reinterpret_cast<uint32_t *>(rec0);
  const uint32_t k = (uint32_t)k_of_device(g, p);
  hdr[0] = k;
  hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
  if (HALF) {
    uint16_t *val16 = reinterpret_cast<uint16_t *>(rec0 + kHeaderBytes + 4 * ru4(g.k_cap));
    for (uint32_t t = k; t < 2 * (uint32_t)ru4(cdiv(k, 2)); ++t) val16[t] = 0;
  }
}

// Entry `pos` of partition p's record: element j with value v; the buffer keeps 0 there, or
// what rounding to half dropped.
template <bool HALF>
__device__ inline void topk_write_entry(const Geo &g, uint8_t *rec, uint32_t pos, uint32_t j, float v, float *buf_part,
                                        int zero_selected) {
  uint32_t *idx = reinterpret_cast<uint32_t *>(rec + kHeaderBytes);
  float *val = reinterpret_cast<float *>(rec + kHeaderBytes + 4 * ru4(g.k_cap));
  idx[pos] = j;
  if (HALF) {
    const __half h = __float2half_rn(v);
    reinterpret_cast<__half *>(val)[pos] = h;
    if (zero_selected) buf_part[j] = v - __half2float(h);
  } else {
    val[pos] = v;
    if (zero_selected) buf_part[j] = 0.0f;
  }
}

// Select pass: the radix select on the short list of one partition, then the record.  The list
// in index order is the groups' runs in group order.  Wave w owns a stretch of consecutive
// entries of that order, lane l of it the entries l, l + 64, ... of the stretch (neighbouring
// lanes read neighbouring words), and keeps their values in registers throughout; positions in
// the record follow from the counts of the waves before, of the rounds before and of the lanes
// before.  A list shorter than k or longer than its room leaves the partition to the long form.
template <bool HALF>
__global__ __launch_bounds__(kSelThreads) void topk_list_select_kernel(Geo g, float *buf, uint32_t *state,
                                                                       const uint32_t *hist, const uint32_t *groupcnt,
                                                                       const uint32_t *cand_idx, const uint32_t *cand_val,
                                                                       uint8_t *payload, int zero_selected) {
  constexpr int kWaves = kSelThreads / 64;
  __shared__ uint32_t h[kBins23];
  __shared__ uint32_t vstart[kSelThreads + 1];  // entries of the list before group t's run
  __shared__ uint32_t goff[kSelThreads];        // where group t's run sits in the list
  __shared__ uint32_t scan[kWaves];
  __shared__ uint32_t sel[2];
  __shared__ uint32_t wave_gt[kWaves], wave_eq[kWaves];
  const uint32_t p = blockIdx.x;
  const uint32_t n = __builtin_amdgcn_readfirstlane(state[p * 8 + kStListLen]);
  const uint32_t k = (uint32_t)k_of_device(g, p);
  if (n < k || n > kTopkListCap) {
    if (threadIdx.x == 0) state[p * 8 + kStLong] = 1;
    return;
  }
  const uint32_t groups_per_part = (uint32_t)cdiv(g.tiles_per_part, kTpgLoad);            // at most kSelThreads
  const uint32_t n_groups_p = (uint32_t)cdiv(cdiv(g.part_size(p), kTile), kTpgLoad);
  {
    const uint64_t t = (uint64_t)p * groups_per_part + threadIdx.x;
    const uint32_t c = threadIdx.x < n_groups_p ? groupcnt[2 * t + 1] : 0u;
    goff[threadIdx.x] = threadIdx.x < n_groups_p ? groupcnt[2 * t] : 0u;
    uint32_t total;
    vstart[threadIdx.x] = block_exclusive_scan<kSelThreads>(c, scan, &total);
    if (threadIdx.x == 0) vstart[kSelThreads] = n;
  }
  __syncthreads();
  const uint32_t rounds = (uint32_t)cdiv(n, kSelThreads);  // at most kSelPer
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint32_t first = wave * rounds * 64 + lane;        // the thread's entries: first + 64 i, i < rounds
  const uint32_t cnt = first < n ? (uint32_t)cdiv(n - first, 64) < rounds ? (uint32_t)cdiv(n - first, 64) : rounds : 0u;
  // the group whose run holds the first entry: the last one that starts at or before it
  uint32_t group0 = 0;
  if (cnt) {
    uint32_t a = 0, b = kSelThreads;  // vstart[a] <= first < vstart[b] (vstart[kSelThreads] = n > first)
    while (b - a > 1) {
      const uint32_t m = (a + b) >> 1;
      if (vstart[m] <= first) a = m; else b = m;
    }
    group0 = a;
  }
  const uint64_t list = (uint64_t)p * kTopkListCap;
  // Place in the list of an entry of the order.  The run of the current group is kept in
  // registers; LDS is read only when the walk crosses into a later group.
  struct Walk {
    uint32_t group, begin, end, off;  // entries [begin, end) of the order sit at off..
  };
  auto walk_to = [&](Walk &w, uint32_t entry) {
    while (entry >= w.end) {
      ++w.group;
      w.begin = w.end;
      w.end = vstart[w.group + 1];
      w.off = goff[w.group];
    }
    return w.off + (entry - w.begin);
  };
  const Walk walk0{group0, vstart[group0], vstart[group0 + 1], goff[group0]};
  // every load is issued whether or not the entry exists (entry 0 of the list stands in), so
  // none of them is waited for before the last is on its way
  uint32_t bits[kSelPer], where[kSelPer];   // value and index of the thread's entries
  auto key = [&](int i) { return bits[i] & 0x7fffffffu; };
  {
    Walk w = walk0;
#pragma unroll
    for (int i = 0; i < kSelPer; ++i) {
      bits[i] = 0;
      where[i] = 0;
      if ((uint32_t)i >= rounds) continue;   // (the same for all threads)
      const uint32_t at = (uint32_t)i < cnt ? walk_to(w, first + 64 * i) : 0u;
      bits[i] = cand_val[list + at];
      where[i] = cand_idx[list + at];
    }
  }
  // level 1 is known from the histogram of the whole partition
  pick_bin<kBins1, kBits1, kSelThreads>(hist + (uint64_t)p * kTopkHistWords + kHist1, k, 0, scan, sel);
  const uint32_t b1 = sel[0], k_rem1 = sel[1];
  __syncthreads();
  levels23_in_registers<kSelPer, kSelThreads>(bits, cnt, rounds, b1, k_rem1, h, scan, sel);
  const uint32_t T = sel[0], r = sel[1];
  if (threadIdx.x == 0) topk_write_header<HALF>(g, p, payload);
  // keys above T and equal to T in the waves before this one
  {
    uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
    for (int i = 0; i < kSelPer; ++i) {
      if ((uint32_t)i >= rounds) break;
      n_gt += (uint32_t)i < cnt && key(i) > T;
      n_eq += (uint32_t)i < cnt && key(i) == T;
    }
    n_gt = wave_sum_u32(n_gt);
    n_eq = wave_sum_u32(n_eq);
    if (lane == 0) { wave_gt[wave] = n_gt; wave_eq[wave] = n_eq; }
  }
  __syncthreads();
  uint32_t gt_base = 0, eq_base = 0;
#pragma unroll
  for (int v = 0; v < kWaves; ++v) {
    gt_base += (uint32_t)v < wave ? wave_gt[v] : 0u;
    eq_base += (uint32_t)v < wave ? wave_eq[v] : 0u;
  }
  uint8_t *rec = payload + (uint64_t)p * g.stride;
  float *buf_part = buf + g.part_base(p);
  const uint64_t lanes_before = (1ull << lane) - 1ull;
  // which entries are kept and where they go
#pragma unroll
  for (int i = 0; i < kSelPer; ++i) {
    if ((uint32_t)i < rounds) {   // (the same for all threads)
      const bool valid = (uint32_t)i < cnt;
      const uint64_t gtm = __ballot(valid && key(i) > T), eqm = __ballot(valid && key(i) == T);
      const uint32_t gt_before = gt_base + __popcll(gtm & lanes_before);
      const uint32_t eq_before = eq_base + __popcll(eqm & lanes_before);
      const bool t = valid && (key(i) > T || (key(i) == T && eq_before < r));
      gt_base += __popcll(gtm);
      eq_base += __popcll(eqm);
      if (t) topk_write_entry<HALF>(g, rec, gt_before + (eq_before < r ? eq_before : r), where[i], __uint_as_float(bits[i]), buf_part, zero_selected);
    }
  }
}

// Ordered compaction of the long form.  Thread t of a tile owns 16 consecutive elements, so
// positions follow from an exclusive scan over threads, on top of the counts of the partition's
// earlier tiles (at most a few hundred numbers, summed by every workgroup for itself).  The
// workgroup of the first tile writes the record's header.
// HALF: values are sent as halves (round to nearest even) and a kept slot of the buffer keeps
// what the rounding dropped instead of 0.
template <bool HALF>
__device__ inline void topk_emit_body(const Geo &g, float *buf, const uint32_t *state, const uint32_t *tilecnt,
                                      uint8_t *payload, int zero_selected, uint32_t n_items, int gated) {
  __shared__ uint32_t scan[kThreads];
  __shared__ uint32_t before[2][kThreads / 64];
  constexpr int kPer = kTile / kThreads;
  for (uint32_t blk = blockIdx.x; blk < n_items; blk += gridDim.x) {
    const uint32_t p = blk / g.tiles_per_part;
    const uint32_t tile = blk % g.tiles_per_part;
    if (gated && !long_form(state, p)) continue;
    const uint32_t d = g.part_size(p);
    if (tile >= (uint32_t)cdiv(d, kTile)) continue;
    const uint32_t T = state[p * 8 + 6 + kStPrefix];   // the selection after level 3
    const uint32_t r = state[p * 8 + 6 + kStKRem];
    {
      const uint32_t *tc = tilecnt + 2ull * p * g.tiles_per_part;
      uint32_t a = 0, b = 0;
      for (uint32_t t = threadIdx.x; t < tile; t += kThreads) { a += tc[2 * t]; b += tc[2 * t + 1]; }
      a = wave_sum_u32(a);
      b = wave_sum_u32(b);
      if ((threadIdx.x & 63) == 0) { before[0][threadIdx.x >> 6] = a; before[1][threadIdx.x >> 6] = b; }
      __syncthreads();
    }
    uint32_t gt_before = 0, eq_before = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) { gt_before += before[0][w]; eq_before += before[1][w]; }
    if (tile == 0 && threadIdx.x == 0) topk_write_header<HALF>(g, p, payload);
    const uint64_t base = g.part_base(p);
    const uint32_t j0 = tile * kTile + threadIdx.x * kPer;
    float v[kPer];
    uint32_t n_gt = 0, n_eq = 0;
    if (j0 + kPer <= d) {
      // the thread's 16 elements start at a multiple of 16: four 16-byte loads
      const float4 *src4 = reinterpret_cast<const float4 *>(buf + base + j0);
#pragma unroll
      for (int q = 0; q < kPer / 4; ++q) {
        const float4 f = src4[q];
        v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < kPer; ++i) v[i] = j0 + i < d ? buf[base + j0 + i] : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      uint32_t j = j0 + i;
      uint32_t key = key_of(v[i]);
      n_gt += (j < d) && key > T;
      n_eq += (j < d) && key == T;
    }
    // one scan for both counts: a tile has 4096 elements, so each fits 16 bits
    uint32_t tot;
    const uint32_t ex_both = block_exclusive_scan<kThreads>(n_gt | (n_eq << 16), scan, &tot);
    const uint32_t ex_gt = ex_both & 0xffffu, ex_eq = ex_both >> 16;
    // ties admitted before this tile / before this thread
    const uint32_t ties_tile = eq_before < r ? eq_before : r;
    uint32_t eq_rank = eq_before + ex_eq;                 // rank of this thread's first tie
    const uint32_t ties_thread = (eq_rank < r ? eq_rank : r) - ties_tile;
    uint32_t pos = gt_before + ties_tile + ex_gt + ties_thread;
    uint8_t *rec = payload + (uint64_t)p * g.stride;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      uint32_t j = j0 + i;
      if (j >= d) continue;
      uint32_t key = key_of(v[i]);
      bool take = key > T;
      if (key == T) {
        take = eq_rank < r;
        ++eq_rank;
      }
      if (take) {
        topk_write_entry<HALF>(g, rec, pos, j, v[i], buf + base, zero_selected);
        ++pos;
      }
    }
    __syncthreads();
  }
}

template <bool HALF>
__global__ __launch_bounds__(kThreads) void topk_emit_kernel(Geo g, float *buf, const uint32_t *state,
                                                             const uint32_t *tilecnt, uint8_t *payload,
                                                             int zero_selected, uint32_t n_items) {
  topk_emit_body<HALF>(g, buf, state, tilecnt, payload, zero_selected, n_items, 0);
}

// All workgroups of a grid that is resident as a whole meet here: what they wrote before is
// visible to all of them after (release fence, one arrival each on a counter, acquire fence).
// The wait is bounded like those of cluster.hpp: a workgroup that gives up sets the status word.
__device__ inline void topk_grid_barrier(uint32_t *counter, uint32_t round, uint32_t *status) {
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    atomicAdd(counter, 1u);
    const uint32_t target = round * gridDim.x;
    int spins = 0;
    while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      if (++spins > kSpinLimit) {
        atomicOr(status, 1u);
        break;
      }
      __builtin_amdgcn_s_sleep(16);
    }
  }
  __syncthreads();
  __threadfence();
}

// The long form behind the short-list form, as one launch: returns at once unless some
// partition was left to it (the usual case: one launch and one read instead of four of each),
// else completes their level-1 histograms and runs the four passes for those partitions, with
// the whole grid meeting in between.
// The grid is resident as a whole (the host sizes it by occupancy).  `counter`: zero at launch.
template <bool HALF>
__global__ __launch_bounds__(kThreads) void topk_long_form_kernel(Geo g, float *buf, uint32_t *hist, uint32_t *state,
                                                                  uint32_t *tilecnt, uint8_t *payload, int zero_selected,
                                                                  uint32_t n2, uint32_t n3, uint32_t nc, uint32_t ne,
                                                                  const uint32_t *guess, uint32_t *counter, uint32_t *status) {
  __shared__ uint32_t any;
  if (threadIdx.x == 0) any = 0;
  __syncthreads();
  for (uint32_t p = threadIdx.x; p < g.P; p += kThreads)
    if (state[p * 8 + kStLong]) any = 1;
  __syncthreads();
  if (!any) return;   // (the same answer in every workgroup: the flags were written by the kernel before)
  topk_hist_body<1>(g, buf, hist, state, n3, 1, guess);   // (groups of one tile, as level 3)
  topk_grid_barrier(counter, 1, status);
  topk_hist_body<2>(g, buf, hist, state, n2, 1);
  topk_grid_barrier(counter, 2, status);
  topk_hist_body<3>(g, buf, hist, state, n3, 1);
  topk_grid_barrier(counter, 3, status);
  topk_count_body(g, buf, hist, state, tilecnt, nc, 1);
  topk_grid_barrier(counter, 4, status);
  topk_emit_body<HALF>(g, buf, state, tilecnt, payload, zero_selected, ne, 1);
}

// With tiles of 1 << tile_shift elements, T of them to a full partition:
// table[p * (T + 1) + tile] = the first entry of partition p's record that lies in tile `tile`
// or after it; entry T = the number of entries.
hipError_t topk_tile_starts(const Geo &g, const uint8_t *payload, bool half, uint32_t *table, uint32_t tile_shift,
                            hipStream_t stream) {
  TopkMsgs m{};
  m.msgs.ptr[0] = payload;
  m.msgs.n = 1;
  m.groups_per_part = (uint32_t)cdiv(g.part_elems, 1ull << tile_shift);
  m.k_cap = g.k_cap;
  m.stride = g.stride;
  m.half = half ? 1 : 0;
  m.group_shift = tile_shift;
  topk_starts_kernel<<<dim3((uint32_t)cdiv(g.k_cap + 1, kThreads), g.P, 1), kThreads, 0, stream>>>(g, m, table, nullptr);
  return hipGetLastError();
}

hipError_t topk_encode(const Geo &g, const bpc_params_t &prm, const bpc_params_t *, const Source &src,
                       uint8_t *payload, const Workspace &ws, hipStream_t stream) {
  uint32_t *hist = ws.at<uint32_t>(ws.lay.hist);
  uint32_t *state = ws.at<uint32_t>(ws.lay.state);
  uint32_t *guess = ws.at<uint32_t>(ws.lay.guess);
  uint32_t *tilecnt = ws.at<uint32_t>(ws.lay.tilecnt);   // also the per-group (place, count) of the short lists
  float *dense = ws.at<float>(ws.lay.dense);
  // the vector being compressed ends up in the residual buffer (error feedback) or the workspace
  float *buf = src.residual ? src.residual : dense;
  const bool half = prm.kind == BPC_TOPK16;
  uint32_t *cand_idx = ws.at<uint32_t>(ws.lay.cand);
  uint32_t *cand_val = cand_idx + (size_t)kTopkListCap * g.P;
  // the short-list form wants room for the k winners and as many again; the select pass gives
  // each group of tiles of a partition one thread
  // (and the long form behind it is one resident kernel: its grid comes from the occupancy query)
  const void *long_fn = half ? reinterpret_cast<const void *>(&topk_long_form_kernel<true>)
                             : reinterpret_cast<const void *>(&topk_long_form_kernel<false>);
  static PerDevice cache[2];
  int capacity[2] = {0, 0};
  capacity[half] = cache[half].get([&] { return cluster_capacity(long_fn, kThreads, 0); });
  const int short_list = g.k_cap <= kTopkListCap / 2 && cdiv(g.tiles_per_part, kTpgLoad) <= (uint64_t)kSelThreads &&
                         capacity[half] > 0;
  const uint32_t sample_grid = g.P > 64 ? g.P : 64, load_grid = group_count(g, kTpgLoad);
  auto first_two = [&](auto s_sample, auto s_load) {
    topk_sample_kernel<<<sample_grid, kThreads, 0, stream>>>(g, s_sample, hist, state, guess, short_list, ws.status());
    using Load = decltype(s_load);
    if (short_list) topk_load_hist1_kernel<Load, true><<<load_grid, kThreads, 0, stream>>>(g, s_load, buf, hist, state, guess, tilecnt, cand_idx, cand_val);
    else topk_load_hist1_kernel<Load, false><<<load_grid, kThreads, 0, stream>>>(g, s_load, buf, hist, state, guess, tilecnt, cand_idx, cand_val);
  };
  if (src.grad) {
    if (src.dtype == BPC_F16) {
      GradSource<__half> s{(const __half *)src.grad, src.residual};
      first_two(s, s);
    } else {
      GradSource<float> s{(const float *)src.grad, src.residual};
      first_two(s, s);
    }
  } else {
    // server: Delta straight from the n messages (they are taken to have the format of `prm`)
    uint32_t *starts = ws.at<uint32_t>(ws.lay.starts);
    const TopkMsgs m{src.msgs, src.residual, starts, (uint32_t)cdiv(g.tiles_per_part, kTpgLoad), g.k_cap, g.stride, half ? 1 : 0, 13};
    float *samp = ws.at<float>(ws.lay.samp);
    const hipError_t e = fill_zero(samp, sizeof(float) * kSample * g.P, stream);
    if (e != hipSuccess) return e;
    topk_starts_kernel<<<dim3((uint32_t)cdiv(g.k_cap + 1, kThreads), g.P, src.msgs.n), kThreads, 0, stream>>>(g, m, starts, samp);
    first_two(TopkMsgsSampleSource{m, samp}, TopkMsgsGroupSource{m});
  }
  const int zero_selected = src.residual != nullptr;
  if (short_list) {
    if (half) topk_list_select_kernel<true><<<g.P, kSelThreads, 0, stream>>>(g, buf, state, hist, tilecnt, cand_idx, cand_val, payload, zero_selected);
    else topk_list_select_kernel<false><<<g.P, kSelThreads, 0, stream>>>(g, buf, state, hist, tilecnt, cand_idx, cand_val, payload, zero_selected);
  }
  const uint32_t n2 = group_count(g, kTpgHist2), n3 = group_count(g, kTpgHist3), nc = group_count(g, kTpgCount);
  const uint32_t ne = g.P * g.tiles_per_part;
  if (short_list) {
    // the long form for the partitions the short list could not take: one resident kernel
    const uint32_t grid = (uint32_t)capacity[half] < kGatedGrid ? (uint32_t)capacity[half] : kGatedGrid;
    uint32_t *counter = state + 8ull * g.P;
    uint32_t *status = ws.status();
    hipError_t e = cluster_launch_begin(stream);
    if (e != hipSuccess) return e;
    if (half) topk_long_form_kernel<true><<<grid, kThreads, 0, stream>>>(g, buf, hist, state, tilecnt, payload, zero_selected, n2, n3, nc, ne, guess, counter, status);
    else topk_long_form_kernel<false><<<grid, kThreads, 0, stream>>>(g, buf, hist, state, tilecnt, payload, zero_selected, n2, n3, nc, ne, guess, counter, status);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return cluster_launch_end(stream);
  }
  topk_hist_kernel<2><<<n2, kThreads, 0, stream>>>(g, buf, hist, state, n2);
  topk_hist_kernel<3><<<n3, kThreads, 0, stream>>>(g, buf, hist, state, n3);
  topk_count_kernel<<<nc, kThreads, 0, stream>>>(g, buf, hist, state, tilecnt, nc);
  if (half) topk_emit_kernel<true><<<ne, kThreads, 0, stream>>>(g, buf, state, tilecnt, payload, zero_selected, ne);
  else topk_emit_kernel<false><<<ne, kThreads, 0, stream>>>(g, buf, state, tilecnt, payload, zero_selected, ne);
  return hipGetLastError();
}

}  // namespace bpc
