// Top-k compressor (Section 3.2: of a gradient only its k entries of largest magnitude travel)
// with the residual update of Algorithm 4 in its fused form (Section 4.2, operator fusion: the
// residual is the vector itself with the k sent slots set to zero).
//
// Selection is an exact three-level radix select on the 31-bit magnitude key
// bits(v) & 0x7fffffff (11 + 10 + 10 bits), followed by an ordered compaction in which
// elements equal to the threshold key are admitted lowest index first.  Five passes:
//   load+hist1 : v_j from the source -> dense buffer; histogram of key >> 20
//   hist2      : bucket of level 1 that holds the k-th largest key, histogram inside it
//   hist3      : the same one level down
//   count      : threshold key T and the number r of elements with key == T that are kept;
//                per tile, how many keys are > T and == T
//   emit       : (idx, val) in ascending index order; kept slots of the buffer zeroed
// Each pass works out the selection so far from the histograms of the passes before it (every
// workgroup for itself), so no launches sit between the passes.
#include "sources.hpp"

namespace bpc {

constexpr int kBins1 = 2048, kBins23 = 1024;
constexpr int kHistPerPart = 4096;  // 2048 + 1024 + 1024
// A workgroup of the histogram / count passes handles a few consecutive tiles of one partition
// (template parameter TPG): its LDS histogram is merged into the partition's with one atomic
// per non-empty bin, so more tiles a workgroup mean fewer of those (they were the larger part
// of the level-2 pass), while fewer, longer workgroups hide less latency (8 tiles a workgroup
// doubled the time of the passes that only read).
constexpr int kTpgLoad = 2, kTpgHist2 = 4, kTpgHist3 = 1, kTpgCount = 1;

__device__ inline uint32_t key_of(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// state words per partition: words 2L, 2L + 1 hold (prefix, rank left) after level L = 1..3
enum { kStPrefix = 0, kStKRem = 1 };

struct GroupOf {
  uint32_t p, tile_lo, tile_hi, d;
};
template <int TPG>
__device__ inline GroupOf group_of(const Geo &g) {
  constexpr uint32_t kTilesPerGroup = TPG;
  const uint32_t groups_per_part = (uint32_t)cdiv(g.tiles_per_part, kTilesPerGroup);
  GroupOf r;
  r.p = blockIdx.x / groups_per_part;
  r.d = g.part_size(r.p);
  const uint32_t n_tiles = (uint32_t)cdiv(r.d, kTile);
  r.tile_lo = (blockIdx.x % groups_per_part) * kTilesPerGroup;
  r.tile_hi = r.tile_lo + kTilesPerGroup < n_tiles ? r.tile_lo + kTilesPerGroup : n_tiles;
  return r;
}
inline uint32_t group_grid(const Geo &g, int tpg) { return g.P * (uint32_t)cdiv(g.tiles_per_part, tpg); }

template <class SRC>
__global__ __launch_bounds__(kThreads) void topk_load_hist1_kernel(Geo g, SRC src, float *buf, uint32_t *hist) {
  __shared__ float lds[SRC::kLdsFloats];
  __shared__ uint32_t h[kBins1];
  const GroupOf w = group_of<kTpgLoad>(g);
  for (int b = threadIdx.x; b < kBins1; b += kThreads) h[b] = 0;
  src.begin(g, w.p, lds);
  __syncthreads();
  const uint64_t base = g.part_base(w.p);
  for (uint32_t tile = w.tile_lo; tile < w.tile_hi; ++tile) {
#pragma unroll
    for (int c = 0; c < kTile / kThreads; ++c) {
      uint32_t j = tile * kTile + c * kThreads + threadIdx.x;
      if (j < w.d) {
        float v = src.at(g, w.p, j, lds);
        buf[base + j] = v;
        atomicAdd(&h[key_of(v) >> 20], 1u);
      }
    }
  }
  __syncthreads();
  uint32_t *gh = hist + (uint64_t)w.p * kHistPerPart;
  for (int b = threadIdx.x; b < kBins1; b += kThreads)
    if (h[b]) atomicAdd(&gh[b], h[b]);
}

// All threads of a workgroup: walk the level's histogram of partition p from the highest bin
// down and find the bin b with  count(bins above b) < k_rem <= count(bins above b) + count(b).
// Returns the extended prefix and the rank left inside that bin through `sel` (LDS, 2 words).
// Every workgroup of the pass that follows a histogram pass does this for itself (a few
// microseconds of L2 reads) instead of a launch of its own in between.
template <int LEVEL>
__device__ inline void pick_bin(const uint32_t *hist, uint32_t p, uint32_t k_rem, uint32_t prefix, uint32_t *scan,
                                uint32_t *sel) {
  constexpr int kBins = LEVEL == 1 ? kBins1 : kBins23;
  constexpr int kPer = kBins / kThreads;
  const uint32_t *gh = hist + (uint64_t)p * kHistPerPart + (LEVEL == 1 ? 0 : LEVEL == 2 ? kBins1 : kBins1 + kBins23);
  // thread t owns bins [kBins-1 - t*kPer - (kPer-1), kBins-1 - t*kPer], highest first
  uint32_t cnt[kPer];
  uint32_t local = 0;
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    cnt[i] = gh[kBins - 1 - (threadIdx.x * kPer + i)];
    local += cnt[i];
  }
  uint32_t total;
  uint32_t above = block_exclusive_scan<kThreads>(local, scan, &total);
  if (above < k_rem && k_rem <= above + local) {
    uint32_t run = above;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      if (run < k_rem && k_rem <= run + cnt[i]) {
        uint32_t bin = kBins - 1 - (threadIdx.x * kPer + i);
        sel[0] = LEVEL == 1 ? bin : ((prefix << 10) | bin);
        sel[1] = k_rem - run;
      }
      run += cnt[i];
    }
  }
  __syncthreads();
}

// The selection state of partition p after `LEVEL` levels in sel[0] (prefix / threshold key)
// and sel[1] (rank left among the keys that match it): level 1 from k, each further level
// from the state the pass before recorded.  The first workgroup of the partition records the
// new state for the next pass.
template <int LEVEL>
__device__ inline void selection_after(const Geo &g, const uint32_t *hist, uint32_t *state, uint32_t p, bool first,
                                       uint32_t *scan, uint32_t *sel) {
  if (LEVEL == 1) pick_bin<1>(hist, p, (uint32_t)k_of_device(g, p), 0, scan, sel);
  else pick_bin<LEVEL>(hist, p, state[p * 8 + 2 * (LEVEL - 1) + kStKRem], state[p * 8 + 2 * (LEVEL - 1) + kStPrefix], scan, sel);
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

// LEVEL 2: keys whose top 11 bits equal the prefix, histogram of the next 10 bits.
// LEVEL 3: keys whose top 21 bits equal the prefix, histogram of the last 10 bits.
template <int LEVEL>
__global__ __launch_bounds__(kThreads) void topk_hist_kernel(Geo g, const float *buf, uint32_t *hist, uint32_t *state) {
  __shared__ uint32_t h[kBins23];
  __shared__ uint32_t scan[kThreads];
  __shared__ uint32_t sel[2];
  const GroupOf w = group_of<LEVEL == 2 ? kTpgHist2 : kTpgHist3>(g);
  for (int b = threadIdx.x; b < kBins23; b += kThreads) h[b] = 0;
  selection_after<LEVEL - 1>(g, hist, state, w.p, w.tile_lo == 0, scan, sel);
  const uint32_t prefix = sel[0];
  constexpr int kHiShift = LEVEL == 2 ? 20 : 10;
  constexpr int kLoShift = LEVEL == 2 ? 10 : 0;
  const float *part = buf + g.part_base(w.p);
  for (uint32_t tile = w.tile_lo; tile < w.tile_hi; ++tile) {
#pragma unroll
    for (int c = 0; c < kTile / (kThreads * 4); ++c) {
      uint32_t key[4], n;
      keys4(part, tile * kTile + c * (kThreads * 4) + threadIdx.x * 4, w.d, key, &n);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if ((uint32_t)e < n && (key[e] >> kHiShift) == prefix) atomicAdd(&h[(key[e] >> kLoShift) & 1023u], 1u);
    }
  }
  __syncthreads();
  uint32_t *gh = hist + (uint64_t)w.p * kHistPerPart + (LEVEL == 2 ? kBins1 : kBins1 + kBins23);
  for (int b = threadIdx.x; b < kBins23; b += kThreads)
    if (h[b]) atomicAdd(&gh[b], h[b]);
}

// Per tile: number of keys above the threshold and equal to it.  The first workgroup of a
// partition also records the threshold key T and the number r of keys equal to T that are
// kept, for the compaction.
__global__ __launch_bounds__(kThreads) void topk_count_kernel(Geo g, const float *buf, const uint32_t *hist,
                                                              uint32_t *state, uint32_t *tilecnt) {
  __shared__ uint32_t red[2][kThreads / 64];
  __shared__ uint32_t scan[kThreads];
  __shared__ uint32_t sel[2];
  const GroupOf w = group_of<kTpgCount>(g);
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
}

// Ordered compaction.  Thread t of a tile owns 16 consecutive elements, so positions follow
// from an exclusive scan over threads, on top of the counts of the partition's earlier tiles
// (at most a few hundred numbers, summed by every workgroup for itself).  The workgroup of
// the first tile writes the record's header.
// HALF: values are sent as halves (round to nearest even) and a kept slot of the buffer keeps
// what the rounding dropped instead of 0.
template <bool HALF>
__global__ __launch_bounds__(kThreads) void topk_emit_kernel(Geo g, float *buf, const uint32_t *state,
                                                             const uint32_t *tilecnt, uint8_t *payload,
                                                             int zero_selected) {
  __shared__ uint32_t scan[kThreads];
  constexpr int kPer = kTile / kThreads;
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  const uint32_t T = state[p * 8 + 6 + kStPrefix];   // the selection after level 3
  const uint32_t r = state[p * 8 + 6 + kStKRem];
  __shared__ uint32_t before[2][kThreads / 64];
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
  if (tile == 0 && threadIdx.x == 0) {
    uint8_t *rec0 = payload + (uint64_t)p * g.stride;
    uint32_t *hdr = reinterpret_cast<uint32_t *>(rec0);
    const uint32_t k = (uint32_t)k_of_device(g, p);
    hdr[0] = k;
    hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
    if (HALF) {
      // the format wants zeros from value k to the end of its last group of four words
      // (values 0..k-1 are written below, by whichever tiles hold them)
      uint16_t *val16 = reinterpret_cast<uint16_t *>(rec0 + kHeaderBytes + 4 * ru4(g.k_cap));
      for (uint32_t t = k; t < 2 * (uint32_t)ru4(cdiv(k, 2)); ++t) val16[t] = 0;
    }
  }
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
  uint32_t *idx = reinterpret_cast<uint32_t *>(rec + kHeaderBytes);
  float *val = reinterpret_cast<float *>(rec + kHeaderBytes + 4 * ru4(g.k_cap));
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
      idx[pos] = j;
      if (HALF) {
        const __half h = __float2half_rn(v[i]);
        reinterpret_cast<__half *>(val)[pos] = h;
        if (zero_selected) buf[base + j] = v[i] - __half2float(h);
      } else {
        val[pos] = v[i];
        if (zero_selected) buf[base + j] = 0.0f;
      }
      ++pos;
    }
  }
}

// acc_j = acc_j + val for the entries of one worker's top-k message (indices are distinct
// within a message, so plain read-modify-write suffices).
template <bool HALF>
__global__ __launch_bounds__(kThreads) void topk_accumulate_kernel(Geo g, const uint8_t *payload, float *acc) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint8_t *rec = payload + (uint64_t)p * g.stride;
  uint32_t k = *reinterpret_cast<const uint32_t *>(rec);
  k = k > g.k_cap ? g.k_cap : k;
  const uint32_t *idx = reinterpret_cast<const uint32_t *>(rec + kHeaderBytes);
  const float *val = reinterpret_cast<const float *>(rec + kHeaderBytes + 4 * ru4(g.k_cap));
  const uint64_t base = g.part_base(p);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads) {
    uint32_t j = idx[t];
    if (j < d) acc[base + j] = acc[base + j] + (HALF ? __half2float(reinterpret_cast<const __half *>(val)[t]) : val[t]);
  }
}

hipError_t topk_encode(const Geo &g, const bpc_params_t &prm, const bpc_params_t *, const Source &src,
                       uint8_t *payload, const Workspace &ws, hipStream_t stream) {
  uint32_t *hist = ws.at<uint32_t>(ws.lay.hist);
  uint32_t *state = ws.at<uint32_t>(ws.lay.state);
  uint32_t *tilecnt = ws.at<uint32_t>(ws.lay.tilecnt);
  float *dense = ws.at<float>(ws.lay.dense);
  // the vector being compressed ends up in the residual buffer (error feedback) or the workspace
  float *buf = src.residual ? src.residual : dense;
  const bool half = prm.kind == BPC_TOPK16;
  hipError_t e;
  if (!src.grad) {
    // server: sum the n decoded messages into the workspace in worker order
    e = fill_zero(dense, sizeof(float) * g.D, stream);
    if (e != hipSuccess) return e;
    dim3 grid((uint32_t)cdiv(g.k_cap, kThreads), g.P);
    for (int i = 0; i < src.msgs.n; ++i) {
      if (half) topk_accumulate_kernel<true><<<grid, kThreads, 0, stream>>>(g, src.msgs.ptr[i], dense);
      else topk_accumulate_kernel<false><<<grid, kThreads, 0, stream>>>(g, src.msgs.ptr[i], dense);
    }
  }
  e = fill_zero(hist, sizeof(uint32_t) * kHistPerPart * (size_t)g.P, stream);
  if (e != hipSuccess) return e;
  if (src.grad) {
    if (src.dtype == BPC_F16) {
      GradSource<__half> s{(const __half *)src.grad, src.residual};
      topk_load_hist1_kernel<<<group_grid(g, kTpgLoad), kThreads, 0, stream>>>(g, s, buf, hist);
    } else {
      GradSource<float> s{(const float *)src.grad, src.residual};
      topk_load_hist1_kernel<<<group_grid(g, kTpgLoad), kThreads, 0, stream>>>(g, s, buf, hist);
    }
  } else {
    DenseSumSource s{dense, src.residual, src.msgs.inv_n};
    topk_load_hist1_kernel<<<group_grid(g, kTpgLoad), kThreads, 0, stream>>>(g, s, buf, hist);
  }
  topk_hist_kernel<2><<<group_grid(g, kTpgHist2), kThreads, 0, stream>>>(g, buf, hist, state);
  topk_hist_kernel<3><<<group_grid(g, kTpgHist3), kThreads, 0, stream>>>(g, buf, hist, state);
  topk_count_kernel<<<group_grid(g, kTpgCount), kThreads, 0, stream>>>(g, buf, hist, state, tilecnt);
  if (half) topk_emit_kernel<true><<<g.n_tiles, kThreads, 0, stream>>>(g, buf, state, tilecnt, payload, src.residual != nullptr);
  else topk_emit_kernel<false><<<g.n_tiles, kThreads, 0, stream>>>(g, buf, state, tilecnt, payload, src.residual != nullptr);
  return hipGetLastError();
}

}  // namespace bpc
