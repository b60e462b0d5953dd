// Top-k compressor ("only the k largest gradient elements are sent", Section 3.2) with the
// residual update of Algorithm 4 in its fused form (Section 4.2, operator fusion: the
// residual is the vector itself with the k sent slots set to zero).
//
// Selection is an exact three-level radix select on the 31-bit magnitude key
// bits(v) & 0x7fffffff (11 + 10 + 10 bits), followed by an ordered compaction in which
// elements equal to the threshold key are admitted lowest index first:
//   load+hist1 : v_j from the source -> dense buffer; histogram of key >> 20
//   pick1      : bucket that holds the k-th largest key
//   hist2/pick2, hist3/pick3 : refine inside that bucket -> threshold key T and the number
//                r of elements with key == T that are kept
//   count/scan : per tile, how many keys are > T and == T; exclusive scan over tiles
//   emit       : (idx, val) in ascending index order; kept slots of the buffer zeroed
#include "sources.hpp"

namespace bpc {

constexpr int kBins1 = 2048, kBins23 = 1024;
constexpr int kHistPerPart = 4096;  // 2048 + 1024 + 1024

__device__ inline uint32_t key_of(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// state words per partition
enum { kStPrefix = 0, kStKRem = 1 };

template <class SRC>
__global__ __launch_bounds__(kThreads) void topk_load_hist1_kernel(Geo g, SRC src, float *buf, uint32_t *hist) {
  __shared__ float lds[SRC::kLdsFloats];
  __shared__ uint32_t h[kBins1];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  for (int b = threadIdx.x; b < kBins1; b += kThreads) h[b] = 0;
  src.begin(g, p, lds);
  __syncthreads();
  const uint64_t base = g.part_base(p);
#pragma unroll
  for (int c = 0; c < kTile / kThreads; ++c) {
    uint32_t j = tile * kTile + c * kThreads + threadIdx.x;
    if (j < d) {
      float v = src.at(g, p, j, lds);
      buf[base + j] = v;
      atomicAdd(&h[key_of(v) >> 20], 1u);
    }
  }
  __syncthreads();
  uint32_t *gh = hist + (uint64_t)p * kHistPerPart;
  for (int b = threadIdx.x; b < kBins1; b += kThreads)
    if (h[b]) atomicAdd(&gh[b], h[b]);
}

// LEVEL 2: keys whose top 11 bits equal the prefix, histogram of the next 10 bits.
// LEVEL 3: keys whose top 21 bits equal the prefix, histogram of the last 10 bits.
template <int LEVEL>
__global__ __launch_bounds__(kThreads) void topk_hist_kernel(Geo g, const float *buf, const uint32_t *state,
                                                             uint32_t *hist) {
  __shared__ uint32_t h[kBins23];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  for (int b = threadIdx.x; b < kBins23; b += kThreads) h[b] = 0;
  __syncthreads();
  const uint32_t prefix = state[p * 8 + kStPrefix];
  constexpr int kHiShift = LEVEL == 2 ? 20 : 10;
  constexpr int kLoShift = LEVEL == 2 ? 10 : 0;
  const uint64_t base = g.part_base(p);
#pragma unroll
  for (int c = 0; c < kTile / kThreads; ++c) {
    uint32_t j = tile * kTile + c * kThreads + threadIdx.x;
    if (j < d) {
      uint32_t key = key_of(buf[base + j]);
      if ((key >> kHiShift) == prefix) atomicAdd(&h[(key >> kLoShift) & 1023u], 1u);
    }
  }
  __syncthreads();
  uint32_t *gh = hist + (uint64_t)p * kHistPerPart + (LEVEL == 2 ? kBins1 : kBins1 + kBins23);
  for (int b = threadIdx.x; b < kBins23; b += kThreads)
    if (h[b]) atomicAdd(&gh[b], h[b]);
}

// One workgroup per partition.  Walk the histogram from the highest bin down and find the bin
// b with  count(bins above b) < k_rem <= count(bins above b) + count(b).
template <int LEVEL>
__global__ __launch_bounds__(kThreads) void topk_pick_kernel(Geo g, const uint32_t *hist, uint32_t *state) {
  __shared__ uint32_t scan[kThreads];
  constexpr int kBins = LEVEL == 1 ? kBins1 : kBins23;
  constexpr int kPer = kBins / kThreads;
  const uint32_t p = blockIdx.x;
  const uint32_t *gh = hist + (uint64_t)p * kHistPerPart + (LEVEL == 1 ? 0 : LEVEL == 2 ? kBins1 : kBins1 + kBins23);
  uint32_t k_rem, prefix;
  if (LEVEL == 1) {
    k_rem = (uint32_t)k_of_device(g, p);
    prefix = 0;
  } else {
    k_rem = state[p * 8 + kStKRem];
    prefix = state[p * 8 + kStPrefix];
  }
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
        state[p * 8 + kStPrefix] = LEVEL == 1 ? bin : ((prefix << 10) | bin);
        state[p * 8 + kStKRem] = k_rem - run;
      }
      run += cnt[i];
    }
  }
}

// Per tile: number of keys above the threshold and equal to it.
__global__ __launch_bounds__(kThreads) void topk_count_kernel(Geo g, const float *buf, const uint32_t *state,
                                                              uint32_t *tilecnt) {
  __shared__ uint32_t red[2][kThreads / 64];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  const uint32_t T = state[p * 8 + kStPrefix];
  const uint64_t base = g.part_base(p);
  uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
  for (int c = 0; c < kTile / kThreads; ++c) {
    uint32_t j = tile * kTile + c * kThreads + threadIdx.x;
    if (j < d) {
      uint32_t key = key_of(buf[base + j]);
      n_gt += key > T;
      n_eq += key == T;
    }
  }
  n_gt = wave_sum_u32(n_gt);
  n_eq = wave_sum_u32(n_eq);
  if ((threadIdx.x & 63) == 0) {
    red[0][threadIdx.x >> 6] = n_gt;
    red[1][threadIdx.x >> 6] = n_eq;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t a = 0, b = 0;
    for (int w = 0; w < kThreads / 64; ++w) { a += red[0][w]; b += red[1][w]; }
    tilecnt[2 * blockIdx.x] = a;
    tilecnt[2 * blockIdx.x + 1] = b;
  }
}

// One workgroup per partition: exclusive scan of the tile counts in place, and the header.
__global__ __launch_bounds__(kThreads) void topk_scan_kernel(Geo g, uint32_t *tilecnt, uint8_t *payload, int half_values) {
  __shared__ uint32_t scan[kThreads];
  const uint32_t p = blockIdx.x;
  const uint32_t d = g.part_size(p);
  const uint32_t n_tiles = (uint32_t)cdiv(d, kTile);
  uint32_t *tc = tilecnt + 2ull * p * g.tiles_per_part;
  const uint32_t per = (uint32_t)cdiv(n_tiles, kThreads);
  const uint32_t lo = threadIdx.x * per;
  const uint32_t hi = lo + per < n_tiles ? lo + per : n_tiles;
  uint32_t s_gt = 0, s_eq = 0;
  for (uint32_t t = lo; t < hi; ++t) { s_gt += tc[2 * t]; s_eq += tc[2 * t + 1]; }
  uint32_t tot;
  uint32_t ex_gt = block_exclusive_scan<kThreads>(s_gt, scan, &tot);
  uint32_t ex_eq = block_exclusive_scan<kThreads>(s_eq, scan, &tot);
  for (uint32_t t = lo; t < hi; ++t) {
    uint32_t a = tc[2 * t], b = tc[2 * t + 1];
    tc[2 * t] = ex_gt;
    tc[2 * t + 1] = ex_eq;
    ex_gt += a;
    ex_eq += b;
  }
  if (threadIdx.x == 0) {
    uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride);
    const uint32_t k = (uint32_t)k_of_device(g, p);
    hdr[0] = k;
    hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
    // half-precision values: the format wants zeros from value k to the end of its last
    // group of four words (emit writes values 0..k-1 only)
    if (half_values) {
      uint16_t *val = reinterpret_cast<uint16_t *>(payload + (uint64_t)p * g.stride + kHeaderBytes + 4 * ru4(g.k_cap));
      for (uint32_t t = k; t < 2 * (uint32_t)ru4(cdiv(k, 2)); ++t) val[t] = 0;
    }
  }
}

// Ordered compaction.  Thread t of a tile owns 16 consecutive elements, so positions follow
// from an exclusive scan over threads.
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
  const uint32_t T = state[p * 8 + kStPrefix];
  const uint32_t r = state[p * 8 + kStKRem];
  const uint32_t gt_before = tilecnt[2 * blockIdx.x];
  const uint32_t eq_before = tilecnt[2 * blockIdx.x + 1];
  const uint64_t base = g.part_base(p);
  const uint32_t j0 = tile * kTile + threadIdx.x * kPer;
  float v[kPer];
  uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    uint32_t j = j0 + i;
    v[i] = j < d ? buf[base + j] : 0.0f;
    uint32_t key = key_of(v[i]);
    n_gt += (j < d) && key > T;
    n_eq += (j < d) && key == T;
  }
  uint32_t tot;
  uint32_t ex_gt = block_exclusive_scan<kThreads>(n_gt, scan, &tot);
  uint32_t ex_eq = block_exclusive_scan<kThreads>(n_eq, scan, &tot);
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
      topk_load_hist1_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, s, buf, hist);
    } else {
      GradSource<float> s{(const float *)src.grad, src.residual};
      topk_load_hist1_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, s, buf, hist);
    }
  } else {
    DenseSumSource s{dense, src.residual, src.msgs.inv_n};
    topk_load_hist1_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, s, buf, hist);
  }
  topk_pick_kernel<1><<<g.P, kThreads, 0, stream>>>(g, hist, state);
  topk_hist_kernel<2><<<g.n_tiles, kThreads, 0, stream>>>(g, buf, state, hist);
  topk_pick_kernel<2><<<g.P, kThreads, 0, stream>>>(g, hist, state);
  topk_hist_kernel<3><<<g.n_tiles, kThreads, 0, stream>>>(g, buf, state, hist);
  topk_pick_kernel<3><<<g.P, kThreads, 0, stream>>>(g, hist, state);
  topk_count_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, buf, state, tilecnt);
  topk_scan_kernel<<<g.P, kThreads, 0, stream>>>(g, tilecnt, payload, half ? 1 : 0);
  if (half) topk_emit_kernel<true><<<g.n_tiles, kThreads, 0, stream>>>(g, buf, state, tilecnt, payload, src.residual != nullptr);
  else topk_emit_kernel<false><<<g.n_tiles, kThreads, 0, stream>>>(g, buf, state, tilecnt, payload, src.residual != nullptr);
  return hipGetLastError();
}

}  // namespace bpc
