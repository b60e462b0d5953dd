// Random-k compressor (Section 3.2: k randomly chosen entries of the gradient travel): k indices
// drawn uniformly with replacement from a Philox stream that sender and receiver share, so
// only the k values travel.  The decode multiplies by `value_scale` (d/k makes the operator
// unbiased, Definition 1; 1 gives the plain zero-fill residual of Section 4.2).  Residual
// update as in Algorithm 4: residual = v - decode(message).
//   store  : v_j from the source -> dense buffer (the residual buffer under error feedback)
//   gather : val_t = v[idx_t] -> message
//   fixup  : residual[idx_t] -= scale * val_t   (atomic: an index may repeat)
// Server: Delta is formed slice by slice in LDS (`randk_sum_kernel`): an atomic add on global
// memory costs some 11 ns of a memory channel's time, so scattering the n messages into a dense
// buffer in HBM (n k adds per partition) took half the server's time; a workgroup that keeps
// 32768 elements of Delta in LDS regenerates every draw of its partition instead and keeps
// those that fall into its slice.
#include "sources.hpp"
#include "tile_rows.hpp"
#include "cluster.hpp"
#include <hip/hip_runtime.h>

namespace bpc {

__device__ inline uint32_t randk_index(const Philox &rng, uint32_t t, uint32_t d) {
  return (uint32_t)(((uint64_t)rng.word(t) * d) >> 32);
}

template <class SRC>
__global__ __launch_bounds__(kThreads) void randk_store_kernel(Geo g, SRC src, float *buf) {
  __shared__ float lds[SRC::kLdsFloats];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  src.begin(g, p, lds);
  const uint64_t base = g.part_base(p);
#pragma unroll
  for (int c = 0; c < kTile / (kThreads * 8); ++c) {
    const uint32_t j0 = tile * kTile + c * (kThreads * 8) + threadIdx.x * 8;
    if (j0 >= d) continue;
    float v[8];
    source_at8(src, g, p, j0, d, lds, v);
    if (j0 + 8 <= d) {
      float4 *dst = reinterpret_cast<float4 *>(buf + base + j0);
      dst[0] = make_float4(v[0], v[1], v[2], v[3]);
      dst[1] = make_float4(v[4], v[5], v[6], v[7]);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (j0 + e < d) buf[base + j0 + e] = v[e];
    }
  }
}

// Server side: Delta_j = (sum_i decode(delta_i)_j) / n + e~_j for one slice of kRsSlice elements
// of one partition, summed in LDS in worker order (a barrier between workers; within a message
// repeated indices add equal values, so the order of its adds does not matter), then written to
// `buf` with the mean and the residual applied.
constexpr int kRsThreads = 1024;
constexpr uint32_t kRsSlice = 32768;
struct RandkScales { float value_scale[kMaxWorkers]; };

__global__ __launch_bounds__(kRsThreads) void randk_sum_kernel(Geo g, WorkerMsgs msgs, RandkScales sc, const float *res,
                                                               float *buf) {
  extern __shared__ float acc[];  // kRsSlice
  const uint32_t slices_per_part = (uint32_t)cdiv(g.part_elems, kRsSlice);
  const uint32_t p = blockIdx.x / slices_per_part, lo = (blockIdx.x % slices_per_part) * kRsSlice;
  const uint32_t d = g.part_size(p);
  if (lo >= d) return;
  const uint32_t len = d - lo < kRsSlice ? d - lo : kRsSlice;
  for (uint32_t q = threadIdx.x; q < kRsSlice / 4; q += kRsThreads) reinterpret_cast<float4 *>(acc)[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  __syncthreads();
  for (int i = 0; i < msgs.n; ++i) {
    const uint8_t *rec = msgs.ptr[i] + (uint64_t)p * g.stride;
    uint32_t k = *reinterpret_cast<const uint32_t *>(rec);
    k = k > g.k_cap ? g.k_cap : k;
    const float *val = reinterpret_cast<const float *>(rec + kHeaderBytes);
    const float scale = sc.value_scale[i] >= 0.0f ? sc.value_scale[i] : (float)d / (float)k;
    const Philox rng(msgs.seed[i], msgs.stream_id[i], p + g.part0);
    for (uint32_t t4 = threadIdx.x; 4 * t4 < k; t4 += kRsThreads) {
      uint32_t rnd[4];
      rng.block(t4, rnd);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t t = 4 * t4 + c;
        const uint32_t rel = (uint32_t)(((uint64_t)rnd[c] * d) >> 32) - lo;
        if (t < k && rel < len) atomicAdd(&acc[rel], scale * val[t]);
      }
    }
    __syncthreads();
  }
  const uint64_t at = g.part_base(p) + lo;
  for (uint32_t q = threadIdx.x * 4; q < len; q += kRsThreads * 4) {
    if (q + 4 <= len) {
      const float4 a = *reinterpret_cast<const float4 *>(acc + q);
      float4 r = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (res) r = *reinterpret_cast<const float4 *>(res + at + q);
      const float m0 = a.x * msgs.inv_n, m1 = a.y * msgs.inv_n, m2 = a.z * msgs.inv_n, m3 = a.w * msgs.inv_n;
      *reinterpret_cast<float4 *>(buf + at + q) = res ? make_float4(m0 + r.x, m1 + r.y, m2 + r.z, m3 + r.w) : make_float4(m0, m1, m2, m3);
    } else {
      for (uint32_t e = q; e < len; ++e) {
        const float mean = acc[e] * msgs.inv_n;
        buf[at + e] = res ? mean + res[at + e] : mean;
      }
    }
  }
}

// The same in two steps, for when the dense workspace is free to hold lists (the server has a
// residual buffer for Delta and the lists fit): `randk_bin_kernel` writes each message's draws
// as (index, scaled value) pairs grouped by slice, with a table of where each slice's group
// starts; `randk_sum_binned_kernel` then adds up only the pairs of its own slice, so no draw is
// regenerated more than twice and slices can be small (8192 elements: several workgroups a
// compute unit, loads and stores of different slices overlap).
constexpr int kRbThreads = 1024;    // (workgroups of 256, four bins a thread, took a third longer)
constexpr uint32_t kRbMaxBins = 1024;   // slices of a partition, at most
constexpr int kRbSumThreads = 256;

// OUT: the draws of a message still to be written (stream i of `msgs`, k by the rule): the
// pairs are (index, number of the draw).
// STAGE: the pairs are put in order in LDS (k_cap * 8 bytes of dynamic LDS) and written out in
// whole lines; else each pair is stored where it belongs directly (scattered 8-byte stores,
// which were most of this kernel's time with eight messages of 10 K draws a partition).
template <bool OUT, bool STAGE>
__global__ __launch_bounds__(kRbThreads) void randk_bin_kernel(Geo g, WorkerMsgs msgs, RandkScales sc, uint32_t slice_shift,
                                                               uint2 *lists, uint32_t *table, uint32_t *status) {
  extern __shared__ uint2 staged[];
  // (status, where given: the workspace's status word; random-k has no waits, so it reads "none gave up")
  if (status && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) status[0] = 0;
  __shared__ uint32_t cnt[kRbMaxBins];
  __shared__ uint32_t scan[kRbThreads];
  const uint32_t p = blockIdx.x, i = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint8_t *rec = OUT ? nullptr : msgs.ptr[i] + (uint64_t)p * g.stride;
  uint32_t k = OUT ? (uint32_t)k_of_device(g, p) : *reinterpret_cast<const uint32_t *>(rec);
  k = k > g.k_cap ? g.k_cap : k;
  const float *val = reinterpret_cast<const float *>(rec + kHeaderBytes);
  const float scale = sc.value_scale[i] >= 0.0f ? sc.value_scale[i] : (float)d / (float)k;
  const Philox rng(msgs.seed[i], msgs.stream_id[i], p + g.part0);
  constexpr int kMine = kRbMaxBins / kRbThreads;   // bins a thread owns: 4 consecutive ones
  for (int b = threadIdx.x; b < (int)kRbMaxBins; b += kRbThreads) cnt[b] = 0;
  __syncthreads();
  for (uint32_t t4 = threadIdx.x; 4 * t4 < k; t4 += kRbThreads) {
    uint32_t rnd[4];
    rng.block(t4, rnd);
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (4 * t4 + c < k) atomicAdd(&cnt[(uint32_t)(((uint64_t)rnd[c] * d) >> 32) >> slice_shift], 1u);
  }
  __syncthreads();
  uint32_t mine[kMine], local = 0;
#pragma unroll
  for (int b = 0; b < kMine; ++b) {
    mine[b] = cnt[threadIdx.x * kMine + b];
    local += mine[b];
  }
  uint32_t total;
  uint32_t start = block_exclusive_scan<kRbThreads>(local, scan, &total);
  uint32_t *tab = table + ((uint64_t)i * g.P + p) * (kRbMaxBins + 1);
#pragma unroll
  for (int b = 0; b < kMine; ++b) {
    tab[threadIdx.x * kMine + b] = start;
    cnt[threadIdx.x * kMine + b] = start;   // from here on: where the slice's next pair goes
    start += mine[b];
  }
  if (threadIdx.x == 0) tab[kRbMaxBins] = total;
  __syncthreads();
  uint2 *list = lists + ((uint64_t)i * g.P + p) * g.k_cap;
  for (uint32_t t4 = threadIdx.x; 4 * t4 < k; t4 += kRbThreads) {
    uint32_t rnd[4];
    rng.block(t4, rnd);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t t = 4 * t4 + c;
      if (t < k) {
        const uint32_t j = (uint32_t)(((uint64_t)rnd[c] * d) >> 32);
        const uint32_t pos = atomicAdd(&cnt[j >> slice_shift], 1u);
        const uint2 pair = make_uint2(j, OUT ? t : __float_as_uint(scale * val[t]));
        if (STAGE) staged[pos] = pair;
        else list[pos] = pair;
      }
    }
  }
  if (STAGE) {
    __syncthreads();
    for (uint32_t q = threadIdx.x; q < k; q += kRbThreads) list[q] = staged[q];
  }
}

// The message's draws that fall into the slice [lo, lo + len) of v, which the workgroup holds in
// `acc` (LDS): val_t = v[idx_t] goes to the record, then every draw takes scale * val_t off its
// element (all reads first: draws of one index read the same value).  `list`: (index, t) pairs,
// those of this slice at [from, to).  All threads of the workgroup; leaves acc = the residual.
template <int THREADS>
__device__ inline void randk_apply_draws(float *acc, uint32_t lo, const uint2 *list, uint32_t from, uint32_t to, float scale,
                                         float *val) {
  __syncthreads();
  const bool mine = from + threadIdx.x < to;
  uint2 ent = make_uint2(lo, 0u);
  float v = 0.0f;
  if (mine) {
    ent = list[from + threadIdx.x];
    v = acc[ent.x - lo];
    val[ent.y] = v;
  }
  for (uint32_t q = from + THREADS + threadIdx.x; q < to; q += THREADS) {   // (rare: more draws than threads)
    const uint2 e2 = list[q];
    val[e2.y] = acc[e2.x - lo];
  }
  __syncthreads();
  if (mine) atomicAdd(&acc[ent.x - lo], -(scale * v));
  for (uint32_t q = from + THREADS + threadIdx.x; q < to; q += THREADS) {
    const uint2 e2 = list[q];
    atomicAdd(&acc[e2.x - lo], -(scale * val[e2.y]));
  }
  __syncthreads();
}

// Worker with error feedback in one pass over the data: a workgroup forms its tile of q = g + e
// in LDS, serves the draws that fall into it (binned per tile by `randk_bin_kernel<true>`) and
// writes the tile of the residual.
template <class SRC>
__global__ __launch_bounds__(kThreads) void randk_tile_kernel(Geo g, SRC src, float *buf, uint8_t *payload, float value_scale,
                                                              const uint2 *lists, const uint32_t *table) {
  __shared__ float acc[kTile];
  const uint32_t p = blockIdx.x / g.tiles_per_part, tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  const uint32_t lo = tile * kTile;
  if (lo >= d) return;
  const uint32_t k = (uint32_t)k_of_device(g, p);
  if (tile == 0 && threadIdx.x == 0) {
    uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride);
    hdr[0] = k; hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
  }
  const uint32_t *tab = table + (uint64_t)p * (kRbMaxBins + 1);
  const uint32_t from = tab[tile], to = tab[tile + 1];
  // the tile as rows of 1024 elements, 4 consecutive a thread, through descriptors of the
  // elements that exist: whole-line non-temporal accesses, all loads requested before the first
  // is used (elements past a shorter last partition read as zero and are not written back)
  using T = typename SRC::Elem;
  constexpr int kRowElems = kThreads * 4, kRows = kTile / kRowElems;
  const uint32_t valid = __builtin_amdgcn_readfirstlane(d - lo < (uint32_t)kTile ? d - lo : (uint32_t)kTile);
  const uint64_t base = uniform_off(g.part_base(p) + lo);
  {
    const bool ef = src.res != nullptr;
    const TileBuf gb(src.grad + base, valid * (uint32_t)sizeof(T));
    const TileBuf eb(ef ? src.res + base : nullptr, ef ? valid * 4 : 0);
    typename Vec4Of<T>::type gr[kRows];
    u32x4 er[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      gr[u] = tile_load4(gb, threadIdx.x * 4 * (uint32_t)sizeof(T), u * kRowElems * (uint32_t)sizeof(T), (const T *)nullptr);
      er[u] = eb.load16<kNonTemporal>(threadIdx.x * 16, u * kRowElems * 4);
    }
    if constexpr (sizeof(T) == 2) patch_last_half<kRows, kRowElems>(gb, valid, gr);
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      float x[4], e[4];
      widen4(gr[u], x);
      widen4(er[u], e);
      reinterpret_cast<float4 *>(acc)[u * kThreads + threadIdx.x] =
          ef ? make_float4(x[0] + e[0], x[1] + e[1], x[2] + e[2], x[3] + e[3]) : make_float4(x[0], x[1], x[2], x[3]);
    }
  }
  const float scale = value_scale >= 0.0f ? value_scale : (float)d / (float)k;
  float *val = reinterpret_cast<float *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
  randk_apply_draws<kThreads>(acc, lo, lists + (uint64_t)p * g.k_cap, from < k ? from : k, to < k ? to : k, scale, val);
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    const float4 a = reinterpret_cast<const float4 *>(acc)[u * kThreads + threadIdx.x];
    row_buf(buf + base, valid, u * kRowElems, kRowElems).store16<kNonTemporal>(as_u32x4(a.x, a.y, a.z, a.w), threadIdx.x * 16);
  }
}

// EARLY (slices of 8192 elements): the residual's elements of the slice are requested before
// the sum is formed (32 registers a thread).
template <bool EARLY>
__global__ __launch_bounds__(kRbSumThreads) void randk_sum_binned_kernel(Geo g, int n, float inv_n, uint32_t slice_shift,
                                                                         const uint2 *lists, const uint32_t *table,
                                                                         const float *res, float *buf, uint8_t *payload,
                                                                         float value_scale) {
  extern __shared__ float acc[];  // 1 << slice_shift
  __shared__ uint32_t from[kMaxWorkers], to[kMaxWorkers];
  const uint32_t slice = 1u << slice_shift;
  const uint32_t slices_per_part = (uint32_t)cdiv(g.part_elems, slice);
  const uint32_t p = blockIdx.x / slices_per_part, s = blockIdx.x % slices_per_part, lo = s << slice_shift;
  const uint32_t d = g.part_size(p);
  if (lo >= d) return;
  const uint32_t len = d - lo < slice ? d - lo : slice;
  if (threadIdx.x < (uint32_t)n) {
    const uint32_t *tab = table + ((uint64_t)threadIdx.x * g.P + p) * (kRbMaxBins + 1);
    from[threadIdx.x] = tab[s];
    to[threadIdx.x] = tab[s + 1];
  }
  constexpr int kEarly = 8192 / (kRbSumThreads * 4);   // 16-byte pieces of a slice of 8192 elements a thread
  // the residual and the buffer through descriptors of the slice's elements that exist (what lies
  // past them reads as zero and is not written): 4 consecutive elements a thread and access,
  // whole lines a wave, non-temporal
  const uint64_t at = uniform_off(g.part_base(p) + lo);
  const TileBuf rb(res ? res + at : nullptr, res ? len * 4 : 0);
  u32x4 early[kEarly];
  if (EARLY) {
#pragma unroll
    for (int c = 0; c < kEarly; ++c) early[c] = rb.load16<kNonTemporal>((c * kRbSumThreads + threadIdx.x) * 16, 0);
  }
  for (uint32_t q = threadIdx.x; q < slice / 4; q += kRbSumThreads) reinterpret_cast<float4 *>(acc)[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  __syncthreads();
  // worker by worker (a barrier in between); the first pair a thread adds for the next worker
  // is requested before the adds of this one
  auto first_pair = [&](int i) {
    const uint32_t q = from[i] + threadIdx.x;
    return lists[((uint64_t)i * g.P + p) * g.k_cap + (q < to[i] ? q : from[i] < to[i] ? from[i] : 0u)];
  };
  uint2 next = first_pair(0);
  for (int i = 0; i < n; ++i) {
    const uint2 mine = next;
    if (i + 1 < n) next = first_pair(i + 1);
    const uint2 *list = lists + ((uint64_t)i * g.P + p) * g.k_cap;
    const uint32_t b = from[i], e = to[i];
    if (b + threadIdx.x < e) atomicAdd(&acc[mine.x - lo], __uint_as_float(mine.y));
    for (uint32_t q = b + kRbSumThreads + threadIdx.x; q < e; q += kRbSumThreads) {
      const uint2 ent = list[q];
      atomicAdd(&acc[ent.x - lo], __uint_as_float(ent.y));
    }
    __syncthreads();
  }
  {
    // Delta in LDS, the recompression's draws served from there (list n is the output's),
    // and what is left is the new residual
    if (EARLY) {
#pragma unroll
      for (int c = 0; c < kEarly; ++c) {
        const uint32_t q = (c * kRbSumThreads + threadIdx.x) * 4;
        const float4 a = *reinterpret_cast<const float4 *>(acc + q);
        const float m0 = a.x * inv_n, m1 = a.y * inv_n, m2 = a.z * inv_n, m3 = a.w * inv_n;
        float r[4];
        widen4(early[c], r);
        *reinterpret_cast<float4 *>(acc + q) = res ? make_float4(m0 + r[0], m1 + r[1], m2 + r[2], m3 + r[3])
                                                    : make_float4(m0, m1, m2, m3);
      }
    }
    for (uint32_t q = threadIdx.x * 4; !EARLY && q < slice; q += kRbSumThreads * 4) {
      float4 a = *reinterpret_cast<const float4 *>(acc + q);
      float r[4];
      widen4(rb.load16<kNonTemporal>(q * 4, 0), r);
      const float m0 = a.x * inv_n, m1 = a.y * inv_n, m2 = a.z * inv_n, m3 = a.w * inv_n;
      *reinterpret_cast<float4 *>(acc + q) = res ? make_float4(m0 + r[0], m1 + r[1], m2 + r[2], m3 + r[3]) : make_float4(m0, m1, m2, m3);
    }
    const uint32_t k = (uint32_t)k_of_device(g, p);
    if (s == 0 && threadIdx.x == 0) {
      uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride);
      hdr[0] = k; hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
    }
    const uint32_t *tab = table + ((uint64_t)n * g.P + p) * (kRbMaxBins + 1);
    const uint32_t f0 = tab[s] < k ? tab[s] : k, t0 = tab[s + 1] < k ? tab[s + 1] : k;
    const float scale = value_scale >= 0.0f ? value_scale : (float)d / (float)k;
    randk_apply_draws<kRbSumThreads>(acc, lo, lists + ((uint64_t)n * g.P + p) * g.k_cap, f0, t0, scale,
                                     reinterpret_cast<float *>(payload + (uint64_t)p * g.stride + kHeaderBytes));
    const TileBuf ob(buf + at, len * 4);
    for (uint32_t q = threadIdx.x * 4; q < len; q += kRbSumThreads * 4) {
      const float4 a = *reinterpret_cast<const float4 *>(acc + q);
      ob.store16<kNonTemporal>(as_u32x4(a.x, a.y, a.z, a.w), q * 4);
    }
  }
}

__device__ inline void randk_header(const Geo &g, uint32_t p, uint32_t k, uint8_t *payload) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride);
    hdr[0] = k; hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
  }
}

// val_t = buf[idx_t]
__global__ __launch_bounds__(kThreads) void randk_gather_kernel(Geo g, const float *buf, uint8_t *payload,
                                                                uint64_t seed, uint64_t stream_id) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint32_t k = (uint32_t)k_of_device(g, p);
  randk_header(g, p, k, payload);
  float *val = reinterpret_cast<float *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
  const uint64_t base = g.part_base(p);
  const Philox rng(seed, stream_id, p + g.part0);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads)
    val[t] = buf[base + randk_index(rng, t, d)];
}

// Same, reading the worker's gradient directly (no error feedback: nothing dense is written).
template <class SRC>
__global__ __launch_bounds__(kThreads) void randk_gather_src_kernel(Geo g, SRC src, uint8_t *payload,
                                                                    uint64_t seed, uint64_t stream_id) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint32_t k = (uint32_t)k_of_device(g, p);
  randk_header(g, p, k, payload);
  float *val = reinterpret_cast<float *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
  const Philox rng(seed, stream_id, p + g.part0);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads)
    val[t] = src.at(g, p, randk_index(rng, t, d), nullptr);
}

__global__ __launch_bounds__(kThreads) void randk_fixup_kernel(Geo g, float *buf, const uint8_t *payload,
                                                               float value_scale, uint64_t seed,
                                                               uint64_t stream_id) {
  const uint32_t p = blockIdx.y;
  const uint32_t d = g.part_size(p);
  const uint32_t k = (uint32_t)k_of_device(g, p);
  const float *val = reinterpret_cast<const float *>(payload + (uint64_t)p * g.stride + kHeaderBytes);
  const float scale = value_scale >= 0.0f ? value_scale : (float)d / (float)k;
  const uint64_t base = g.part_base(p);
  const Philox rng(seed, stream_id, p + g.part0);
  for (uint32_t t = blockIdx.x * kThreads + threadIdx.x; t < k; t += gridDim.x * kThreads)
    atomicAdd(buf + base + randk_index(rng, t, d), -(scale * val[t]));
}

// Launches the binning kernel over P partitions x n streams, staged through LDS where the list of
// a partition fits.
template <bool OUT>
static hipError_t launch_randk_bin(const Geo &g, const WorkerMsgs &msgs, const RandkScales &sc, int n, uint32_t slice_shift,
                                   uint2 *lists, uint32_t *table, hipStream_t stream, uint32_t *status = nullptr) {
  const size_t lds = (size_t)g.k_cap * sizeof(uint2);
  constexpr size_t kMaxStage = 96 * 1024;
  static PerDevice attr;
  const bool big_ok = attr.get([] { return lds_limit_raised(reinterpret_cast<const void *>(&randk_bin_kernel<OUT, true>), kMaxStage); }) > 0;
  if (lds <= kMaxStage && (big_ok || lds <= 48 * 1024))
    randk_bin_kernel<OUT, true><<<dim3(g.P, n), kRbThreads, lds, stream>>>(g, msgs, sc, slice_shift, lists, table, status);
  else
    randk_bin_kernel<OUT, false><<<dim3(g.P, n), kRbThreads, 0, stream>>>(g, msgs, sc, slice_shift, lists, table, status);
  return hipGetLastError();
}

// One message's draws as (index, scaled value) pairs grouped by tile of 1 << tile_shift elements:
// lists[p * k_cap ..], table[p * kRandkTableStride + tile] = where the tile's pairs start.
// Needs at most 1024 tiles to a partition.
hipError_t randk_bin_tiles(const Geo &g, const bpc_params_t &prm, const uint8_t *payload, uint2 *lists, uint32_t *table,
                           uint32_t tile_shift, hipStream_t stream) {
  static_assert(kRandkTableStride == kRbMaxBins + 1, "table layout");
  WorkerMsgs msgs{};
  msgs.ptr[0] = payload;
  msgs.seed[0] = prm.seed;
  msgs.stream_id[0] = prm.stream_id;
  msgs.n = 1;
  RandkScales sc{};
  sc.value_scale[0] = prm.value_scale;
  return launch_randk_bin<false>(g, msgs, sc, 1, tile_shift, lists, table, stream);
}

hipError_t randk_encode(const Geo &g, const bpc_params_t &prm, const bpc_params_t *in_prm, const Source &src,
                        uint8_t *payload, const Workspace &ws, hipStream_t stream) {
  float *dense = ws.at<float>(ws.lay.dense);
  float *buf = src.residual ? src.residual : dense;
  dim3 grid((uint32_t)cdiv(g.k_cap, kThreads), g.P);
  // the message's own draws, for the kernels that serve them from LDS
  WorkerMsgs out_stream{};
  out_stream.seed[0] = prm.seed;
  out_stream.stream_id[0] = prm.stream_id;
  out_stream.n = 1;
  RandkScales out_scale{};
  out_scale.value_scale[0] = prm.value_scale;
  const uint64_t one_list = ((uint64_t)g.P * g.k_cap * sizeof(uint2) + 255) / 256 * 256;
  const uint64_t one_table = ((uint64_t)g.P * (kRbMaxBins + 1) * sizeof(uint32_t) + 255) / 256 * 256;
  // the status word: cleared by the binning kernel on the paths that start with it, by a fill elsewhere
  uint32_t *status = ws.status();
  if (src.grad) {
    if (!src.residual) {
      hipError_t e0 = fill_zero(status, 16, stream);
      if (e0 != hipSuccess) return e0;
      if (src.dtype == BPC_F16)
        randk_gather_src_kernel<<<grid, kThreads, 0, stream>>>(g, GradSource<__half>{(const __half *)src.grad, nullptr},
                                                               payload, prm.seed, prm.stream_id);
      else
        randk_gather_src_kernel<<<grid, kThreads, 0, stream>>>(g, GradSource<float>{(const float *)src.grad, nullptr},
                                                               payload, prm.seed, prm.stream_id);
      return hipGetLastError();
    }
    if (g.tiles_per_part <= kRbMaxBins && one_list + one_table <= sizeof(float) * g.D) {
      // one pass over the data (q goes to the residual buffer, so the dense workspace is free for the list)
      uint2 *lists = reinterpret_cast<uint2 *>(dense);
      uint32_t *table = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(dense) + one_list);
      hipError_t e = launch_randk_bin<true>(g, out_stream, out_scale, 1, 12, lists, table, stream, status);
      if (e != hipSuccess) return e;
      if (src.dtype == BPC_F16)
        randk_tile_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, GradSource<__half>{(const __half *)src.grad, src.residual}, buf,
                                                              payload, prm.value_scale, lists, table);
      else
        randk_tile_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, GradSource<float>{(const float *)src.grad, src.residual}, buf,
                                                              payload, prm.value_scale, lists, table);
      return hipGetLastError();
    }
    hipError_t e0 = fill_zero(status, 16, stream);
    if (e0 != hipSuccess) return e0;
    if (src.dtype == BPC_F16)
      randk_store_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, GradSource<__half>{(const __half *)src.grad, src.residual}, buf);
    else
      randk_store_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, GradSource<float>{(const float *)src.grad, src.residual}, buf);
  } else {
    // workers that drew from one stream sent values for the same indices
    bool shared = src.msgs.n > 1;
    for (int i = 1; i < src.msgs.n; ++i)
      shared = shared && in_prm[i].seed == in_prm[0].seed && in_prm[i].stream_id == in_prm[0].stream_id &&
               in_prm[i].value_scale == in_prm[0].value_scale;
    static PerDevice attr1;
    const bool lds_ok = attr1.get([] { return lds_limit_raised(reinterpret_cast<const void *>(&randk_sum_kernel), kRsSlice * sizeof(float)); }) > 0;
    if (shared || !lds_ok) {
      hipError_t e = fill_zero(status, 16, stream);
      if (e != hipSuccess) return e;
      e = fill_zero(dense, sizeof(float) * g.D, stream);
      if (e != hipSuccess) return e;
      if (shared) {
        e = scatter_add_randk_shared(g, in_prm[0], src.msgs, dense, stream);
        if (e != hipSuccess) return e;
      } else {
        for (int i = 0; i < src.msgs.n; ++i) {
          e = scatter_add_sparse(g, in_prm[i], src.msgs.ptr[i], dense, stream);
          if (e != hipSuccess) return e;
        }
      }
      randk_store_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, DenseSumSource{dense, src.residual, src.msgs.inv_n}, buf);
    } else {
      RandkScales sc;
      for (int i = 0; i < src.msgs.n; ++i) sc.value_scale[i] = in_prm[i].value_scale;
      // slices of 8192 elements, larger (up to what LDS holds) if a partition would have more than kRbMaxBins of them
      uint32_t slice_shift = 13;
      while (slice_shift < 15 && cdiv(g.part_elems, 1ull << slice_shift) > kRbMaxBins) ++slice_shift;
      const int n = src.msgs.n;
      // n lists and tables for the messages and one more for the output's draws, in the dense
      // workspace (free: Delta goes to the residual buffer)
      const bool binned = src.residual != nullptr && cdiv(g.part_elems, 1ull << slice_shift) <= kRbMaxBins &&
                          (n + 1) * (one_list + one_table) <= sizeof(float) * g.D;
      static PerDevice attr2;
      const bool lds2_ok = attr2.get([] { return lds_limit_raised(reinterpret_cast<const void *>(&randk_sum_binned_kernel<false>), 4u << 15); }) > 0;
      if (binned && (lds2_ok || slice_shift == 13)) {
        uint2 *lists = reinterpret_cast<uint2 *>(dense);
        uint32_t *table = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(dense) + (n + 1) * one_list);
        hipError_t e = launch_randk_bin<false>(g, src.msgs, sc, n, slice_shift, lists, table, stream, status);
        if (e != hipSuccess) return e;
        e = launch_randk_bin<true>(g, out_stream, out_scale, 1, slice_shift, lists + (uint64_t)n * g.P * g.k_cap,
                                   table + (uint64_t)n * g.P * (kRbMaxBins + 1), stream);
        if (e != hipSuccess) return e;
        const uint32_t slices = g.P * (uint32_t)cdiv(g.part_elems, 1ull << slice_shift);
        if (slice_shift == 13)
          randk_sum_binned_kernel<true><<<slices, kRbSumThreads, sizeof(float) << slice_shift, stream>>>(
              g, n, src.msgs.inv_n, slice_shift, lists, table, src.residual, buf, payload, prm.value_scale);
        else
          randk_sum_binned_kernel<false><<<slices, kRbSumThreads, sizeof(float) << slice_shift, stream>>>(
              g, n, src.msgs.inv_n, slice_shift, lists, table, src.residual, buf, payload, prm.value_scale);
        return hipGetLastError();
      }
      const uint32_t slices = g.P * (uint32_t)cdiv(g.part_elems, kRsSlice);
      hipError_t e = fill_zero(status, 16, stream);
      if (e != hipSuccess) return e;
      randk_sum_kernel<<<slices, kRsThreads, kRsSlice * sizeof(float), stream>>>(g, src.msgs, sc, src.residual, buf);
    }
  }
  randk_gather_kernel<<<grid, kThreads, 0, stream>>>(g, buf, payload, prm.seed, prm.stream_id);
  if (src.residual)
    randk_fixup_kernel<<<grid, kThreads, 0, stream>>>(g, buf, payload, prm.value_scale, prm.seed, prm.stream_id);
  return hipGetLastError();
}

}  // namespace bpc
