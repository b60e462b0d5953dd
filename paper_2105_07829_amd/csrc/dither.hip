// Dithering, multi-pass form (linear levels: the stochastic multi-level quantiser the paper
// cites for its dithering compressors, Section 3.2; natural levels: powers of two): with
// a = s|v_j|/nu the level is floor(a)+1 with probability a-floor(a), else floor(a).  Message:
// nu once, then one nibble (sign, low level bits) per element and, beyond 7 levels, one bit
// plane per further level bit.
// Residual update as in Algorithm 4.  Three launches per call:
//   reduce : per-tile partial of sum v_j^2 (f64) or max |v_j|
//   finish : nu per partition -> record header
//   apply  : levels from Philox draws, packed nibbles, residual_j = v_j - decode_j
#include "cluster.hpp"
#include "sources.hpp"

namespace bpc {

constexpr int kPerThread = 8;                       // one message word per thread
constexpr int kRowElems = kThreads * kPerThread;    // 2048
constexpr int kRows = kTile / kRowElems;            // 2

template <class SRC>
__global__ __launch_bounds__(kThreads) void dither_reduce_kernel(Geo g, SRC src, double *partials, int linf) {
  __shared__ float lds[SRC::kLdsFloats];
  __shared__ double red[kThreads / 64];
  __shared__ float redf[kThreads / 64];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  src.begin(g, p, lds);
  double acc = 0.0;
  float mx = 0.0f;
  if constexpr (has_at8<SRC>::value) {
    // sources that decode a message word at a time: 8 consecutive elements a thread
#pragma unroll
    for (int row = 0; row < kRows; ++row) {
      const uint32_t j0 = tile * kTile + row * kRowElems + threadIdx.x * kPerThread;
      if (j0 >= d) continue;
      float v8[8];
      source_at8(src, g, p, j0, d, lds, v8);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        acc = fma((double)v8[e], (double)v8[e], acc);
        mx = fmaxf(mx, fabsf(v8[e]));
      }
    }
  } else {
#pragma unroll
    for (int c = 0; c < kTile / kThreads; ++c) {
      uint32_t j = tile * kTile + c * kThreads + threadIdx.x;
      float v = j < d ? src.at(g, p, j, lds) : 0.0f;
      acc = fma((double)v, (double)v, acc);  // the product of two f32 is exact in f64
      mx = fmaxf(mx, fabsf(v));
    }
  }
  if (linf) {
    float m = block_max<kThreads>(mx, redf);
    if (threadIdx.x == 0) partials[blockIdx.x] = (double)m;
  } else {
    double s = block_sum<kThreads>(acc, red);
    if (threadIdx.x == 0) partials[blockIdx.x] = s;
  }
}

__global__ __launch_bounds__(64) void dither_finish_kernel(Geo g, const double *partials, const float *override,
                                                           int linf, uint8_t *payload, uint32_t *status) {
  // (status: NULL when a single-pass kernel of the same call may have set the word)
  if (status && blockIdx.x == 0 && threadIdx.x == 0) status[0] = 0;
  const uint32_t p = blockIdx.x;
  const uint32_t d = g.part_size(p);
  const uint32_t n_tiles = (uint32_t)cdiv(d, kTile);
  float nu;
  if (override) {
    nu = override[p];
  } else if (linf) {
    float m = 0.0f;
    for (uint32_t t = threadIdx.x; t < n_tiles; t += 64)
      m = fmaxf(m, (float)partials[(uint64_t)p * g.tiles_per_part + t]);
    nu = wave_max(m);
  } else {
    double s = 0.0;
    for (uint32_t t = threadIdx.x; t < n_tiles; t += 64) s += partials[(uint64_t)p * g.tiles_per_part + t];
    s = wave_sum(s);
    nu = (float)sqrt(s);
  }
  if (threadIdx.x == 0) {
    uint32_t *hdr = reinterpret_cast<uint32_t *>(payload + (uint64_t)p * g.stride);
    hdr[0] = __float_as_uint(nu);
    hdr[1] = 0; hdr[2] = 0; hdr[3] = 0;
  }
}

// Level and residual of one element; `r` is the element's random word.
__device__ inline uint32_t dither_one(float v, float nu, uint32_t s, bool natural, uint32_t r, const float *mags,
                                      float *resid) {
  if (!(nu > 0.0f)) {
    *resid = v;
    return 0u;
  }
  const float top = dither_top(s, natural);
  const float top_over_nu = top / nu;   // once per partition in effect: nu and s are uniform
  const float a = top_over_nu <= 3.402823466e38f ? fabsf(v) * top_over_nu : (fabsf(v) * top) / nu;
  uint32_t lower;
  float f;
  if (!natural) {
    const float l = floorf(a);
    f = a - l;
    lower = (uint32_t)l;
  } else {   // levels at a = 0, 1, 2, 4, ...: exponent field and fraction bits of a
    const uint32_t bits = __float_as_uint(a);
    const bool below = a < 1.0f;
    lower = below ? 0u : (bits >> 23) - 126u;
    f = below ? a : __uint_as_float((bits & 0x007fffffu) | 0x3f800000u) - 1.0f;
  }
  const float u = (float)(r >> 8) * 0x1p-24f;
  uint32_t level = lower + (u < f ? 1u : 0u);
  level = level > s ? s : level;
  const float mag = mags[level];
  *resid = v - (v < 0.0f ? -mag : mag);
  return (v < 0.0f ? 64u : 0u) | level;   // bit 6: sign, bits 0..5: level
}

template <class SRC>
__global__ __launch_bounds__(kThreads) void dither_apply_kernel(Geo g, SRC src, uint8_t *payload, float *residual,
                                                                uint32_t levels, bool natural, uint64_t seed,
                                                                uint64_t stream_id) {
  __shared__ float lds[SRC::kLdsFloats];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  __shared__ float mags[64];   // decoded magnitudes of the levels 0..s
  uint8_t *rec = payload + (uint64_t)p * g.stride;
  const float nu = *reinterpret_cast<const float *>(rec);
  if (threadIdx.x <= levels) mags[threadIdx.x] = dither_mag(nu, threadIdx.x, levels, natural);
  src.begin(g, p, lds);   // ends with a barrier when it fills its tables
  __syncthreads();
  uint32_t *nibs = reinterpret_cast<uint32_t *>(rec + kHeaderBytes);
  const uint32_t n_words = (uint32_t)ru4(cdiv(d, 8));
  // bit planes of the levels above 7 (none for up to 7 levels): a byte per thread and plane
  const uint32_t planes = natural ? 0u : dither_planes(levels);
  uint8_t *plane0 = rec + dither_plane0(g.part_elems);
  const uint64_t plane_stride = dither_plane_bytes(g.part_elems);
  const uint32_t plane_bytes = planes ? (uint32_t)(4 * ru4(cdiv(d, 32))) : 0u;
  const uint64_t base = g.part_base(p);
  const Philox rng(seed, stream_id, p + g.part0);
#pragma unroll
  for (int row = 0; row < kRows; ++row) {
    const uint32_t j0 = tile * kTile + row * kRowElems + threadIdx.x * kPerThread;
    const uint32_t w = j0 >> 3;
    if (w >= n_words && w >= plane_bytes) continue;
    uint32_t rnd[8];
    rng.block(j0 >> 2, rnd);
    rng.block((j0 >> 2) + 1, rnd + 4);
    uint32_t word = 0, hi[3] = {0, 0, 0};
    float v8[8];
    source_at8(src, g, p, j0, d, lds, v8);
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
      uint32_t j = j0 + e;
      if (j < d) {
        float r;
        float v = v8[e];
        const uint32_t code = dither_one(v, nu, levels, natural, rnd[e], mags, &r);
        word |= (((code >> 6) << 3) | (code & 7u)) << (4 * e);
#pragma unroll
        for (int t = 0; t < 3; ++t) hi[t] |= ((code >> (3 + t)) & 1u) << e;
        if (residual) residual[base + j] = r;
      }
    }
    if (w < n_words) nibs[w] = word;
    if (w < plane_bytes) {
      for (uint32_t t = 0; t < planes; ++t) plane0[t * plane_stride + w] = (uint8_t)hi[t];
    }
  }
}

hipError_t dither_encode(const Geo &g_in, const bpc_params_t &prm_in, const Source &src_in, uint8_t *payload,
                         const Workspace &ws, hipStream_t stream) {
  // Full partitions that are a whole number of register tiles go to the single-pass kernel,
  // a ragged last partition (or everything, if the shape does not fit) to the passes below.
  // The single-pass kernels bound a shorter last partition through their buffer descriptors
  // (dword granularity, so an odd number of f16 gradient elements is left to the passes below).
  const bool ragged_ok = !(src_in.grad && src_in.dtype == BPC_F16 && (g_in.D & 1));
  const SplitGeo sp = split_geo(g_in, src_in.grad ? kWTile : kSTile, ragged_ok);
  Geo g = g_in;
  Source src = src_in;
  bpc_params_t prm = prm_in;
  uint32_t *status = ws.status();
  // (the single-pass server handles up to 15 levels; beyond that it declines and the server
  // side takes the passes below)
  const bool wide = prm_in.kind == BPC_DITHER && dither_planes(prm_in.levels) > 0;
  if (sp.single_pass && sp.head.P > 0) {
    bool used = false;
    hipError_t e = src.grad ? dither_worker_single_pass(sp.head, prm, src, payload, ws, stream, &used)
                            : dither_server_single_pass(sp.head, prm, src, payload, ws, stream, &used);
    if (e != hipSuccess) return e;
    if (used) {
      if (sp.tail.D == 0) return hipSuccess;
      advance_to_tail(sp.head.P, g_in, &src, &payload, &prm);
      g = sp.tail;
      status = nullptr;
    }
  }
  double *partials = ws.at<double>(ws.lay.partials);
  const int linf = prm.norm == BPC_NORM_LINF;
  const bool natural = prm.kind == BPC_NATDITHER;
  auto run = [&](auto s) -> hipError_t {
    using S = decltype(s);
    if (!prm.norm_override) dither_reduce_kernel<S><<<g.n_tiles, kThreads, 0, stream>>>(g, s, partials, linf);
    dither_finish_kernel<<<g.P, 64, 0, stream>>>(g, partials, prm.norm_override, linf, payload, status);
    dither_apply_kernel<S><<<g.n_tiles, kThreads, 0, stream>>>(g, s, payload, src.residual, prm.levels, natural, prm.seed,
                                                               prm.stream_id);
    return hipGetLastError();
  };
  if (wide && !src.grad) return run(DitherWideMsgSource{src.msgs, src.residual, g.stride, prm.levels});
  auto make_server = [&] { return DitherMsgSource{src.msgs, src.residual, g.stride, prm.levels, natural}; };
  return with_source(src, make_server, run);
}

}  // namespace bpc
