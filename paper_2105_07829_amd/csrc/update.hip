// Moment and parameter update of compressed LANS (Algorithm 5, the lines after the push-pull
// call), fused with the decode of the pulled message g~ = decode(p_t).
//   ADAM : one launch, x -= lr * (r + wd*x)
//   LANS : moments + block norms (||x_b||, ||r + wd x||_b, ||c + wd x||_b, f64 sums), then
//          x -= lr * phi(||x_b||) * (beta1 (r+wd x)/||.|| + (1-beta1) (c+wd x)/||.||)
#include "cluster_launch.hpp"
#include "sources.hpp"

#include <type_traits>

namespace bpc {

struct SignDec {
  const uint8_t *payload; uint64_t stride;
  __device__ const float *dense_base() const { return nullptr; }
  static constexpr int kLdsFloats = 1;
  __device__ void begin(uint32_t, float *) const {}
  __device__ float at(const Geo &, uint32_t p, uint32_t j, const float *) const {
    const uint8_t *rec = payload + (uint64_t)p * stride;
    float s = *reinterpret_cast<const float *>(rec);
    uint32_t w = reinterpret_cast<const uint32_t *>(rec + kHeaderBytes)[j >> 5];
    return ((w >> (j & 31)) & 1u) ? -s : s;
  }
  // 4 consecutive elements from j (a multiple of 4)
  __device__ void at4(const Geo &, uint32_t p, uint32_t j, const TileBuf &, const float *, float out[4]) const {
    const uint8_t *rec = payload + (uint64_t)p * stride;
    const float s = *reinterpret_cast<const float *>(rec);
    const uint32_t nib = rec[kHeaderBytes + (j >> 3)] >> (j & 4);
#pragma unroll
    for (int c = 0; c < 4; ++c) out[c] = ((nib >> c) & 1u) ? -s : s;
  }
  // The same in two steps, for callers that request a tile ahead of its use: the record's
  // header value and the raw bits first, the values later.
  using R4 = uint32_t;
  __device__ float header(uint32_t p) const { return *reinterpret_cast<const float *>(payload + (uint64_t)p * stride); }
  __device__ void table(float, float *) const {}
  __device__ R4 load4(const Geo &, uint32_t p, uint32_t j, const TileBuf &) const {
    return (payload + (uint64_t)p * stride)[kHeaderBytes + (j >> 3)];
  }
  __device__ void decode4(R4 r, uint32_t j, float hdr, const float *, float out[4]) const {
    const uint32_t nib = r >> (j & 4);
#pragma unroll
    for (int c = 0; c < 4; ++c) out[c] = ((nib >> c) & 1u) ? -hdr : hdr;
  }
};
struct DitherDec {
  const uint8_t *payload; uint64_t stride; uint32_t levels; bool natural;
  __device__ const float *dense_base() const { return nullptr; }
  static constexpr int kLdsFloats = 16;
  __device__ void begin(uint32_t p, float *lds) const {
    if (threadIdx.x < 16) {
      float nu = *reinterpret_cast<const float *>(payload + (uint64_t)p * stride);
      float mag = dither_mag(nu, threadIdx.x & 7, levels, natural);
      lds[threadIdx.x] = (threadIdx.x & 8) ? -mag : mag;
    }
    __syncthreads();
  }
  __device__ float at(const Geo &, uint32_t p, uint32_t j, const float *lds) const {
    const uint32_t *nibs = reinterpret_cast<const uint32_t *>(payload + (uint64_t)p * stride + kHeaderBytes);
    return lds[(nibs[j >> 3] >> (4 * (j & 7))) & 15u];
  }
  __device__ void at4(const Geo &, uint32_t p, uint32_t j, const TileBuf &, const float *lds, float out[4]) const {
    const uint32_t *nibs = reinterpret_cast<const uint32_t *>(payload + (uint64_t)p * stride + kHeaderBytes);
    const uint32_t w = nibs[j >> 3] >> (4 * (j & 4));
#pragma unroll
    for (int c = 0; c < 4; ++c) out[c] = lds[(w >> (4 * c)) & 15u];
  }
  using R4 = uint32_t;
  __device__ float header(uint32_t p) const { return *reinterpret_cast<const float *>(payload + (uint64_t)p * stride); }
  // all threads; the caller synchronises before and after
  __device__ void table(float nu, float *lds) const {
    if (threadIdx.x < 16) {
      float mag = dither_mag(nu, threadIdx.x & 7, levels, natural);
      lds[threadIdx.x] = (threadIdx.x & 8) ? -mag : mag;
    }
  }
  __device__ R4 load4(const Geo &, uint32_t p, uint32_t j, const TileBuf &) const {
    return reinterpret_cast<const uint32_t *>(payload + (uint64_t)p * stride + kHeaderBytes)[j >> 3];
  }
  __device__ void decode4(R4 r, uint32_t j, float, const float *lds, float out[4]) const {
    const uint32_t w = r >> (4 * (j & 4));
#pragma unroll
    for (int c = 0; c < 4; ++c) out[c] = lds[(w >> (4 * c)) & 15u];
  }
};
// Linear dithering with bit planes (more than 7 levels).  Table index = plane bits << 4 | nibble,
// i.e. (level bits 3..5, sign, level bits 0..2); entries beyond the levels in use are never read.
struct DitherWideDec {
  const uint8_t *payload; uint64_t stride; uint32_t levels; uint64_t part_elems;
  __device__ const float *dense_base() const { return nullptr; }
  static constexpr int kLdsFloats = 128;
  __device__ float entry(float nu, uint32_t e) const {
    const uint32_t level = (e & 7u) | ((e >> 4) << 3);
    const float mag = level <= levels ? dither_mag(nu, level, levels, false) : 0.0f;
    return (e & 8u) ? -mag : mag;
  }
  __device__ void begin(uint32_t p, float *lds) const {
    if (threadIdx.x < 128) lds[threadIdx.x] = entry(*reinterpret_cast<const float *>(payload + (uint64_t)p * stride), threadIdx.x);
    __syncthreads();
  }
  // The nibbles of 4 elements and the byte of each plane that holds their bits, as loaded:
  // nothing is combined here, so a caller that requests a tile ahead of its use does not wait
  // for the loads at the request.
  struct R4 { uint32_t nib, plane[3]; };
  __device__ float header(uint32_t p) const { return *reinterpret_cast<const float *>(payload + (uint64_t)p * stride); }
  __device__ void table(float nu, float *lds) const {
    if (threadIdx.x < 128) lds[threadIdx.x] = entry(nu, threadIdx.x);
  }
  __device__ R4 load4(const Geo &, uint32_t p, uint32_t j, const TileBuf &) const {
    const uint8_t *rec = payload + (uint64_t)p * stride;
    R4 r;
    r.nib = reinterpret_cast<const uint16_t *>(rec + kHeaderBytes)[j >> 2];
    const uint32_t planes = dither_planes(levels);
    const uint8_t *plane = rec + dither_plane0(part_elems) + (j >> 3);
    r.plane[0] = plane[0];
    r.plane[1] = planes > 1 ? plane[dither_plane_bytes(part_elems)] : 0u;
    r.plane[2] = planes > 2 ? plane[2 * dither_plane_bytes(part_elems)] : 0u;
    return r;
  }
  __device__ void decode4(R4 r, uint32_t j, float, const float *lds, float out[4]) const {
    uint32_t bits[3];
#pragma unroll
    for (uint32_t t = 0; t < 3; ++t) bits[t] = (r.plane[t] >> (j & 4u)) & 15u;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t nib = (r.nib >> (4 * c)) & 15u;
      const uint32_t hi = ((bits[0] >> c) & 1u) | (((bits[1] >> c) & 1u) << 1) | (((bits[2] >> c) & 1u) << 2);
      out[c] = lds[(hi << 4) | nib];
    }
  }
  // Load and decode in one place: the nibbles of 4 elements in bits 0..15, then 4 bits of each
  // plane in bits 16.., 20.., 24..
  __device__ void at4(const Geo &, uint32_t p, uint32_t j, const TileBuf &, const float *lds, float out[4]) const {
    const uint8_t *rec = payload + (uint64_t)p * stride;
    uint32_t r = reinterpret_cast<const uint16_t *>(rec + kHeaderBytes)[j >> 2];
    const uint32_t planes = dither_planes(levels);
    const uint8_t *plane = rec + dither_plane0(part_elems) + (j >> 3);
    for (uint32_t t = 0; t < planes; ++t)
      r |= (((uint32_t)plane[t * dither_plane_bytes(part_elems)] >> (j & 4)) & 15u) << (16 + 4 * t);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t nib = (r >> (4 * c)) & 15u;
      const uint32_t hi = ((r >> (16 + c)) & 1u) | (((r >> (20 + c)) & 1u) << 1) | (((r >> (24 + c)) & 1u) << 2);
      out[c] = lds[(hi << 4) | nib];
    }
  }
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *lds) const {
    float out[4];
    at4(g, p, j & ~3u, TileBuf(nullptr, 0), lds, out);
    const uint32_t c = j & 3u;
    return c == 0 ? out[0] : c == 1 ? out[1] : c == 2 ? out[2] : out[3];
  }
};
struct IdentityDec {
  const uint8_t *payload; uint64_t stride;
  __device__ const float *dense_base() const { return nullptr; }
  static constexpr int kLdsFloats = 1;
  __device__ void begin(uint32_t, float *) const {}
  __device__ float at(const Geo &, uint32_t p, uint32_t j, const float *) const {
    return reinterpret_cast<const float *>(payload + (uint64_t)p * stride + kHeaderBytes)[j];
  }
  // the record is padded to a full partition, so the 16 bytes are always inside it
  __device__ void at4(const Geo &, uint32_t p, uint32_t j, const TileBuf &, const float *, float out[4]) const {
    const float4 a = reinterpret_cast<const float4 *>(payload + (uint64_t)p * stride + kHeaderBytes)[j >> 2];
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
  }
  using R4 = u32x4;
  __device__ float header(uint32_t) const { return 0.0f; }
  __device__ void table(float, float *) const {}
  __device__ R4 load4(const Geo &, uint32_t p, uint32_t j, const TileBuf &) const {
    return reinterpret_cast<const u32x4 *>(payload + (uint64_t)p * stride + kHeaderBytes)[j >> 2];
  }
  __device__ void decode4(R4 r, uint32_t, float, const float *, float out[4]) const {
    out[0] = __uint_as_float(r.x); out[1] = __uint_as_float(r.y); out[2] = __uint_as_float(r.z); out[3] = __uint_as_float(r.w);
  }
};
struct Fp16Dec {
  const uint8_t *payload; uint64_t stride;
  __device__ const float *dense_base() const { return nullptr; }
  static constexpr int kLdsFloats = 1;
  __device__ void begin(uint32_t, float *) const {}
  __device__ float at(const Geo &, uint32_t p, uint32_t j, const float *) const {
    return __half2float(reinterpret_cast<const __half *>(payload + (uint64_t)p * stride + kHeaderBytes)[j]);
  }
  using R4 = u32x2;
  __device__ float header(uint32_t) const { return 0.0f; }
  __device__ void table(float, float *) const {}
  // the record is padded to a full partition, so the 8 bytes are always inside it
  __device__ R4 load4(const Geo &, uint32_t p, uint32_t j, const TileBuf &) const {
    return reinterpret_cast<const u32x2 *>(payload + (uint64_t)p * stride + kHeaderBytes)[j >> 2];
  }
  __device__ void decode4(R4 r, uint32_t, float, const float *, float out[4]) const {
    const uint32_t lo = r.x, hi = r.y;
    const float2 a = __half22float2(*reinterpret_cast<const __half2 *>(&lo));
    const float2 b = __half22float2(*reinterpret_cast<const __half2 *>(&hi));
    out[0] = a.x; out[1] = a.y; out[2] = b.x; out[3] = b.y;
  }
  __device__ void at4(const Geo &g, uint32_t p, uint32_t j, const TileBuf &row, const float *lds, float out[4]) const {
    decode4(load4(g, p, j, row), j, 0.0f, lds, out);
  }
};
struct DenseDec {
  const float *dense;
  __device__ const float *dense_base() const { return dense; }
  static constexpr int kLdsFloats = 1;
  __device__ void begin(uint32_t, float *) const {}
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *) const { return dense[g.part_base(p) + j]; }
  // `row` bounds the row this thread's 4 elements belong to (the same descriptor in every
  // lane); reads past the partition's end return 0
  __device__ void at4(const Geo &, uint32_t, uint32_t, const TileBuf &row, const float *, float out[4]) const {
    const u32x4 lo = row.load16<kNonTemporal>(threadIdx.x * 16, 0);
    out[0] = __uint_as_float(lo.x); out[1] = __uint_as_float(lo.y); out[2] = __uint_as_float(lo.z); out[3] = __uint_as_float(lo.w);
  }
  using R4 = u32x4;
  __device__ float header(uint32_t) const { return 0.0f; }
  __device__ void table(float, float *) const {}
  __device__ R4 load4(const Geo &, uint32_t, uint32_t, const TileBuf &row) const { return row.load16<kNonTemporal>(threadIdx.x * 16, 0); }
  __device__ void decode4(R4 r, uint32_t, float, const float *, float out[4]) const {
    out[0] = __uint_as_float(r.x); out[1] = __uint_as_float(r.y); out[2] = __uint_as_float(r.z); out[3] = __uint_as_float(r.w);
  }
};

// Top-k and random-k messages without a dense decode: the entries of a tile of kTile elements
// are one stretch of a list (top-k: of the record itself, whose entries come by ascending
// index; random-k: of the record's draws binned per tile beforehand), found through a table of
// where each tile's stretch starts, and laid out in LDS by the workgroup that has the tile.
template <int TILE, int THREADS>
struct SparseTileDec {
  const uint8_t *payload;
  uint64_t stride;
  uint32_t k_cap;
  int mode;                  // 0: top-k, f32 values; 1: top-k, half values; 2: random-k pairs
  const uint32_t *starts;    // [partition][tile .. ], `starts_stride` words a partition
  uint32_t starts_stride;
  const uint2 *pairs;        // random-k: [partition][k_cap]
  __device__ const float *dense_base() const { return nullptr; }
  static constexpr int kLdsFloats = TILE;
  __device__ void begin(uint32_t, float *) const {}
  __device__ void begin_tile(uint32_t p, uint32_t tile, float *lds) const {
    __syncthreads();   // (the tile before is done with)
    for (uint32_t q = threadIdx.x; q < TILE / 4; q += THREADS) reinterpret_cast<float4 *>(lds)[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    const uint8_t *rec = payload + (uint64_t)p * stride;
    uint32_t k = *reinterpret_cast<const uint32_t *>(rec);
    k = k > k_cap ? k_cap : k;
    const uint32_t *tab = starts + (uint64_t)p * starts_stride;
    uint32_t s = tab[tile], e = tab[tile + 1];
    s = s < k ? s : k;
    e = e < k ? e : k;
    const uint32_t lo = tile * TILE;
    __syncthreads();
    if (mode == 2) {
      const uint2 *list = pairs + (uint64_t)p * k_cap;
      for (uint32_t q = s + threadIdx.x; q < e; q += THREADS) {
        const uint2 ent = list[q];
        if (ent.x - lo < (uint32_t)TILE) atomicAdd(&lds[ent.x - lo], __uint_as_float(ent.y));   // an index may repeat
      }
    } else {
      const uint32_t *idx = reinterpret_cast<const uint32_t *>(rec + kHeaderBytes);
      const uint8_t *val = rec + kHeaderBytes + 4 * ru4(k_cap);
      for (uint32_t q = s + threadIdx.x; q < e; q += THREADS) {
        const uint32_t rel = idx[q] - lo;
        const float v = mode == 1 ? __half2float(reinterpret_cast<const __half *>(val)[q]) : reinterpret_cast<const float *>(val)[q];
        if (rel < (uint32_t)TILE) lds[rel] = v;
      }
    }
    __syncthreads();
  }
  __device__ void at4(const Geo &, uint32_t, uint32_t j, const TileBuf &, const float *lds, float out[4]) const {
    const float4 f = *reinterpret_cast<const float4 *>(lds + (j & (TILE - 1)));
    out[0] = f.x; out[1] = f.y; out[2] = f.z; out[3] = f.w;
  }
  // (the forms the single-pass LANS kernel uses: nothing to request ahead, the tile is in LDS)
  using R4 = uint32_t;
  __device__ float header(uint32_t) const { return 0.0f; }
  __device__ void table(float, float *) const {}
  __device__ R4 load4(const Geo &, uint32_t, uint32_t, const TileBuf &) const { return 0u; }
  __device__ void decode4(R4, uint32_t j, float, const float *lds, float out[4]) const {
    const float4 f = *reinterpret_cast<const float4 *>(lds + (j & (TILE - 1)));
    out[0] = f.x; out[1] = f.y; out[2] = f.z; out[3] = f.w;
  }
};
template <class DEC, class = void>
struct has_begin_tile : std::false_type {};
template <class DEC>
struct has_begin_tile<DEC, std::void_t<decltype(&DEC::begin_tile)>> : std::true_type {};

struct OptArgs {
  float lr, beta1, beta2, eps, wd, bc1, bc2, phi_lo, phi_hi;
  const uint64_t *block_offsets;  // device, or NULL: blocks are the partitions
  uint64_t n_blocks;
  uint32_t *status;               // the workspace's status word (cleared by kernels that have no waits)
};

// r + wd*x and c + wd*x from the updated moments.
__device__ inline void ratios(const OptArgs &o, float g, float m, float v, float x, float *u_r, float *u_c) {
  float m_hat = m / o.bc1;
  float v_hat = v / o.bc2;
  float denom = sqrtf(v_hat) + o.eps;
  float decay = o.wd * x;
  *u_r = m_hat / denom + decay;
  *u_c = g / denom + decay;
}

// The same for the single-pass LANS kernel, which is bound by its arithmetic: the bias
// corrections as factors, and the hardware's reciprocal and square root (1 ulp each) in place
// of the correctly rounded sequences.  r and c differ from the divisions above by a few ulp;
// in x that is far inside the 1e-6 the update is held to.
__device__ inline void ratios_fast(const OptArgs &o, float inv_bc1, float inv_bc2, float g, float m, float v, float x,
                                   float *u_r, float *u_c) {
  float m_hat = m * inv_bc1;
  float v_hat = v * inv_bc2;
  float inv = __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(v_hat) + o.eps);
  float decay = o.wd * x;
  *u_r = m_hat * inv + decay;
  *u_c = g * inv + decay;
}

__device__ inline uint32_t find_block(const uint64_t *offs, uint64_t n_blocks, uint64_t i) {
  uint64_t lo = 0, hi = n_blocks;  // offs[lo] <= i < offs[hi]
  while (hi - lo > 1) {
    uint64_t mid = (lo + hi) / 2;
    if (offs[mid] <= i) lo = mid; else hi = mid;
  }
  return (uint32_t)lo;
}

template <class DEC, bool LANS>
__global__ __launch_bounds__(kThreads) void update_moments_kernel(Geo g, DEC dec, float *x, float *m, float *v,
                                                                  OptArgs o, double *norms) {
  __shared__ float lds[DEC::kLdsFloats];
  __shared__ double red[kThreads / 64];
  if (blockIdx.x == 0 && threadIdx.x == 0) o.status[0] = 0;   // no wait in this call
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  dec.begin(p, lds);
  const uint64_t base = g.part_base(p);
  const float omb1 = 1.0f - o.beta1, omb2 = 1.0f - o.beta2;
  // LANS: does this whole tile lie in one block?
  uint32_t blk_first = p, blk_last = p;
  if (LANS && o.block_offsets) {
    uint32_t j_last = (tile + 1) * kTile - 1;
    j_last = j_last < d ? j_last : d - 1;
    blk_first = find_block(o.block_offsets, o.n_blocks, base + tile * kTile);
    blk_last = find_block(o.block_offsets, o.n_blocks, base + j_last);
  }
  const bool one_block = blk_first == blk_last;
  double s_x = 0.0, s_r = 0.0, s_c = 0.0;
#pragma unroll
  for (int c = 0; c < kTile / kThreads; ++c) {
    uint32_t j = tile * kTile + c * kThreads + threadIdx.x;
    if (j < d) {
      uint64_t i = base + j;
      float gj = dec.at(g, p, j, lds);
      float mj = o.beta1 * m[i] + omb1 * gj;
      float vj = o.beta2 * v[i] + omb2 * (gj * gj);
      m[i] = mj;
      v[i] = vj;
      float xj = x[i], u_r, u_c;
      ratios(o, gj, mj, vj, xj, &u_r, &u_c);
      if (!LANS) {
        x[i] = xj - o.lr * u_r;
      } else if (one_block) {
        s_x = fma((double)xj, (double)xj, s_x);
        s_r = fma((double)u_r, (double)u_r, s_r);
        s_c = fma((double)u_c, (double)u_c, s_c);
      } else {
        uint32_t b = find_block(o.block_offsets, o.n_blocks, i);
        atomicAdd(&norms[3 * (uint64_t)b + 0], (double)xj * (double)xj);
        atomicAdd(&norms[3 * (uint64_t)b + 1], (double)u_r * (double)u_r);
        atomicAdd(&norms[3 * (uint64_t)b + 2], (double)u_c * (double)u_c);
      }
    }
  }
  if (LANS && one_block) {
    double t_x = block_sum<kThreads>(s_x, red);
    double t_r = block_sum<kThreads>(s_r, red);
    double t_c = block_sum<kThreads>(s_c, red);
    if (threadIdx.x == 0) {
      atomicAdd(&norms[3 * (uint64_t)blk_first + 0], t_x);
      atomicAdd(&norms[3 * (uint64_t)blk_first + 1], t_r);
      atomicAdd(&norms[3 * (uint64_t)blk_first + 2], t_c);
    }
  }
}

// ADAM in one pass.  A thread owns 4 consecutive elements per row of 1024, so every 16-byte
// access of a wave covers whole cache lines (which is what lets the stores be non-temporal);
// all loads of a tile are requested before the first is used.  x, m and v go through buffer
// descriptors that end with the partition: reads past it return 0 and stores past it are
// dropped, so a ragged last tile needs no other care.
constexpr int kURow = kThreads * 4;
constexpr int kURows = kTile / kURow;
template <class DEC>
__global__ __launch_bounds__(kThreads) void adam_update_kernel(Geo g, DEC dec, float *x, float *m, float *v, OptArgs o) {
  __shared__ __align__(16) float lds[DEC::kLdsFloats];
  if (blockIdx.x == 0 && threadIdx.x == 0) o.status[0] = 0;   // no wait in this call
  const uint32_t p = __builtin_amdgcn_readfirstlane(blockIdx.x / g.tiles_per_part);
  const uint32_t tile = __builtin_amdgcn_readfirstlane(blockIdx.x % g.tiles_per_part);
  const uint32_t d = g.part_size(p);
  dec.begin(p, lds);
  const uint64_t tile_base = g.part_base(p) + (uint64_t)tile * kTile;
  const uint32_t valid = d - tile * kTile < (uint32_t)kTile ? d - tile * kTile : (uint32_t)kTile;
  const float omb1 = 1.0f - o.beta1, omb2 = 1.0f - o.beta2;
  u32x4 xr[kURows], mr[kURows], vr[kURows];
  if constexpr (has_begin_tile<DEC>::value) {
    // the loads of m, v, x are requested first, so they are under way while the tile of the
    // message is laid out in LDS
#pragma unroll
    for (int u = 0; u < kURows; ++u) {
      mr[u] = row_buf(m + tile_base, valid, u * kURow, kURow).load16<kNonTemporal>(threadIdx.x * 16, 0);
      vr[u] = row_buf(v + tile_base, valid, u * kURow, kURow).load16<kNonTemporal>(threadIdx.x * 16, 0);
      xr[u] = row_buf(x + tile_base, valid, u * kURow, kURow).load16<kNonTemporal>(threadIdx.x * 16, 0);
    }
    dec.begin_tile(p, tile, lds);
  }
  float gr[kURows][4];
#pragma unroll
  for (int u = 0; u < kURows; ++u) {
    if constexpr (!has_begin_tile<DEC>::value) {
      mr[u] = row_buf(m + tile_base, valid, u * kURow, kURow).load16<kNonTemporal>(threadIdx.x * 16, 0);
      vr[u] = row_buf(v + tile_base, valid, u * kURow, kURow).load16<kNonTemporal>(threadIdx.x * 16, 0);
      xr[u] = row_buf(x + tile_base, valid, u * kURow, kURow).load16<kNonTemporal>(threadIdx.x * 16, 0);
    }
    const uint32_t j = tile * kTile + u * kURow + threadIdx.x * 4;
    dec.at4(g, p, j, row_buf(dec.dense_base() + tile_base, valid, u * kURow, kURow), lds, gr[u]);
  }
#pragma unroll
  for (int u = 0; u < kURows; ++u) {
    const uint32_t mi[4] = {mr[u].x, mr[u].y, mr[u].z, mr[u].w};
    const uint32_t vi[4] = {vr[u].x, vr[u].y, vr[u].z, vr[u].w};
    const uint32_t xi[4] = {xr[u].x, xr[u].y, xr[u].z, xr[u].w};
    float mo[4], vo[4], xo[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float gj = gr[u][c];
      const float mj = o.beta1 * __uint_as_float(mi[c]) + omb1 * gj;
      const float vj = o.beta2 * __uint_as_float(vi[c]) + omb2 * (gj * gj);
      const float xj = __uint_as_float(xi[c]);
      float u_r, u_c;
      ratios(o, gj, mj, vj, xj, &u_r, &u_c);
      mo[c] = mj;
      vo[c] = vj;
      xo[c] = xj - o.lr * u_r;
    }
    row_buf(m + tile_base, valid, u * kURow, kURow).store16<kNonTemporal>(as_u32x4(mo[0], mo[1], mo[2], mo[3]), threadIdx.x * 16);
    row_buf(v + tile_base, valid, u * kURow, kURow).store16<kNonTemporal>(as_u32x4(vo[0], vo[1], vo[2], vo[3]), threadIdx.x * 16);
    row_buf(x + tile_base, valid, u * kURow, kURow).store16<kNonTemporal>(as_u32x4(xo[0], xo[1], xo[2], xo[3]), threadIdx.x * 16);
  }
}

// LANS in one pass when the blocks are the partitions.  A workgroup (1024 threads, 8 elements
// a thread, an 8192-element tile; tiles at a fixed stride, the grid resident as a whole)
// updates and stores the moments, keeps x, r + wd x and c + wd x in registers and publishes its
// three partial square sums (one f64 slot each, as in cluster.hpp).  It writes a tile's x
// only after phase 1 of its next tile: by then the other tiles of the older tile's partition
// have been published, so collecting the three totals is one read of the slots, and the loads
// of the next tile are already under way.  Sums are combined in slot order, so the result
// does not depend on timing.  Same traffic as ADAM: payload, m, v, x read once, m, v, x
// written once.
constexpr int kLThreads = 1024;
constexpr int kLPer = kSTile / kLThreads;   // 8
constexpr int kLRows = kLPer / 4;           // 2 rows of 4096 elements, 4 consecutive a thread
constexpr int kLRow = kLThreads * 4;

struct LansTile {
  uint32_t p, tile, valid, tiles_in_part;
  uint64_t base;
};
__device__ inline LansTile lans_tile(const Geo &g, const ClusterGeo &cg, uint32_t item) {
  LansTile t;
  t.p = __builtin_amdgcn_readfirstlane(item / cg.tiles_per_part);
  t.tile = __builtin_amdgcn_readfirstlane(item % cg.tiles_per_part);
  const uint32_t d = g.part_size(t.p);
  t.tiles_in_part = (uint32_t)cdiv(d, kSTile);
  t.base = uniform_off(g.part_base(t.p) + (uint64_t)t.tile * kSTile);
  const uint32_t left = d - t.tile * kSTile;
  t.valid = __builtin_amdgcn_readfirstlane(left < (uint32_t)kSTile ? left : (uint32_t)kSTile);
  return t;
}
template <class DEC>
struct LansRaw {
  u32x4 m[kLRows], v[kLRows], x[kLRows];
  typename DEC::R4 g[kLRows];
  float hdr;
};
struct LansHeld { float xs[kLPer], ur[kLPer], uc[kLPer]; };

template <class DEC>
__device__ inline void lans_issue(const Geo &g, const ClusterGeo &cg, const DEC &dec, const float *x, const float *m,
                                  const float *v, uint32_t item, LansRaw<DEC> &raw) {
  const LansTile t = lans_tile(g, cg, item);
  raw.hdr = dec.header(t.p);
#pragma unroll
  for (int u = 0; u < kLRows; ++u) {
    raw.m[u] = row_buf(m + t.base, t.valid, u * kLRow, kLRow).load16<kNonTemporal>(threadIdx.x * 16, 0);
    raw.v[u] = row_buf(v + t.base, t.valid, u * kLRow, kLRow).load16<kNonTemporal>(threadIdx.x * 16, 0);
    raw.x[u] = row_buf(x + t.base, t.valid, u * kLRow, kLRow).load16<kNonTemporal>(threadIdx.x * 16, 0);
    const uint32_t j = t.tile * kSTile + u * kLRow + threadIdx.x * 4;
    raw.g[u] = dec.load4(g, t.p, j, row_buf(dec.dense_base() + t.base, t.valid, u * kLRow, kLRow));
  }
}

// First wave: the three totals of a partition once all its tiles have published theirs.
__device__ inline void lans_collect(const OptArgs &o, const double *ps, uint32_t tiles_in_part, uint32_t *status,
                                    float *weights_sh) {
  const uint32_t lane = threadIdx.x;
  double a0, a1, a2;
  int spins = 0;
  for (;;) {
    bool ok = true;
    a0 = 0.0; a1 = 0.0; a2 = 0.0;
    for (uint32_t s = lane; s < tiles_in_part; s += 64) {
      const double q0 = __hip_atomic_load(ps + 3 * s + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const double q1 = __hip_atomic_load(ps + 3 * s + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const double q2 = __hip_atomic_load(ps + 3 * s + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ok = ok && slot_published(q0) && slot_published(q1) && slot_published(q2);
      a0 += slot_published(q0) ? q0 : 0.0;
      a1 += slot_published(q1) ? q1 : 0.0;
      a2 += slot_published(q2) ? q2 : 0.0;
    }
    if (__all(ok)) break;
    if (++spins > kSpinLimit) {
      if (lane == 0) atomicOr(status, 1u);
      break;
    }
    __builtin_amdgcn_s_sleep(16);
  }
  a0 = wave_sum(a0);
  a1 = wave_sum(a1);
  a2 = wave_sum(a2);
  if (lane == 0) {
    // phi(||x||) and the two weights beta1 / ||r + wd x||, (1 - beta1) / ||c + wd x||, once per tile
    // (three square roots of doubles and two divisions: as much arithmetic as a thread's eight
    // elements take, when every thread did them)
    const float norm_x = (float)sqrt(a0);
    const float norm_r = (float)sqrt(a1);
    const float norm_c = (float)sqrt(a2);
    float phi = norm_x < o.phi_lo ? o.phi_lo : norm_x;
    phi = phi > o.phi_hi ? o.phi_hi : phi;
    weights_sh[0] = phi;
    weights_sh[1] = norm_r > 0.0f ? o.beta1 / norm_r : 0.0f;
    weights_sh[2] = norm_c > 0.0f ? (1.0f - o.beta1) / norm_c : 0.0f;
  }
}

// x of a tile whose partition's phi and weights are in weights_sh.
__device__ inline void lans_write_x(const Geo &g, const ClusterGeo &cg, const OptArgs &o, float *x, uint32_t item,
                                    const LansHeld &h, const float *weights_sh) {
  const LansTile t = lans_tile(g, cg, item);
  const float phi = weights_sh[0], w_r = weights_sh[1], w_c = weights_sh[2];
#pragma unroll
  for (int u = 0; u < kLRows; ++u) {
    float xo[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float dir = phi * (w_r * h.ur[4 * u + c] + w_c * h.uc[4 * u + c]);
      xo[c] = h.xs[4 * u + c] - o.lr * dir;
    }
    row_buf(x + t.base, t.valid, u * kLRow, kLRow).store16<kNonTemporal>(as_u32x4(xo[0], xo[1], xo[2], xo[3]), threadIdx.x * 16);
  }
}

template <class DEC>
__global__ __launch_bounds__(kLThreads) void lans_single_kernel(Geo g, ClusterGeo cg, DEC dec, float *x, float *m, float *v,
                                                               OptArgs o, double *slots, uint32_t *status) {
  __shared__ __align__(16) float lds[DEC::kLdsFloats];
  __shared__ double red3[3 * (kLThreads / 64)];
  __shared__ float total_sh[3];   // phi and the two weights of the tile being written
  constexpr uint32_t kNone = 0xffffffffu;
  uint32_t item = __builtin_amdgcn_readfirstlane(blockIdx.x);
  if (item >= cg.n_items) return;
  LansRaw<DEC> raw;
  lans_issue(g, cg, dec, x, m, v, item, raw);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the loop is entered with nothing in flight
  LansHeld prev_h;
  uint32_t prev = kNone;
  const float omb1 = 1.0f - o.beta1, omb2 = 1.0f - o.beta2;
  const float inv_bc1 = 1.0f / o.bc1, inv_bc2 = 1.0f / o.bc2;
  for (;;) {
    const LansTile t = lans_tile(g, cg, item);
    if constexpr (has_begin_tile<DEC>::value) {
      dec.begin_tile(t.p, t.tile, lds);   // the tile of the message, laid out in LDS
    } else {
      __syncthreads();   // the table of the tile before
      dec.table(raw.hdr, lds);
      __syncthreads();
    }
    LansHeld h;
    // a thread's eight squares are summed in f32 (a relative error of a few 1e-7 in its share,
    // the same order as the reciprocals of `ratios_fast`), everything above that in f64
    float f_x = 0.0f, f_r = 0.0f, f_c = 0.0f;
#pragma unroll
    for (int u = 0; u < kLRows; ++u) {
      const uint32_t mi[4] = {raw.m[u].x, raw.m[u].y, raw.m[u].z, raw.m[u].w};
      const uint32_t vi[4] = {raw.v[u].x, raw.v[u].y, raw.v[u].z, raw.v[u].w};
      const uint32_t xi[4] = {raw.x[u].x, raw.x[u].y, raw.x[u].z, raw.x[u].w};
      float gr[4];
      dec.decode4(raw.g[u], t.tile * kSTile + u * kLRow + threadIdx.x * 4, raw.hdr, lds, gr);
      float mo[4], vo[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float gj = gr[c];
        const float mj = o.beta1 * __uint_as_float(mi[c]) + omb1 * gj;
        const float vj = o.beta2 * __uint_as_float(vi[c]) + omb2 * (gj * gj);
        const float xj = __uint_as_float(xi[c]);
        float u_r, u_c;
        ratios_fast(o, inv_bc1, inv_bc2, gj, mj, vj, xj, &u_r, &u_c);
        mo[c] = mj;
        vo[c] = vj;
        // what the padded record decodes to past the partition's end takes no part in the norms
        const bool in = (uint32_t)(u * kLRow) + threadIdx.x * 4 + c < t.valid;
        h.xs[4 * u + c] = xj;
        h.ur[4 * u + c] = u_r;
        h.uc[4 * u + c] = u_c;
        f_x = in ? fmaf(xj, xj, f_x) : f_x;
        f_r = in ? fmaf(u_r, u_r, f_r) : f_r;
        f_c = in ? fmaf(u_c, u_c, f_c) : f_c;
      }
      row_buf(m + t.base, t.valid, u * kLRow, kLRow).store16<kNonTemporal>(as_u32x4(mo[0], mo[1], mo[2], mo[3]), threadIdx.x * 16);
      row_buf(v + t.base, t.valid, u * kLRow, kLRow).store16<kNonTemporal>(as_u32x4(vo[0], vo[1], vo[2], vo[3]), threadIdx.x * 16);
    }
    const uint32_t next = __builtin_amdgcn_readfirstlane(item + gridDim.x);
    const bool have_next = next < cg.n_items;
    if (have_next) lans_issue(g, cg, dec, x, m, v, next, raw);
    // the three sums over the workgroup: a tree in f32 inside each wave (six levels, the same
    // order of error as the threads' own sums; shuffling doubles cost a tenth of the kernel's
    // instructions), the 16 waves' sums in f64 in fixed order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      f_x = f_x + __shfl_xor(f_x, off, 64);
      f_r = f_r + __shfl_xor(f_r, off, 64);
      f_c = f_c + __shfl_xor(f_c, off, 64);
    }
    __syncthreads();   // (red3 of the tile before has been read)
    if ((threadIdx.x & 63) == 0) {
      red3[3 * (threadIdx.x >> 6) + 0] = (double)f_x;
      red3[3 * (threadIdx.x >> 6) + 1] = (double)f_r;
      red3[3 * (threadIdx.x >> 6) + 2] = (double)f_c;
    }
    __syncthreads();
    double t_x = 0.0, t_r = 0.0, t_c = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
      for (int w = 0; w < kLThreads / 64; ++w) {
        t_x += red3[3 * w + 0];
        t_r += red3[3 * w + 1];
        t_c += red3[3 * w + 2];
      }
    }
    if (threadIdx.x == 0) {
      // slot 3*tile + k of the partition holds this tile's k-th partial
      double *ps = slots + 3ull * t.p * cg.tiles_per_part;
      slot_publish(ps + 3 * t.tile + 0, t_x);
      slot_publish(ps + 3 * t.tile + 1, t_r);
      slot_publish(ps + 3 * t.tile + 2, t_c);
    }
    if (prev != kNone && threadIdx.x < 64) {
      const LansTile tp = lans_tile(g, cg, prev);
      lans_collect(o, slots + 3ull * tp.p * cg.tiles_per_part, tp.tiles_in_part, status, total_sh);
    }
    __syncthreads();
    if (prev != kNone) lans_write_x(g, cg, o, x, prev, prev_h, total_sh);
    prev_h = h;
    prev = item;
    if (!have_next) break;
    item = next;
  }
  // the last tile
  __syncthreads();
  if (threadIdx.x < 64) {
    const LansTile tp = lans_tile(g, cg, prev);
    lans_collect(o, slots + 3ull * tp.p * cg.tiles_per_part, tp.tiles_in_part, status, total_sh);
  }
  __syncthreads();
  lans_write_x(g, cg, o, x, prev, prev_h, total_sh);
}

template <class DEC>
__global__ __launch_bounds__(kThreads) void lans_apply_kernel(Geo g, DEC dec, float *x, const float *m,
                                                              const float *v, OptArgs o, const double *norms) {
  __shared__ float lds[DEC::kLdsFloats];
  const uint32_t p = blockIdx.x / g.tiles_per_part;
  const uint32_t tile = blockIdx.x % g.tiles_per_part;
  const uint32_t d = g.part_size(p);
  dec.begin(p, lds);
  const uint64_t base = g.part_base(p);
  const float omb1 = 1.0f - o.beta1;
#pragma unroll
  for (int c = 0; c < kTile / kThreads; ++c) {
    uint32_t j = tile * kTile + c * kThreads + threadIdx.x;
    if (j < d) {
      uint64_t i = base + j;
      uint32_t b = o.block_offsets ? find_block(o.block_offsets, o.n_blocks, i) : p;
      float norm_x = (float)sqrt(norms[3 * (uint64_t)b + 0]);
      float norm_r = (float)sqrt(norms[3 * (uint64_t)b + 1]);
      float norm_c = (float)sqrt(norms[3 * (uint64_t)b + 2]);
      float phi = norm_x < o.phi_lo ? o.phi_lo : norm_x;
      phi = phi > o.phi_hi ? o.phi_hi : phi;
      float w_r = norm_r > 0.0f ? o.beta1 / norm_r : 0.0f;
      float w_c = norm_c > 0.0f ? omb1 / norm_c : 0.0f;
      float gj = dec.at(g, p, j, lds);
      float xj = x[i], u_r, u_c;
      ratios(o, gj, m[i], v[i], xj, &u_r, &u_c);
      float dir = phi * (w_r * u_r + w_c * u_c);
      x[i] = xj - o.lr * dir;
    }
  }
}

// LANS with the partitions as blocks, one pass.  *used = false: shape not supported.
template <class DEC>
static hipError_t run_lans_single(const Geo &g, DEC dec, float *x, float *m, float *v, const OptArgs &o,
                                  const Workspace &ws, hipStream_t stream, bool *used) {
  *used = false;
  if (g.part_elems % kSTile != 0) return hipSuccess;
  const ClusterGeo cg = make_cluster_geo(g, kSTile);
  static PerDevice cache;
  const int capacity = cache.get([] { return cluster_capacity(reinterpret_cast<const void *>(&lans_single_kernel<DEC>), kLThreads, 0); });
  if (capacity <= 0 || cg.tiles_per_part > (uint32_t)capacity) return hipSuccess;
  *used = true;
  double *slots = ws.at<double>(ws.lay.slots);
  uint32_t *status = ws.at<uint32_t>(ws.lay.status);
  hipError_t e = cluster_launch_begin(stream);
  if (e != hipSuccess) return e;
  const uint32_t n_slots = 3 * g.P * cg.tiles_per_part;
  slots_reset_kernel<<<(uint32_t)cdiv(n_slots, 256), 256, 0, stream>>>(slots, n_slots, status);
  const uint32_t grid = cg.n_items > (uint32_t)capacity ? (uint32_t)capacity : cg.n_items;
  lans_single_kernel<DEC><<<grid, kLThreads, 0, stream>>>(g, cg, dec, x, m, v, o, slots, status);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  return cluster_launch_end(stream);
}

template <class DEC>
static hipError_t run_update(const Geo &g, DEC dec, float *x, float *m, float *v, const bpc_opt_t &opt,
                             double *norms, const Workspace &ws, hipStream_t stream) {
  OptArgs o{opt.lr, opt.beta1, opt.beta2, opt.eps, opt.weight_decay, opt.bias_corr1, opt.bias_corr2,
            opt.phi_lo, opt.phi_hi, opt.block_offsets, opt.n_blocks, ws.at<uint32_t>(ws.lay.status)};
  if (opt.kind == BPC_OPT_ADAM) {
    adam_update_kernel<DEC><<<g.n_tiles, kThreads, 0, stream>>>(g, dec, x, m, v, o);
    return hipGetLastError();
  }
  if (!opt.block_offsets) {
    bool used = false;
    hipError_t e1 = run_lans_single(g, dec, x, m, v, o, ws, stream, &used);
    if (e1 != hipSuccess || used) return e1;
  }
  uint64_t nb = opt.block_offsets ? opt.n_blocks : g.P;
  hipError_t e = fill_zero(norms, sizeof(double) * 3 * nb, stream);
  if (e != hipSuccess) return e;
  update_moments_kernel<DEC, true><<<g.n_tiles, kThreads, 0, stream>>>(g, dec, x, m, v, o, norms);
  lans_apply_kernel<DEC><<<g.n_tiles, kThreads, 0, stream>>>(g, dec, x, m, v, o, norms);
  return hipGetLastError();
}

hipError_t adaptive_update(const Geo &g, const bpc_params_t &prm, const uint8_t *payload, float *x, float *m,
                           float *v, const bpc_opt_t &opt, const Workspace &ws, hipStream_t stream) {
  double *norms = ws.at<double>(ws.lay.norms);
  switch (prm.kind) {
    case BPC_SIGN: return run_update(g, SignDec{payload, g.stride}, x, m, v, opt, norms, ws, stream);
    case BPC_DITHER: case BPC_NATDITHER:
      if (prm.kind == BPC_DITHER && dither_planes(prm.levels) > 0) {
        return run_update(g, DitherWideDec{payload, g.stride, prm.levels, g.part_elems}, x, m, v, opt, norms, ws, stream);
      }
      return run_update(g, DitherDec{payload, g.stride, prm.levels, prm.kind == BPC_NATDITHER}, x, m, v, opt, norms, ws, stream);
    case BPC_IDENTITY: return run_update(g, IdentityDec{payload, g.stride}, x, m, v, opt, norms, ws, stream);
    case BPC_FP16: return run_update(g, Fp16Dec{payload, g.stride}, x, m, v, opt, norms, ws, stream);
    default: break;
  }
  float *dense = ws.at<float>(ws.lay.dense);
  const bool lans_single = opt.kind == BPC_OPT_LANS && !opt.block_offsets && g.part_elems % kSTile == 0;
  if ((opt.kind == BPC_OPT_ADAM || lans_single) && (prm.kind == BPC_TOPK || prm.kind == BPC_TOPK16 || prm.kind == BPC_RANDK)) {
    // no dense decode: the update kernel lays each tile of the message out in LDS itself
    // (tiles of 4096 elements in the Adam-style kernel, of 8192 in the single-pass LANS kernel)
    OptArgs o{opt.lr, opt.beta1, opt.beta2, opt.eps, opt.weight_decay, opt.bias_corr1, opt.bias_corr2,
              opt.phi_lo, opt.phi_hi, opt.block_offsets, opt.n_blocks, ws.at<uint32_t>(ws.lay.status)};
    const uint32_t shift = lans_single ? 13 : 12;
    const uint32_t tiles = (uint32_t)cdiv(g.part_elems, 1ull << shift);
    const uint32_t *table = nullptr;
    const uint2 *pairs = nullptr;
    uint32_t table_stride = 0;
    int mode = -1;
    if (prm.kind == BPC_RANDK) {
      const uint64_t list_bytes = ((uint64_t)g.P * g.k_cap * sizeof(uint2) + 255) / 256 * 256;
      const uint64_t table_bytes = (uint64_t)g.P * kRandkTableStride * sizeof(uint32_t);
      if (tiles <= 1024 && list_bytes + table_bytes <= sizeof(float) * g.D) {
        uint2 *lists = reinterpret_cast<uint2 *>(dense);   // (the dense workspace is free on this path)
        uint32_t *tab = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(dense) + list_bytes);
        hipError_t e = randk_bin_tiles(g, prm, payload, lists, tab, shift, stream);
        if (e != hipSuccess) return e;
        table = tab; pairs = lists; table_stride = kRandkTableStride; mode = 2;
      }
    } else {
      uint32_t *tab = ws.at<uint32_t>(ws.lay.starts);
      const bool half = prm.kind == BPC_TOPK16;
      hipError_t e = topk_tile_starts(g, payload, half, tab, shift, stream);
      if (e != hipSuccess) return e;
      table = tab; table_stride = tiles + 1; mode = half ? 1 : 0;
    }
    if (mode >= 0) {
      if (!lans_single) {
        adam_update_kernel<<<g.n_tiles, kThreads, 0, stream>>>(g, SparseTileDec<kTile, kThreads>{payload, g.stride, g.k_cap, mode, table, table_stride, pairs}, x, m, v, o);
        return hipGetLastError();
      }
      bool used = false;
      hipError_t e = run_lans_single(g, SparseTileDec<kSTile, kLThreads>{payload, g.stride, g.k_cap, mode, table, table_stride, pairs},
                                     x, m, v, o, ws, stream, &used);
      if (e != hipSuccess || used) return e;
      // (the single-pass kernel declined the shape: the dense decode below overwrites the lists)
    }
  }
  hipError_t e = decode_dense(g, prm, payload, dense, stream);
  if (e != hipSuccess) return e;
  return run_update(g, DenseDec{dense}, x, m, v, opt, norms, ws, stream);
}

}  // namespace bpc
