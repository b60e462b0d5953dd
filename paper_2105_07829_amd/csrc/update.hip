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

// ---------------------------------------------------------------------------------------------
// LANS with caller-defined blocks (Algorithm 5 normalises over layers G_b), one pass over the
// data where the blocks allow it.
//
// The tile structure, the lagged exchange and the arithmetic are those of lans_single_kernel;
// what changes is whose sums a tile needs.  A tile of 8192 elements meets its blocks as
//   * blocks that lie inside it ("interior"): their three sums are complete in the workgroup;
//   * at most two blocks that reach beyond it: the one that holds its first element and the
//     one that holds its last.  The tile's share of the first goes to slot A of the tile, its
//     share of the last (if that is another block) to slot B, and the tile counts itself in
//     at the block (one atomic add).  The tile that finds itself the last of a block's
//     t1 - t0 + 1 tiles adds up the shares in tile order (first tile: slot A if the block
//     starts on the tile's first element, else B; every later tile: slot A), which makes the
//     totals independent of timing, and publishes phi and the two weights of the block.  Tiles
//     wait for those three words in their lagged phase 2, not for slots.
// A workgroup that holds a tile cannot take its next one before the tile's x is written.  With
// G workgroups taking tiles w, w + G, ... (round i = tiles iG .. iG + G - 1), a workgroup writes
// the x of its round-(i-1) tile after phase 1 of its round-i tile; so a wait for a block whose
// tiles lie in at most two consecutive rounds is for tiles of rounds <= i, and by induction over
// the rounds (phase 1 never waits for a tile that has not counted itself in) every such wait
// ends.  A block that reaches over three rounds or more could stall the grid, and a tile with
// more blocks than the kernel keeps weights for does not fit either.  Such tiles are
// "deferred": they update their moments, publish their shares and count in like all others,
// but leave x alone and put their number on a list; lans_deferred_kernel, launched after this
// one (when every block's totals are known), recomputes r + wd x and c + wd x from the
// updated moments and writes their x (16.5 more bytes per element, for those tiles only).
constexpr int kLMaxLocal = 32;                  // blocks of a tile the one-pass kernel keeps weights for
constexpr uint32_t kTotUnset = 0xffffffffu;     // a block total not yet published (never the bits of a result:
                                                // a NaN that arithmetic produces is 0x7fc00000 or carries a payload of its input)

__global__ void lans_blocks_prepare_kernel(BlockWs w, const uint64_t *offs, uint64_t n_blocks, uint32_t tiles, uint32_t *status) {
  const uint64_t step = (uint64_t)gridDim.x * blockDim.x;
  const uint64_t i0 = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (uint64_t i = i0; i < 4 * n_blocks; i += step) w.tot[i] = kTotUnset;
  for (uint64_t i = i0; i < n_blocks; i += step) w.cnt[i] = 0;
  for (uint64_t i = i0; i < 6ull * tiles; i += step) w.tslots[i] = -1.0;
  for (uint64_t i = i0; i < tiles; i += step) w.first[i] = find_block(offs, n_blocks, i * kSTile);
  if (i0 == 0) {
    w.list[0] = 0;
    status[0] = 0;
    status[1] = 0;
  }
}

// A thread's three sums of squares over those of its eight elements whose position in the tile
// lies in [lo, hi) (f32, elements in index order), then over the wave (a tree in f32).
__device__ __forceinline__ void lans_wave_sums(const LansHeld &h, uint32_t lo, uint32_t hi, float out[3]) {
  float f_x = 0.0f, f_r = 0.0f, f_c = 0.0f;
#pragma unroll
  for (int u = 0; u < kLRows; ++u) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t pos = (uint32_t)(u * kLRow) + threadIdx.x * 4 + c;
      const bool in = pos >= lo && pos < hi;
      f_x = in ? fmaf(h.xs[4 * u + c], h.xs[4 * u + c], f_x) : f_x;
      f_r = in ? fmaf(h.ur[4 * u + c], h.ur[4 * u + c], f_r) : f_r;
      f_c = in ? fmaf(h.uc[4 * u + c], h.uc[4 * u + c], f_c) : f_c;
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    f_x = f_x + __shfl_xor(f_x, off, 64);
    f_r = f_r + __shfl_xor(f_r, off, 64);
    f_c = f_c + __shfl_xor(f_c, off, 64);
  }
  out[0] = f_x; out[1] = f_r; out[2] = f_c;
}

// phi(||x||) and the two weights from a block's three sums.
__device__ __forceinline__ void lans_weights(const OptArgs &o, double s_x, double s_r, double s_c, float w[3]) {
  const float norm_x = (float)sqrt(s_x);
  const float norm_r = (float)sqrt(s_r);
  const float norm_c = (float)sqrt(s_c);
  float phi = norm_x < o.phi_lo ? o.phi_lo : norm_x;
  phi = phi > o.phi_hi ? o.phi_hi : phi;
  w[0] = phi;
  w[1] = norm_r > 0.0f ? o.beta1 / norm_r : 0.0f;
  w[2] = norm_c > 0.0f ? (1.0f - o.beta1) / norm_c : 0.0f;
}

// What a workgroup knows about the blocks of a tile (LDS; two of them: the tile in phase 1
// and the tile whose x is still to be written).
struct TileBlocks {
  uint64_t bound[kLMaxLocal + 1];    // bound[q] = first element of the tile's q-th block (bound[nloc] = end of the last)
  uint32_t rel[kLMaxLocal + 1];      // the same relative to the tile, clamped to [0, 8192]
  float wts[kLMaxLocal][3];          // phi, w_r, w_c of the tile's q-th block
  // the blocks that reach beyond the tile: side 0 holds its first element, side 1 its last
  double share[2][3];                // the tile's own sums over its part of that block
  uint64_t far_lo[2], far_hi[2];     // the block's elements [lo, hi)
  uint32_t far_b[2];                 // its number, or kNoBlock
  uint32_t far_q[2];                 // its index in the tile's block list
  uint32_t nloc;                     // blocks of the tile (kLMaxLocal + 1: more than the kernel keeps weights for)
  uint32_t fb;                       // number of the tile's first block
  uint32_t deferred;
};
constexpr uint32_t kNoBlock = 0xffffffffu;

// Index in the tile's block list of the block that holds tile-relative position `pos`.
__device__ __forceinline__ uint32_t lans_block_of(const TileBlocks &tb, uint32_t pos) {
  uint32_t q = 0;
  for (uint32_t k = 1; k < tb.nloc; ++k) q += tb.rel[k] <= pos ? 1u : 0u;
  return q;
}

// First wave: the three words of block b's totals once they are published.
__device__ __forceinline__ void lans_wait_block(const uint32_t *tot, uint32_t *status, float w[3]) {
  uint32_t a, b, c;
  int spins = 0;
  for (;;) {
    a = __hip_atomic_load(tot + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    b = __hip_atomic_load(tot + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    c = __hip_atomic_load(tot + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (a != kTotUnset && b != kTotUnset && c != kTotUnset) break;
    if (++spins > kSpinLimit) {
      if ((threadIdx.x & 63) == 0) atomicOr(status, 1u);
      break;
    }
    __builtin_amdgcn_s_sleep(16);
  }
  w[0] = __uint_as_float(a); w[1] = __uint_as_float(b); w[2] = __uint_as_float(c);
}

// One wave: the tile `item` has the share `share` of block b, which covers tiles t0..t1.
// Publishes the share, counts the tile in, and if it is the block's last tile adds up all
// shares in tile order and publishes the block's totals.
__device__ __forceinline__ void lans_publish_share(const OptArgs &o, const BlockWs &w, uint32_t item, int side, uint32_t b,
                                          uint64_t lo, uint64_t hi, const double share[3], uint32_t *status) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t t0 = (uint32_t)(lo / kSTile), t1 = (uint32_t)((hi - 1) / kSTile);
  uint32_t arrived = 0;
  if (lane == 0) {
    double *ps = w.tslots + 6ull * item + 3 * side;
    slot_publish(ps + 0, share[0]);
    slot_publish(ps + 1, share[1]);
    slot_publish(ps + 2, share[2]);
    arrived = __hip_atomic_fetch_add(w.cnt + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
  }
  arrived = __builtin_amdgcn_readfirstlane(arrived);
  if (arrived != t1 - t0 + 1) return;
  // the last tile of the block: every other tile has issued the stores of its share
  const bool starts_on_tile = lo % kSTile == 0;
  double a0 = 0.0, a1 = 0.0, a2 = 0.0;
  for (uint32_t idx = lane; idx <= t1 - t0; idx += 64) {
    const double *ps = w.tslots + 6ull * (t0 + idx) + ((idx == 0 && !starts_on_tile) ? 3 : 0);
    double q0, q1, q2;
    int spins = 0;
    for (;;) {
      q0 = __hip_atomic_load(ps + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      q1 = __hip_atomic_load(ps + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      q2 = __hip_atomic_load(ps + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (slot_published(q0) && slot_published(q1) && slot_published(q2)) break;
      if (++spins > kSpinLimit) {
        atomicOr(status, 1u);
        break;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    a0 += q0; a1 += q1; a2 += q2;
  }
  a0 = wave_sum(a0);
  a1 = wave_sum(a1);
  a2 = wave_sum(a2);
  if (lane == 0) {
    float wt[3];
    lans_weights(o, a0, a1, a2, wt);
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      uint32_t bits = __float_as_uint(wt[k]);
      bits = bits == kTotUnset ? 0x7fc00000u : bits;
      __hip_atomic_store(w.tot + 4ull * b + k, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Phase 1, block part: from the tile's held values and its block bounds (already in tb.bound /
// tb.rel / tb.nloc / tb.fb) to the weights of the interior blocks, the published shares of the
// far-reaching ones and the decision whether the tile is deferred.  `red` holds
// kLMaxLocal x waves x 3 doubles.  All threads; contains barriers.
__device__ __forceinline__ void lans_tile_blocks(const OptArgs &o, const BlockWs &w, uint32_t item, uint32_t n_items, const LansTile &t,
                                        const LansHeld &h, TileBlocks &tb, double *red, uint32_t span_limit, uint64_t D,
                                        uint32_t *status) {
  const uint32_t nloc = tb.nloc;
  const bool many = nloc > (uint32_t)kLMaxLocal;
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  constexpr int kWaves = kLThreads / 64;
  const uint64_t tile_first = (uint64_t)item * kSTile;
  const uint64_t tile_end = tile_first + t.valid;
  // a tile with more blocks than weights are kept for: only its first and last block can matter
  // to other tiles; the last one is the block that holds the next tile's first element, if
  // that block starts inside this tile
  uint32_t last_b = kNoBlock;
  uint64_t last_lo = 0, last_hi = 0;
  if (many && item + 1 < n_items) {
    last_b = __builtin_amdgcn_readfirstlane(w.first[item + 1]);
    last_lo = uniform_off(o.block_offsets[last_b]);
    last_hi = uniform_off(o.block_offsets[last_b + 1]);
    if (last_lo >= tile_end) last_b = kNoBlock;
  }
  const uint32_t n_sums = many ? 2u : nloc;
#pragma unroll 1
  for (uint32_t q = 0; q < n_sums; ++q) {
    // positions of the tile that belong to the q-th sum (past the partition's end: to none)
    uint32_t lo, hi;
    if (many) {
      lo = q == 0 ? 0u : (last_b != kNoBlock ? (uint32_t)(last_lo - tile_first) : t.valid);
      hi = q == 0 ? tb.rel[1] : t.valid;
    } else {
      lo = tb.rel[q];
      hi = tb.rel[q + 1];
    }
    float f[3];
    lans_wave_sums(h, lo, hi, f);
    if (lane == 0) {
      red[(q * kWaves + wave) * 3 + 0] = (double)f[0];
      red[(q * kWaves + wave) * 3 + 1] = (double)f[1];
      red[(q * kWaves + wave) * 3 + 2] = (double)f[2];
    }
  }
  if (threadIdx.x == 0) {
    tb.far_b[0] = kNoBlock;
    tb.far_b[1] = kNoBlock;
    tb.deferred = many ? 1u : 0u;
  }
  __syncthreads();
  if (threadIdx.x < n_sums) {
    const uint32_t q = threadIdx.x;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0;
    // (not unrolled: sixteen waves' sums in flight at once would need a hundred registers)
#pragma unroll 2
    for (int wv = 0; wv < kWaves; ++wv) {
      s0 += red[(q * kWaves + wv) * 3 + 0];
      s1 += red[(q * kWaves + wv) * 3 + 1];
      s2 += red[(q * kWaves + wv) * 3 + 2];
    }
    uint64_t lo, hi;
    uint32_t b;
    if (many) {
      lo = q == 0 ? tb.bound[0] : last_lo;
      hi = q == 0 ? tb.bound[1] : last_hi;
      b = q == 0 ? tb.fb : last_b;
    } else {
      lo = tb.bound[q];
      hi = tb.bound[q + 1];
      b = tb.fb + q;
    }
    const bool interior = lo >= tile_first && hi <= tile_end;
    if (!interior && b != kNoBlock) {
      const int side = q == 0 ? 0 : 1;     // (only the first and the last block of a tile can reach beyond it)
      tb.share[side][0] = s0; tb.share[side][1] = s1; tb.share[side][2] = s2;
      tb.far_b[side] = b;
      tb.far_q[side] = q;
      tb.far_lo[side] = lo;
      tb.far_hi[side] = hi;
    } else if (!many) {
      float wt[3];
      lans_weights(o, s0, s1, s2, wt);
      tb.wts[q][0] = wt[0]; tb.wts[q][1] = wt[1]; tb.wts[q][2] = wt[2];
    }
  }
  __syncthreads();
  if (wave < 2) {
    const int side = (int)wave;
    const uint32_t b = __builtin_amdgcn_readfirstlane(tb.far_b[side]);
    if (b != kNoBlock) {
      const uint64_t lo = uniform_off(tb.far_lo[side]), hi = uniform_off(tb.far_hi[side]);
      const double share[3] = {tb.share[side][0], tb.share[side][1], tb.share[side][2]};
      // (rounds: workgroup w of G takes tiles w, w + G, ...; the tiles w + iG form round i)
      if ((hi - 1) / kSTile / span_limit - lo / kSTile / span_limit > 1 && lane == 0) tb.deferred = 1u;
      lans_publish_share(o, w, item, side, b, lo, hi, share, status);
    }
  }
}

// x of a tile whose blocks' weights are all in tb.wts.
__device__ __forceinline__ void lans_write_x_blocks(const Geo &g, const ClusterGeo &cg, const OptArgs &o, float *x, uint32_t item,
                                           const LansHeld &h, const TileBlocks &tb) {
  const LansTile t = lans_tile(g, cg, item);
  const uint32_t nloc = tb.nloc;
#pragma unroll
  for (int u = 0; u < kLRows; ++u) {
    float xo[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t q = nloc == 1 ? 0u : lans_block_of(tb, (uint32_t)(u * kLRow) + threadIdx.x * 4 + c);
      const float phi = tb.wts[q][0], w_r = tb.wts[q][1], w_c = tb.wts[q][2];
      const float dir = phi * (w_r * h.ur[4 * u + c] + w_c * h.uc[4 * u + c]);
      xo[c] = h.xs[4 * u + c] - o.lr * dir;
    }
    row_buf(x + t.base, t.valid, u * kLRow, kLRow).store16<kNonTemporal>(as_u32x4(xo[0], xo[1], xo[2], xo[3]), threadIdx.x * 16);
  }
}

template <class DEC>
__global__ __launch_bounds__(kLThreads) void lans_blocks_kernel(Geo g, ClusterGeo cg, DEC dec, float *x, float *m, float *v,
                                                               OptArgs o, BlockWs w, uint32_t span_limit /* = gridDim.x */) {
  __shared__ __align__(16) float lds[DEC::kLdsFloats];
  __shared__ double red[kLMaxLocal * (kLThreads / 64) * 3];
  __shared__ TileBlocks tbs[2];
  constexpr uint32_t kNone = 0xffffffffu;
  uint32_t *status = o.status;
  uint32_t item = __builtin_amdgcn_readfirstlane(blockIdx.x);
  if (item >= cg.n_items) return;
  LansRaw<DEC> raw;
  lans_issue(g, cg, dec, x, m, v, item, raw);
  uint32_t fb_raw = w.first[item];
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the loop is entered with nothing in flight
  LansHeld prev_h;
  uint32_t prev = kNone;
  int cur = 0;
  const float omb1 = 1.0f - o.beta1, omb2 = 1.0f - o.beta2;
  const float inv_bc1 = 1.0f / o.bc1, inv_bc2 = 1.0f / o.bc2;
  for (;;) {
    const LansTile t = lans_tile(g, cg, item);
    TileBlocks &tb = tbs[cur];
    // the bounds of the tile's blocks: thread k asks for the first element of block fb + k
    const uint32_t fb = __builtin_amdgcn_readfirstlane(fb_raw);
    uint64_t my_bound = 0;
    if (threadIdx.x <= (uint32_t)kLMaxLocal) {
      const uint64_t k = (uint64_t)fb + threadIdx.x;
      my_bound = o.block_offsets[k < o.n_blocks ? k : o.n_blocks];
    }
    if constexpr (has_begin_tile<DEC>::value) {
      dec.begin_tile(t.p, t.tile, lds);
    } else {
      __syncthreads();
      dec.table(raw.hdr, lds);
      __syncthreads();
    }
    LansHeld h;
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
        h.xs[4 * u + c] = xj;
        h.ur[4 * u + c] = u_r;
        h.uc[4 * u + c] = u_c;
      }
      row_buf(m + t.base, t.valid, u * kLRow, kLRow).store16<kNonTemporal>(as_u32x4(mo[0], mo[1], mo[2], mo[3]), threadIdx.x * 16);
      row_buf(v + t.base, t.valid, u * kLRow, kLRow).store16<kNonTemporal>(as_u32x4(vo[0], vo[1], vo[2], vo[3]), threadIdx.x * 16);
    }
    const uint32_t next = __builtin_amdgcn_readfirstlane(item + gridDim.x);
    const bool have_next = next < cg.n_items;
    if (have_next) {
      lans_issue(g, cg, dec, x, m, v, next, raw);
      fb_raw = w.first[next];
    }
    // the tile's block list: bounds, their positions in the tile, the number of blocks
    const uint64_t tile_first = (uint64_t)item * kSTile;
    const uint64_t tile_end = tile_first + t.valid;
    if (threadIdx.x < 64) {
      const bool inside = threadIdx.x >= 1 && threadIdx.x <= (uint32_t)kLMaxLocal && my_bound < tile_end;
      const uint32_t n_inside = (uint32_t)__popcll(__ballot(inside));     // (bounds ascend: these are lanes 1..n_inside)
      if (threadIdx.x <= (uint32_t)kLMaxLocal) {
        tb.bound[threadIdx.x] = my_bound;
        const uint64_t c = my_bound < tile_first ? tile_first : (my_bound > tile_end ? tile_end : my_bound);
        tb.rel[threadIdx.x] = (uint32_t)(c - tile_first);
      }
      if (threadIdx.x == 0) {
        tb.nloc = n_inside + 1;
        tb.fb = fb;
      }
    }
    __syncthreads();
    lans_tile_blocks(o, w, item, cg.n_items, t, h, tb, red, span_limit, g.D, status);
    __syncthreads();
    if (threadIdx.x == 0 && tb.deferred) {
      const uint32_t at = __hip_atomic_fetch_add(w.list, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      w.list[1 + at] = item;
    }
    // the older tile: totals of its far-reaching blocks, then its x
    if (prev != kNone) {
      TileBlocks &tp = tbs[cur ^ 1];
      if (!tp.deferred) {
        if (threadIdx.x < 128) {
          const int side = (int)(threadIdx.x >> 6);
          const uint32_t b = __builtin_amdgcn_readfirstlane(tp.far_b[side]);
          if (b != kNoBlock) {
            const uint32_t q = tp.far_q[side];
            float wt[3];
            lans_wait_block(w.tot + 4ull * b, status, wt);
            if ((threadIdx.x & 63) == 0) { tp.wts[q][0] = wt[0]; tp.wts[q][1] = wt[1]; tp.wts[q][2] = wt[2]; }
          }
        }
        __syncthreads();
        lans_write_x_blocks(g, cg, o, x, prev, prev_h, tp);
      }
    }
    prev_h = h;
    prev = item;
    cur ^= 1;
    if (!have_next) break;
    item = next;
    __syncthreads();
  }
  // the last tile
  __syncthreads();
  TileBlocks &tp = tbs[cur ^ 1];
  if (!tp.deferred) {
    if (threadIdx.x < 128) {
      const int side = (int)(threadIdx.x >> 6);
      const uint32_t b = __builtin_amdgcn_readfirstlane(tp.far_b[side]);
      if (b != kNoBlock) {
        const uint32_t q = tp.far_q[side];
        float wt[3];
        lans_wait_block(w.tot + 4ull * b, status, wt);
        if ((threadIdx.x & 63) == 0) { tp.wts[q][0] = wt[0]; tp.wts[q][1] = wt[1]; tp.wts[q][2] = wt[2]; }
      }
    }
    __syncthreads();
    lans_write_x_blocks(g, cg, o, x, prev, prev_h, tp);
  }
}

// x of the deferred tiles, after lans_blocks_kernel: every block's totals are known by now.
// Workgroup i takes entries i, i + grid, ... of the list.  The moments in memory are the
// updated ones, so r + wd x and c + wd x come out as in the first kernel; the sums of blocks
// inside the tile are formed again the same way (same order, same bits), block by block, which
// needs no table and so handles any number of blocks in a tile.
template <class DEC>
__global__ __launch_bounds__(kLThreads) void lans_deferred_kernel(Geo g, ClusterGeo cg, DEC dec, float *x, const float *m,
                                                                 const float *v, OptArgs o, BlockWs w) {
  __shared__ __align__(16) float lds[DEC::kLdsFloats];
  __shared__ double red[(kLThreads / 64) * 3];
  __shared__ float wts_sh[3];
  constexpr int kWaves = kLThreads / 64;
  const uint32_t n_list = __builtin_amdgcn_readfirstlane(w.list[0]);
  const float inv_bc1 = 1.0f / o.bc1, inv_bc2 = 1.0f / o.bc2;
  for (uint32_t at = blockIdx.x; at < n_list; at += gridDim.x) {
    const uint32_t item = __builtin_amdgcn_readfirstlane(w.list[1 + at]);
    const LansTile t = lans_tile(g, cg, item);
    LansRaw<DEC> raw;
    lans_issue(g, cg, dec, x, m, v, item, raw);
    if constexpr (has_begin_tile<DEC>::value) {
      dec.begin_tile(t.p, t.tile, lds);
    } else {
      __syncthreads();
      dec.table(raw.hdr, lds);
      __syncthreads();
    }
    LansHeld h;
#pragma unroll
    for (int u = 0; u < kLRows; ++u) {
      const uint32_t mi[4] = {raw.m[u].x, raw.m[u].y, raw.m[u].z, raw.m[u].w};
      const uint32_t vi[4] = {raw.v[u].x, raw.v[u].y, raw.v[u].z, raw.v[u].w};
      const uint32_t xi[4] = {raw.x[u].x, raw.x[u].y, raw.x[u].z, raw.x[u].w};
      float gr[4];
      dec.decode4(raw.g[u], t.tile * kSTile + u * kLRow + threadIdx.x * 4, raw.hdr, lds, gr);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float xj = __uint_as_float(xi[c]);
        float u_r, u_c;
        ratios_fast(o, inv_bc1, inv_bc2, gr[c], __uint_as_float(mi[c]), __uint_as_float(vi[c]), xj, &u_r, &u_c);
        h.xs[4 * u + c] = xj;
        h.ur[4 * u + c] = u_r;
        h.uc[4 * u + c] = u_c;
      }
    }
    const uint64_t tile_first = (uint64_t)item * kSTile;
    const uint64_t tile_end = tile_first + t.valid;
    float xo[kLPer];
#pragma unroll
    for (int e = 0; e < kLPer; ++e) xo[e] = h.xs[e];
#pragma unroll 1
    for (uint64_t b = __builtin_amdgcn_readfirstlane(w.first[item]); b < o.n_blocks; ++b) {
      const uint64_t lo = uniform_off(o.block_offsets[b]), hi = uniform_off(o.block_offsets[b + 1]);
      if (lo >= tile_end) break;
      const uint32_t rlo = (uint32_t)((lo > tile_first ? lo : tile_first) - tile_first);
      const uint32_t rhi = (uint32_t)((hi < tile_end ? hi : tile_end) - tile_first);
      float phi, w_r, w_c;
      if (lo < tile_first || hi > tile_end) {
        phi = __uint_as_float(w.tot[4 * b + 0]);
        w_r = __uint_as_float(w.tot[4 * b + 1]);
        w_c = __uint_as_float(w.tot[4 * b + 2]);
      } else {
        float f[3];
        lans_wave_sums(h, rlo, rhi, f);
        __syncthreads();   // (red and wts_sh of the block before have been read)
        if ((threadIdx.x & 63) == 0) {
          red[(threadIdx.x >> 6) * 3 + 0] = (double)f[0];
          red[(threadIdx.x >> 6) * 3 + 1] = (double)f[1];
          red[(threadIdx.x >> 6) * 3 + 2] = (double)f[2];
        }
        __syncthreads();
        if (threadIdx.x == 0) {
          double s0 = 0.0, s1 = 0.0, s2 = 0.0;
#pragma unroll
          for (int wv = 0; wv < kWaves; ++wv) {
            s0 += red[wv * 3 + 0];
            s1 += red[wv * 3 + 1];
            s2 += red[wv * 3 + 2];
          }
          float wt[3];
          lans_weights(o, s0, s1, s2, wt);
          wts_sh[0] = wt[0]; wts_sh[1] = wt[1]; wts_sh[2] = wt[2];
        }
        __syncthreads();
        phi = wts_sh[0]; w_r = wts_sh[1]; w_c = wts_sh[2];
      }
#pragma unroll
      for (int u = 0; u < kLRows; ++u)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const uint32_t pos = (uint32_t)(u * kLRow) + threadIdx.x * 4 + c;
          const float dir = phi * (w_r * h.ur[4 * u + c] + w_c * h.uc[4 * u + c]);
          xo[4 * u + c] = pos >= rlo && pos < rhi ? h.xs[4 * u + c] - o.lr * dir : xo[4 * u + c];
        }
    }
#pragma unroll
    for (int u = 0; u < kLRows; ++u)
      row_buf(x + t.base, t.valid, u * kLRow, kLRow).store16<kNonTemporal>(as_u32x4(xo[4 * u], xo[4 * u + 1], xo[4 * u + 2], xo[4 * u + 3]), threadIdx.x * 16);
    __syncthreads();   // (lds of this tile has been read)
  }
}

// LANS with caller-defined blocks in one pass (plus the pass over the deferred tiles).
// *used = false: shape not supported, nothing enqueued.
template <class DEC>
static hipError_t run_lans_blocks(const Geo &g, DEC dec, float *x, float *m, float *v, const OptArgs &o,
                                  const Workspace &ws, hipStream_t stream, bool *used) {
  *used = false;
  if (g.part_elems % kSTile != 0) return hipSuccess;
  const ClusterGeo cg = make_cluster_geo(g, kSTile);
  static PerDevice cache;
  const int capacity = cache.get([] { return cluster_capacity(reinterpret_cast<const void *>(&lans_blocks_kernel<DEC>), kLThreads, 0); });
  if (capacity <= 0) return hipSuccess;
  *used = true;
  const BlockWs w = block_ws(ws.base + ws.lay.norms, o.n_blocks, cg.n_items);
  hipError_t e = cluster_launch_begin(stream);
  if (e != hipSuccess) return e;
  const uint64_t most = 6ull * cg.n_items > 4 * o.n_blocks ? 6ull * cg.n_items : 4 * o.n_blocks;
  const uint32_t prep_grid = (uint32_t)(cdiv(most, 256) < 4096 ? cdiv(most, 256) : 4096);
  lans_blocks_prepare_kernel<<<prep_grid, 256, 0, stream>>>(w, o.block_offsets, o.n_blocks, cg.n_items, o.status);
  const uint32_t grid = cg.n_items > (uint32_t)capacity ? (uint32_t)capacity : cg.n_items;
  lans_blocks_kernel<DEC><<<grid, kLThreads, 0, stream>>>(g, cg, dec, x, m, v, o, w, grid);
  const uint32_t sweep_grid = cg.n_items < 1024u ? cg.n_items : 1024u;
  lans_deferred_kernel<DEC><<<sweep_grid, kLThreads, 0, stream>>>(g, cg, dec, x, m, v, o, w);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  return cluster_launch_end(stream);
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
  uint32_t *status = ws.status();
  hipError_t e = cluster_launch_begin(stream);
  if (e != hipSuccess) return e;
  const uint32_t n_slots = 3 * g.P * cg.tiles_per_part;
  slots_reset_kernel<<<(uint32_t)cdiv(n_slots, 256), 256, 0, stream>>>(slots, n_slots, status, nullptr);
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
            opt.phi_lo, opt.phi_hi, opt.block_offsets, opt.n_blocks, ws.status()};
  if (opt.kind == BPC_OPT_ADAM) {
    adam_update_kernel<DEC><<<g.n_tiles, kThreads, 0, stream>>>(g, dec, x, m, v, o);
    return hipGetLastError();
  }
  {
    bool used = false;
    hipError_t e1 = opt.block_offsets ? run_lans_blocks(g, dec, x, m, v, o, ws, stream, &used)
                                      : run_lans_single(g, dec, x, m, v, o, ws, stream, &used);
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
              opt.phi_lo, opt.phi_hi, opt.block_offsets, opt.n_blocks, ws.status()};
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
