// Device helpers shared by the kernels: Philox4x32-10, fixed-order reductions,
// gradient loads with exact fp16 widening.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace bpc {

// Philox4x32-10 (Salmon et al., SC'11).  One 64-bit multiply-add yields both halves of a product.
struct Philox {
  uint32_t k0, k1, c1, c2, c3;
  __device__ Philox(uint64_t seed, uint64_t stream_id, uint32_t partition)
      : k0((uint32_t)seed), k1((uint32_t)(seed >> 32)), c1(partition), c2((uint32_t)stream_id),
        c3((uint32_t)(stream_id >> 32)) {}
  __device__ void block(uint32_t blk, uint32_t out[4]) const {
    uint32_t a = blk, b = c1, c = c2, d = c3, ka = k0, kb = k1;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
      uint64_t p0 = (uint64_t)0xD2511F53u * a;
      uint64_t p1 = (uint64_t)0xCD9E8D57u * c;
      // three-way exclusive or in one instruction (truth table 0x96)
      uint32_t na = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), b, ka, 0x96);
      uint32_t nc = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), d, kb, 0x96);
      b = (uint32_t)p1;
      d = (uint32_t)p0;
      a = na;
      c = nc;
      ka += 0x9E3779B9u;
      kb += 0xBB67AE85u;
    }
    out[0] = a; out[1] = b; out[2] = c; out[3] = d;
  }
  __device__ uint32_t word(uint32_t t) const {
    uint32_t o[4];
    block(t >> 2, o);
    uint32_t s = t & 3;
    return s == 0 ? o[0] : s == 1 ? o[1] : s == 2 ? o[2] : o[3];
  }
};

// Marks an element offset that is the same in every lane as such, so that `base + offset`
// stays a scalar and accesses take the "scalar base + 32-bit lane offset" addressing form
// instead of needing a 64-bit address register pair per access.
__device__ inline uint64_t uniform_off(uint64_t v) {
  uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return ((uint64_t)hi << 32) | lo;
}

// A window of memory addressed through a buffer descriptor: accesses are "descriptor (scalar
// registers) + 32-bit lane offset + scalar offset", so a tile's rows need no per-row address
// registers.  `base` must be the same in every lane; `bytes` bounds the window (reads past it
// return 0 and writes past it are dropped by the hardware).  store16 deliberately has no
// scalar-offset parameter (see there): keep 16-byte stores unable to take one.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// AUX is the cache policy of an access: 0 = default, kNonTemporal = data used once.
constexpr int kNonTemporal = 2;
struct TileBuf {
  __amdgpu_buffer_rsrc_t r;
  __device__ TileBuf(const void *base, uint32_t bytes)
      : r(__builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000)) {}
  template <int AUX = 0>
  __device__ u32x4 load16(uint32_t lane_off, uint32_t row_off) const {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)row_off, AUX);
  }
  template <int AUX = 0>
  __device__ u32x2 load8(uint32_t lane_off, uint32_t row_off) const {
    return __builtin_amdgcn_raw_buffer_load_b64(r, (int)lane_off, (int)row_off, AUX);
  }
  template <int AUX = 0>
  __device__ uint32_t load4(uint32_t lane_off, uint32_t row_off) const {
    return __builtin_amdgcn_raw_buffer_load_b32(r, (int)lane_off, (int)row_off, AUX);
  }
  template <int AUX = 0>
  __device__ uint32_t load2(uint32_t lane_off, uint32_t row_off) const {
    return (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)lane_off, (int)row_off, AUX);
  }
  template <int AUX = 0>
  __device__ uint32_t load1(uint32_t lane_off, uint32_t row_off) const {
    return (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(r, (int)lane_off, (int)row_off, AUX);
  }
  // 16-byte stores take no scalar offset: with one, the hardware was seen to pick up a data
  // register that the next instruction overwrites (the compiler only spaces the two apart
  // when the offset field is a constant).  Callers put the row into the descriptor's base.
  template <int AUX = 0>
  __device__ void store16(u32x4 v, uint32_t lane_off) const {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)lane_off, 0, AUX);
  }
  template <int AUX = 0>
  __device__ void store8(u32x2 v, uint32_t lane_off) const {
    __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)lane_off, 0, AUX);
  }
  template <int AUX = 0>
  __device__ void store1(uint32_t v, uint32_t lane_off, uint32_t row_off) const {
    __builtin_amdgcn_raw_buffer_store_b8((uint8_t)v, r, (int)lane_off, (int)row_off, AUX);
  }
  template <int AUX = 0>
  __device__ void store2(uint32_t v, uint32_t lane_off, uint32_t row_off) const {
    __builtin_amdgcn_raw_buffer_store_b16((uint16_t)v, r, (int)lane_off, (int)row_off, AUX);
  }
  template <int AUX = 0>
  __device__ void store4(uint32_t v, uint32_t lane_off, uint32_t row_off) const {
    __builtin_amdgcn_raw_buffer_store_b32(v, r, (int)lane_off, (int)row_off, AUX);
  }
};
// A value every lane loads from the same address, moved to a scalar register inside the
// branch that loads it: the wait for the load then stays in that branch instead of draining
// every load in flight where the branches join (vector-memory waits are counted in order).
__device__ inline float uniform_load(const float *p) {
  return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(*p)));
}
// Descriptor of row elements [row0, row0 + row_elems) of an f32 tile of which only the first
// `valid` elements exist: accesses to the rest read 0 / are dropped.
__device__ inline TileBuf row_buf(const float *tile_base, uint32_t valid, uint32_t row0, uint32_t row_elems) {
  const uint32_t in_row = valid > row0 ? valid - row0 : 0u;
  return TileBuf(tile_base + row0, (in_row < row_elems ? in_row : row_elems) * 4);
}
__device__ inline u32x4 as_u32x4(float a, float b, float c, float d) {
  u32x4 v;
  v.x = __float_as_uint(a); v.y = __float_as_uint(b); v.z = __float_as_uint(c); v.w = __float_as_uint(d);
  return v;
}

__device__ inline float load_grad(const float *g, uint64_t i) { return g[i]; }
__device__ inline float load_grad(const __half *g, uint64_t i) { return __half2float(g[i]); }

// The two dithering level maps.  Linear: level l stands for (nu * l) / s.  Natural: level 0
// for 0, level l >= 1 for (nu * 2^(l-1)) / 2^(s-1).  `dither_top` is the value of
// a = |q| * top / nu at the highest level.
__device__ inline float dither_top(uint32_t s, bool natural) { return natural ? (float)(1u << (s - 1)) : (float)s; }
__device__ inline float dither_mag(float nu, uint32_t level, uint32_t s, bool natural) {
  if (!natural) return (nu * (float)level) / (float)s;
  return level == 0 ? 0.0f : (nu * (float)(1u << (level - 1))) / (float)(1u << (s - 1));
}

// Inclusive prefix sum over the 64 lanes of a wave with DPP moves: shifts by 1, 2, 4, 8 inside
// the 16-lane rows (a lane whose source is outside its row adds 0), then lane 15 of rows 0 and
// 2 broadcast to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ inline uint32_t wave_inclusive_scan_u32(uint32_t x) {
  int v = (int)x;
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1, 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2, 3
  return (uint32_t)v;
}

// Sum over the 64 lanes in a fixed butterfly order (same bits on every run).
__device__ inline double wave_sum(double x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}
__device__ inline float wave_max(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
  return x;
}
__device__ inline uint32_t wave_sum_u32(uint32_t x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// Workgroup sum in a fixed order; the result is valid in thread 0.  `scratch` holds one
// double per wave.
template <int THREADS>
__device__ inline double block_sum(double x, double *scratch) {
  x = wave_sum(x);
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) scratch[wave] = x;
  __syncthreads();
  double t = 0.0;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) t += scratch[w];
  }
  return t;
}
template <int THREADS>
__device__ inline float block_max(float x, float *scratch) {
  x = wave_max(x);
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) scratch[wave] = x;
  __syncthreads();
  float t = 0.0f;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) t = fmaxf(t, scratch[w]);
  }
  return t;
}

// Exclusive prefix sum over the workgroup's threads (Hillis-Steele in LDS).  Returns the
// exclusive prefix of `x`; *total receives the sum over all threads.
template <int THREADS>
__device__ inline uint32_t block_exclusive_scan(uint32_t x, uint32_t *lds /*THREADS*/, uint32_t *total) {
  // scan inside each wave with lane moves, then add the totals of the waves before
  const uint32_t incl = wave_inclusive_scan_u32(x);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 63) lds[wave] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) {
    const uint32_t v = lds[w];
    before += w < wave ? v : 0u;
    all += v;
  }
  *total = all;
  __syncthreads();
  return before + incl - x;
}

}  // namespace bpc
