// Pieces shared by the worker kernels that lay a tile out in rows of 4 consecutive elements a
// thread (every 16-byte access of a wave then covers whole cache lines): widening a row's loads,
// and merging the per-lane bit groups of neighbouring lanes into words.
#pragma once
#include "cluster_launch.hpp"

namespace bpc {

__device__ inline void widen4(const u32x4 &g, float out[4]) {
  out[0] = __uint_as_float(g.x); out[1] = __uint_as_float(g.y); out[2] = __uint_as_float(g.z); out[3] = __uint_as_float(g.w);
}
__device__ inline void widen4(const u32x2 &g, float out[4]) {
  const uint32_t lo = g.x, hi = g.y;
  float2 a = __half22float2(*reinterpret_cast<const __half2 *>(&lo));
  float2 b = __half22float2(*reinterpret_cast<const __half2 *>(&hi));
  out[0] = a.x; out[1] = a.y; out[2] = b.x; out[3] = b.y;
}
template <class G> struct Vec4Of;
template <> struct Vec4Of<float> { using type = u32x4; };
template <> struct Vec4Of<__half> { using type = u32x2; };
__device__ inline u32x4 tile_load4(const TileBuf &b, uint32_t lane_off, uint32_t row_off, const float *) { return b.load16<kNonTemporal>(lane_off, row_off); }
__device__ inline u32x2 tile_load4(const TileBuf &b, uint32_t lane_off, uint32_t row_off, const __half *) { return b.load8<kNonTemporal>(lane_off, row_off); }

// An odd number of halves behind a descriptor (the end of an f16 gradient): the range check works
// on whole dwords, so the last half came back as zero; the lane that owns it fetches it alone.
// `gr[u]` holds the thread's 4 halves of row u of ROW_ELEMS elements, `valid` halves exist.
template <int ROWS, int ROW_ELEMS>
__device__ inline void patch_last_half(const TileBuf &gb, uint32_t valid, u32x2 (&gr)[ROWS]) {
  if (valid & 1u) {   // (uniform)
    const uint32_t last = valid - 1;   // even: the low half of its dword
    const uint32_t mine = last - threadIdx.x * 4;
#pragma unroll
    for (int u = 0; u < ROWS; ++u) {
      const uint32_t c = mine - u * ROW_ELEMS;
      if (c < 4u) {
        const uint32_t h = gb.load2(last * 2, 0);
        if (c == 0) gr[u].x = h; else gr[u].y = h;
      }
    }
  }
}
template <int ROWS, int ROW_ELEMS>
__device__ inline void patch_last_half(const TileBuf &, uint32_t, u32x4 (&)[ROWS]) {}

// Sign bits of a row: every lane holds a nibble for its 4 elements; 8 neighbouring lanes are
// merged into one 32-bit word which lane 8w of the wave ends up holding.
// (DPP row_shl:n makes lane i read lane i+n of its 16-lane row; lanes past the row read 0.)
__device__ inline uint32_t from_lane_above(uint32_t x, int n) {
  return n == 1   ? (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x101, 0xf, 0xf, true)
         : n == 2 ? (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x102, 0xf, 0xf, true)
                  : (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x104, 0xf, 0xf, true);
}
__device__ inline uint32_t merge8(uint32_t nib) {
  nib |= from_lane_above(nib, 1) << 4;
  nib |= from_lane_above(nib, 2) << 8;
  nib |= from_lane_above(nib, 4) << 16;
  return nib;
}

}  // namespace bpc
