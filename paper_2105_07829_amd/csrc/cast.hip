// FP32 -> FP16 conversion as a compressor (Section 4.1: the data type conversion used where
// anything heavier would not pay; Section 5.1 lists the half-precision method): every element of
// q = g + e (worker) or Delta (server) is rounded to the nearest half, ties to even, and the
// residual is what the rounding dropped (Algorithm 4).  No partition-wide quantity is needed,
// so one streaming launch does it.  A workgroup takes a tile of 4096 elements as rows of 1024,
// 4 consecutive elements a thread and row: every access of a wave to the gradient and the
// residual covers whole cache lines and is marked non-temporal, and all loads of a tile (worker)
// or of two rows (server: the n messages' halves) are requested before the first is used.
// Everything goes through buffer descriptors sized to what exists of the tile: elements past a
// shorter last partition read as zero, encode as zero halves (the record is zero up to the next
// 16-byte boundary) and are not written to the residual.
//
// The identity "compressor" (with it Algorithms 3 and 4 reduce to plain gradient averaging,
// Algorithm 1; also what partitions under the size threshold of Section 4.2 take) is the same
// pass with the f32 values themselves as the record and q - q as the residual.
#include "sources.hpp"
#include "tile_rows.hpp"

namespace bpc {

constexpr int kCRowElems = kThreads * 4;
constexpr int kCRows = kTile / kCRowElems;

// The two record formats: what a thread holds of a row (4 values), bytes a value, and how many
// rows of the n messages the server requests at once (registers: 2 or 4 a worker and row).
struct HalfFmt { using Vec = u32x2; static constexpr int kBytes = 2, kPair = 2; };
struct FloatFmt { using Vec = u32x4; static constexpr int kBytes = 4, kPair = 1; };
template <class FMT>
__device__ inline typename FMT::Vec msg_load4(const TileBuf &b, uint32_t row_off) {
  // (default cache policy: the rows of a record start 16 bytes off a line)
  if constexpr (FMT::kBytes == 2) return b.load8(threadIdx.x * 8, row_off);
  else return b.load16(threadIdx.x * 16, row_off);
}

// Where a tile lies: its partition, the elements of it that exist, its first element in the flat
// arrays, and the bytes of the record's values that belong to it (halves: whole 16-byte chunks).
struct CastTile {
  uint32_t p, j0, valid, rec_bytes;
  uint64_t base;
};
template <class FMT>
__device__ inline CastTile cast_tile(const Geo &g) {
  CastTile t;
  t.p = __builtin_amdgcn_readfirstlane(blockIdx.x / g.tiles_per_part);
  t.j0 = __builtin_amdgcn_readfirstlane((blockIdx.x % g.tiles_per_part) * kTile);
  const uint32_t d = g.part_size(t.p);
  const uint32_t left = d - t.j0;
  t.valid = __builtin_amdgcn_readfirstlane(left < (uint32_t)kTile ? left : (uint32_t)kTile);
  if (FMT::kBytes == 2) {
    const uint64_t rec_bytes = 4 * ru4(cdiv(d, 2)) - 2 * (uint64_t)t.j0;
    t.rec_bytes = __builtin_amdgcn_readfirstlane(rec_bytes < 2u * kTile ? (uint32_t)rec_bytes : 2u * kTile);
  } else {
    t.rec_bytes = t.valid * 4;
  }
  t.base = uniform_off(g.part_base(t.p) + t.j0);
  return t;
}

// Stores the four values of a thread and row in the record's format and (EF) what that dropped.
template <bool EF, class FMT>
__device__ inline void cast_store_row(const CastTile &t, int u, const float q[4], uint8_t *values, float *residual) {
  float r[4], v[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    // q as an f32 value in a register: left to itself the compiler folds the multiplication by
    // 1/n that produced it into the conversion (one mixed-precision instruction that rounds the
    // exact product to a half once), and a mean over 3 workers then differs from the f32 mean
    // rounded to a half
    v[c] = q[c];
    asm("" : "+v"(v[c]));
  }
  const uint32_t row_bytes = u * kCRowElems * FMT::kBytes;
  const uint32_t in_row = t.rec_bytes > row_bytes ? t.rec_bytes - row_bytes : 0u;
  const TileBuf vb(values + row_bytes, in_row < (uint32_t)(FMT::kBytes * kCRowElems) ? in_row : (uint32_t)(FMT::kBytes * kCRowElems));
  if constexpr (FMT::kBytes == 2) {
    uint32_t packed[2];
#pragma unroll
    for (int c = 0; c < 4; c += 2) {
      const __half lo = __float2half_rn(v[c]), hi = __float2half_rn(v[c + 1]);
      packed[c / 2] = (uint32_t)__half_as_ushort(lo) | ((uint32_t)__half_as_ushort(hi) << 16);
      r[c] = v[c] - __half2float(lo);
      r[c + 1] = v[c + 1] - __half2float(hi);
    }
    u32x2 w;
    w.x = packed[0]; w.y = packed[1];
    vb.store8(w, threadIdx.x * 8);   // (the rows start 16 bytes off a line: not marked non-temporal)
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) r[c] = v[c] - v[c];   // (0, or NaN where q is not finite: q - decode(q) as written)
    vb.store16(as_u32x4(v[0], v[1], v[2], v[3]), threadIdx.x * 16);
  }
  if (EF) row_buf(residual + t.base, t.valid, u * kCRowElems, kCRowElems).store16<kNonTemporal>(as_u32x4(r[0], r[1], r[2], r[3]), threadIdx.x * 16);
}

template <class GT, bool EF, class FMT>
__global__ __launch_bounds__(kThreads) void cast_worker_kernel(Geo g, const GT *grad, float *residual, uint8_t *payload,
                                                               uint32_t *status) {
  if (blockIdx.x == 0 && threadIdx.x == 0) status[0] = 0;   // no wait in this call: the word reads "none gave up"
  const CastTile t = cast_tile<FMT>(g);
  uint8_t *rec = payload + (uint64_t)t.p * g.stride;
  if (t.j0 == 0 && threadIdx.x < 4) reinterpret_cast<uint32_t *>(rec)[threadIdx.x] = 0;
  const TileBuf gb(grad + t.base, t.valid * (uint32_t)sizeof(GT));
  const TileBuf eb(residual + (EF ? t.base : 0), EF ? t.valid * 4 : 0);
  typename Vec4Of<GT>::type gr[kCRows];
  u32x4 er[kCRows];
#pragma unroll
  for (int u = 0; u < kCRows; ++u) {
    gr[u] = tile_load4(gb, threadIdx.x * 4 * (uint32_t)sizeof(GT), u * kCRowElems * (uint32_t)sizeof(GT), (const GT *)nullptr);
    if (EF) er[u] = eb.load16<kNonTemporal>(threadIdx.x * 16, u * kCRowElems * 4);
  }
  patch_last_half<kCRows, kCRowElems>(gb, t.valid, gr);   // (f16 gradients of odd length)
#pragma unroll
  for (int u = 0; u < kCRows; ++u) {
    float q[4];
    widen4(gr[u], q);
    if (EF) {
      float e[4];
      widen4(er[u], e);
#pragma unroll
      for (int c = 0; c < 4; ++c) q[c] = q[c] + e[c];
    }
    cast_store_row<EF, FMT>(t, u, q, rec + kHeaderBytes + (uint64_t)FMT::kBytes * t.j0, residual);
  }
}

struct CastMsgs {
  const uint8_t *ptr[kMaxWorkers];
  int n;
  float inv_n;
};

// NW > 0: number of workers known at compile time; NW == 0: any number, four at a time.
template <bool EF, int NW, class FMT>
__global__ __launch_bounds__(kThreads) void cast_server_kernel(Geo g, CastMsgs msgs, float *residual, uint8_t *payload,
                                                               uint32_t *status) {
  if (blockIdx.x == 0 && threadIdx.x == 0) status[0] = 0;
  const CastTile t = cast_tile<FMT>(g);
  uint8_t *rec = payload + (uint64_t)t.p * g.stride;
  if (t.j0 == 0 && threadIdx.x < 4) reinterpret_cast<uint32_t *>(rec)[threadIdx.x] = 0;
  const uint64_t rec_off = uniform_off((uint64_t)t.p * g.stride + kHeaderBytes + (uint64_t)FMT::kBytes * t.j0);
  const TileBuf eb(residual + (EF ? t.base : 0), EF ? t.valid * 4 : 0);
  constexpr int kPair = FMT::kPair;   // rows whose loads are in flight together
  using Vec = typename FMT::Vec;
#pragma unroll 1
  for (int u0 = 0; u0 < kCRows; u0 += kPair) {
    float acc[kPair][4];
    u32x4 er[kPair];
#pragma unroll
    for (int k = 0; k < kPair; ++k) {
      if (EF) er[k] = eb.load16<kNonTemporal>(threadIdx.x * 16, (u0 + k) * kCRowElems * 4);
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[k][c] = 0.0f;
    }
    if (NW > 0) {
      Vec h[NW > 0 ? NW : 1][kPair];
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        const TileBuf mb(msgs.ptr[i] + rec_off, t.rec_bytes);
#pragma unroll
        for (int k = 0; k < kPair; ++k) h[i][k] = msg_load4<FMT>(mb, (u0 + k) * kCRowElems * FMT::kBytes);
      }
#pragma unroll
      for (int i = 0; i < NW; ++i) {
#pragma unroll
        for (int k = 0; k < kPair; ++k) {
          float v[4];
          widen4(h[i][k], v);
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[k][c] = acc[k][c] + v[c];
        }
      }
    } else {
      for (int i0 = 0; i0 < msgs.n; i0 += 4) {
        Vec h[4][kPair];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (i0 + i < msgs.n) {
            const TileBuf mb(msgs.ptr[i0 + i] + rec_off, t.rec_bytes);
#pragma unroll
            for (int k = 0; k < kPair; ++k) h[i][k] = msg_load4<FMT>(mb, (u0 + k) * kCRowElems * FMT::kBytes);
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (i0 + i < msgs.n) {
#pragma unroll
            for (int k = 0; k < kPair; ++k) {
              float v[4];
              widen4(h[i][k], v);
#pragma unroll
              for (int c = 0; c < 4; ++c) acc[k][c] = acc[k][c] + v[c];
            }
          }
        }
      }
    }
#pragma unroll
    for (int k = 0; k < kPair; ++k) {
      float q[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) q[c] = acc[k][c] * msgs.inv_n;
      if (EF) {
        float e[4];
        widen4(er[k], e);
#pragma unroll
        for (int c = 0; c < 4; ++c) q[c] = q[c] + e[c];
      }
      cast_store_row<EF, FMT>(t, u0 + k, q, rec + kHeaderBytes + (uint64_t)FMT::kBytes * t.j0, residual);
    }
  }
}

template <bool EF, class FMT>
static hipError_t launch_cast_server(const Geo &g, const Source &src, uint8_t *payload, uint32_t *status, hipStream_t stream) {
  CastMsgs m;
  for (int i = 0; i < kMaxWorkers; ++i) m.ptr[i] = i < src.msgs.n ? src.msgs.ptr[i] : nullptr;
  m.n = src.msgs.n;
  m.inv_n = src.msgs.inv_n;
  switch (m.n) {
    case 4: cast_server_kernel<EF, 4, FMT><<<g.n_tiles, kThreads, 0, stream>>>(g, m, src.residual, payload, status); break;
    case 8: cast_server_kernel<EF, 8, FMT><<<g.n_tiles, kThreads, 0, stream>>>(g, m, src.residual, payload, status); break;
    case 16: cast_server_kernel<EF, 16, FMT><<<g.n_tiles, kThreads, 0, stream>>>(g, m, src.residual, payload, status); break;
    default: cast_server_kernel<EF, 0, FMT><<<g.n_tiles, kThreads, 0, stream>>>(g, m, src.residual, payload, status); break;
  }
  return hipGetLastError();
}

template <class FMT>
static hipError_t cast_encode(const Geo &g, const Source &src, uint8_t *payload, const Workspace &ws, hipStream_t stream) {
  uint32_t *status = ws.status();
  float *res = src.residual;
  if (!src.grad) return res ? launch_cast_server<true, FMT>(g, src, payload, status, stream) : launch_cast_server<false, FMT>(g, src, payload, status, stream);
  if (src.dtype == BPC_F16) {
    const __half *gr = (const __half *)src.grad;
    if (res) cast_worker_kernel<__half, true, FMT><<<g.n_tiles, kThreads, 0, stream>>>(g, gr, res, payload, status);
    else cast_worker_kernel<__half, false, FMT><<<g.n_tiles, kThreads, 0, stream>>>(g, gr, res, payload, status);
  } else {
    const float *gr = (const float *)src.grad;
    if (res) cast_worker_kernel<float, true, FMT><<<g.n_tiles, kThreads, 0, stream>>>(g, gr, res, payload, status);
    else cast_worker_kernel<float, false, FMT><<<g.n_tiles, kThreads, 0, stream>>>(g, gr, res, payload, status);
  }
  return hipGetLastError();
}

hipError_t fp16_encode(const Geo &g, const bpc_params_t &, const Source &src, uint8_t *payload, const Workspace &ws,
                       hipStream_t stream) {
  return cast_encode<HalfFmt>(g, src, payload, ws, stream);
}

hipError_t identity_encode(const Geo &g, const bpc_params_t &, const Source &src, uint8_t *payload, const Workspace &ws,
                           hipStream_t stream) {
  return cast_encode<FloatFmt>(g, src, payload, ws, stream);
}

}  // namespace bpc
