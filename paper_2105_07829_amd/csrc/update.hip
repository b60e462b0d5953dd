// Moment and parameter update of compressed LANS (Algorithm 5, the lines after the push-pull
// call), fused with the decode of the pulled message g~ = decode(p_t).
//   ADAM : one launch, x -= lr * (r + wd*x)
//   LANS : moments + block norms (||x_b||, ||r + wd x||_b, ||c + wd x||_b, f64 sums), then
//          x -= lr * phi(||x_b||) * (beta1 (r+wd x)/||.|| + (1-beta1) (c+wd x)/||.||)
#include "sources.hpp"

namespace bpc {

struct SignDec {
  const uint8_t *payload; uint64_t stride;
  static constexpr int kLdsFloats = 1;
  __device__ void begin(uint32_t, float *) const {}
  __device__ float at(const Geo &, uint32_t p, uint32_t j, const float *) const {
    const uint8_t *rec = payload + (uint64_t)p * stride;
    float s = *reinterpret_cast<const float *>(rec);
    uint32_t w = reinterpret_cast<const uint32_t *>(rec + kHeaderBytes)[j >> 5];
    return ((w >> (j & 31)) & 1u) ? -s : s;
  }
};
struct DitherDec {
  const uint8_t *payload; uint64_t stride; uint32_t levels;
  static constexpr int kLdsFloats = 16;
  __device__ void begin(uint32_t p, float *lds) const {
    if (threadIdx.x < 16) {
      float nu = *reinterpret_cast<const float *>(payload + (uint64_t)p * stride);
      float mag = (nu * (float)(threadIdx.x & 7)) / (float)levels;
      lds[threadIdx.x] = (threadIdx.x & 8) ? -mag : mag;
    }
    __syncthreads();
  }
  __device__ float at(const Geo &, uint32_t p, uint32_t j, const float *lds) const {
    const uint32_t *nibs = reinterpret_cast<const uint32_t *>(payload + (uint64_t)p * stride + kHeaderBytes);
    return lds[(nibs[j >> 3] >> (4 * (j & 7))) & 15u];
  }
};
struct IdentityDec {
  const uint8_t *payload; uint64_t stride;
  static constexpr int kLdsFloats = 1;
  __device__ void begin(uint32_t, float *) const {}
  __device__ float at(const Geo &, uint32_t p, uint32_t j, const float *) const {
    return reinterpret_cast<const float *>(payload + (uint64_t)p * stride + kHeaderBytes)[j];
  }
};
struct DenseDec {
  const float *dense;
  static constexpr int kLdsFloats = 1;
  __device__ void begin(uint32_t, float *) const {}
  __device__ float at(const Geo &g, uint32_t p, uint32_t j, const float *) const { return dense[g.part_base(p) + j]; }
};

struct OptArgs {
  float lr, beta1, beta2, eps, wd, bc1, bc2, phi_lo, phi_hi;
  const uint64_t *block_offsets;  // device, or NULL: blocks are the partitions
  uint64_t n_blocks;
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

template <class DEC>
static hipError_t run_update(const Geo &g, DEC dec, float *x, float *m, float *v, const bpc_opt_t &opt,
                             double *norms, hipStream_t stream) {
  OptArgs o{opt.lr, opt.beta1, opt.beta2, opt.eps, opt.weight_decay, opt.bias_corr1, opt.bias_corr2,
            opt.phi_lo, opt.phi_hi, opt.block_offsets, opt.n_blocks};
  if (opt.kind == BPC_OPT_ADAM) {
    update_moments_kernel<DEC, false><<<g.n_tiles, kThreads, 0, stream>>>(g, dec, x, m, v, o, nullptr);
    return hipGetLastError();
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
    case BPC_SIGN: return run_update(g, SignDec{payload, g.stride}, x, m, v, opt, norms, stream);
    case BPC_DITHER: return run_update(g, DitherDec{payload, g.stride, prm.levels}, x, m, v, opt, norms, stream);
    case BPC_IDENTITY: return run_update(g, IdentityDec{payload, g.stride}, x, m, v, opt, norms, stream);
    default: {
      float *dense = ws.at<float>(ws.lay.dense);
      hipError_t e = decode_dense(g, prm, payload, dense, stream);
      if (e != hipSuccess) return e;
      return run_update(g, DenseDec{dense}, x, m, v, opt, norms, stream);
    }
  }
}

}  // namespace bpc
