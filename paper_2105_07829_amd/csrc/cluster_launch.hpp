// Kernel wrappers and launcher shared by the single-pass (cluster) kernels.
#pragma once
#include "cluster.hpp"
#include "kernels.hpp"
#include <type_traits>

namespace bpc {

// Waves per SIMD the kernel is compiled for: 4 (at most 128 vector registers a lane) unless
// the operator asks for more with kWavesPerSimd.
template <class Op, class = void>
struct waves_per_simd { static constexpr int value = 4; };
template <class Op>
struct waves_per_simd<Op, std::void_t<decltype(Op::kWavesPerSimd)>> { static constexpr int value = Op::kWavesPerSimd; };

template <class Op>
__device__ inline void cluster_run(const Op &op, float *table, double *slots, uint32_t *status, uint32_t *tickets) {
  if constexpr (Op::kPersistent) cluster_run_persistent(op, table, slots, status, tickets);
  else cluster_run_ticketed(op, table, slots, status, tickets);
}

template <class Op>
__global__ __launch_bounds__(Op::kThreads, waves_per_simd<Op>::value) void cluster_kernel(const Op op, double *slots, uint32_t *status, uint32_t *tickets) {
  __shared__ __attribute__((aligned(16))) float table[Op::kTableFloats];
  cluster_run(op, table, slots, status, tickets);
}

// Same, with the operator's LDS scratch allocated at launch (sizes above the static limit).
template <class Op>
__global__ __launch_bounds__(Op::kThreads, waves_per_simd<Op>::value) void cluster_kernel_dyn(const Op op, double *slots, uint32_t *status, uint32_t *tickets) {
  extern __shared__ __attribute__((aligned(16))) float dyn_table[];
  cluster_run(op, dyn_table, slots, status, tickets);
}

// Launches `op` over the tiles of `cg`.  *used = false (and nothing is enqueued) when the
// shape cannot take the single-pass kernel: a partition has more tiles than the device holds
// workgroups at once.
template <class Op>
static hipError_t launch_cluster(const Op &op, const ClusterGeo &cg, double *slots, uint32_t *status, uint32_t *tickets,
                                 hipStream_t stream, bool *used, size_t dyn_lds = 0) {
  const void *fn = dyn_lds ? reinterpret_cast<const void *>(&cluster_kernel_dyn<Op>)
                           : reinterpret_cast<const void *>(&cluster_kernel<Op>);
  static PerDevice cache;  // resident workgroups of this kernel on each device
  const size_t max_dyn = dyn_lds ? (size_t)Op::kMaxDynLds : 0;
  const int capacity = cache.get([&]() -> int {
    if (max_dyn && hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dyn) != hipSuccess) {
      (void)hipGetLastError();
      return 0;
    }
    return cluster_capacity(fn, Op::kThreads, max_dyn);
  });
  *used = false;
  if (capacity <= 0) return hipSuccess;
  if (cg.tiles_per_part > (uint32_t)capacity) return hipSuccess;
  // the whole grid is resident at once
  const uint32_t grid = cg.n_items > (uint32_t)capacity ? (uint32_t)capacity : cg.n_items;
  *used = true;
  hipError_t e = cluster_launch_begin(stream);
  if (e != hipSuccess) return e;
  slots_reset_kernel<<<(uint32_t)cdiv(cg.n_items, 256), 256, 0, stream>>>(slots, cg.n_items, status, tickets);
  if (dyn_lds) cluster_kernel_dyn<Op><<<grid, Op::kThreads, dyn_lds, stream>>>(op, slots, status, tickets);
  else cluster_kernel<Op><<<grid, Op::kThreads, 0, stream>>>(op, slots, status, tickets);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  return cluster_launch_end(stream);
}

}  // namespace bpc
