// Kernel wrapper and launcher shared by the single-pass (cluster) kernels.
#pragma once
#include "cluster.hpp"
#include "kernels.hpp"

namespace bpc {

template <class Op>
__global__ __launch_bounds__(kCThreads, 4) void cluster_kernel(Op op, double *slots, uint32_t *status) {
  __shared__ float table[Op::kTableFloats];
  op.set_table(table);
  cluster_run(op, slots, status);
}

template <class Op>
static hipError_t launch_cluster(const Op &op, const ClusterGeo &cg, double *slots, uint32_t *status,
                                 hipStream_t stream, bool *used) {
  const void *fn = reinterpret_cast<const void *>(&cluster_kernel<Op>);
  static int capacity = 0;  // per kernel instantiation; a property of the device and the code object
  if (capacity == 0) capacity = cluster_capacity(fn);
  *used = false;
  if (capacity <= 0) return hipSuccess;
  uint32_t grid = cg.n_items < (uint32_t)capacity ? cg.n_items : (uint32_t)capacity;
  if (cg.tiles_per_part > grid) return hipSuccess;  // a partition must fit in the resident grid
  *used = true;
  hipError_t e = cluster_launch_begin(stream);
  if (e != hipSuccess) return e;
  slots_reset_kernel<<<(uint32_t)cdiv(cg.n_items, 256), 256, 0, stream>>>(slots, cg.n_items, status);
  cluster_kernel<Op><<<grid, kCThreads, 0, stream>>>(op, slots, status);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  return cluster_launch_end(stream);
}

}  // namespace bpc
