// Single-pass kernels that need a partition-wide reduction (a norm) between reading their
// inputs and writing their outputs keep each tile in registers and synchronise the
// workgroups that share a partition through global memory:
//
//   - the grid is persistent and launched cooperatively, so every workgroup is resident;
//   - work items (partition, tile) are numbered partition-major and workgroup w takes items
//     w, w+G, w+2G, ...; a partition has at most G tiles, so the tiles a workgroup waits
//     for always belong to workgroups that are ahead of nothing but earlier partitions
//     (no circular wait);
//   - every item owns one slot (an f64); it is preset to -1 and the workgroup publishes its
//     non-negative partial with one agent-scope atomic store.  The value is its own flag:
//     readers poll the slots of their partition with agent-scope atomic loads until none is
//     negative, so no fence (and no L2 write-back) is involved;
//   - the poll is bounded: after kSpinLimit rounds the workgroup records the failure in a
//     status word and carries on with the values it has, so the kernel always terminates.
#pragma once
#include "device_utils.hpp"
#include "geometry.hpp"

namespace bpc {

constexpr int kCThreads = 1024;               // workgroup size of the cluster kernels
constexpr int kCPerThread = 64;               // elements a thread keeps in registers
constexpr int kCTile = kCThreads * kCPerThread;  // 65536
constexpr int kSpinLimit = 1 << 22;

struct ClusterGeo {
  uint32_t tiles_per_part;  // kCTile-sized tiles of a full partition
  uint32_t n_items;         // tiles over all partitions
};

inline ClusterGeo make_cluster_geo(const Geo &g) {
  ClusterGeo c;
  c.tiles_per_part = (uint32_t)cdiv(g.part_elems, kCTile);
  uint64_t last = g.D - (uint64_t)(g.P - 1) * g.part_elems;
  c.n_items = (g.P - 1) * c.tiles_per_part + (uint32_t)cdiv(last, kCTile);
  return c;
}

#if defined(__HIPCC__)
__device__ inline void slot_publish(double *slot, double value) {
  __hip_atomic_store(slot, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by the first wave of a workgroup.  Polls the `count` slots starting at `slots`
// until all are published, then returns their sum (MAX = false) or maximum (MAX = true),
// combined in a fixed order, in every lane.
template <bool MAX>
__device__ inline double slots_collect(const double *slots, uint32_t count, uint32_t *status) {
  const uint32_t lane = threadIdx.x & 63;
  double v;
  int spins = 0;
  for (;;) {
    bool ok = true;
    v = 0.0;
    for (uint32_t s = lane; s < count; s += 64) {
      double x = __hip_atomic_load(slots + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ok = ok && x >= 0.0;
      x = x >= 0.0 ? x : 0.0;
      v = MAX ? fmax(v, x) : v + x;
    }
    if (__all(ok)) break;
    if (++spins > kSpinLimit) {
      if (lane == 0) atomicOr(status, 1u);
      break;
    }
    __builtin_amdgcn_s_sleep(16);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    double o = __shfl_xor(v, off, 64);
    v = MAX ? fmax(v, o) : v + o;
  }
  return v;
}

// Workgroup-wide sum / max of per-thread values (fixed order); result valid in wave 0.
template <bool MAX>
__device__ inline double cluster_block_reduce(double x, double *red /*kCThreads/64*/) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    double o = __shfl_xor(x, off, 64);
    x = MAX ? fmax(x, o) : x + o;
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = x;
  __syncthreads();
  double t = 0.0;
  if (wave == 0) {
    t = lane < kCThreads / 64 ? red[lane] : 0.0;
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) {
      double o = __shfl_xor(t, off, 64);
      t = MAX ? fmax(t, o) : t + o;
    }
  }
  return t;
}
#endif

}  // namespace bpc
