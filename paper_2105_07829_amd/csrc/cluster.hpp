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
#include <hip/hip_runtime.h>

namespace bpc {

constexpr int kCThreads = 1024;               // workgroup size of the cluster kernels (one per CU)
constexpr int kCPerThread = 32;               // elements a thread keeps in registers
constexpr int kCTile = kCThreads * kCPerThread;  // 32768
constexpr int kSpinLimit = 1 << 22;

struct ClusterGeo {
  uint32_t tiles_per_part;  // kCTile-sized tiles of a full partition
  uint32_t n_items;         // tiles over all partitions
};

// `g` must describe full partitions only, each a whole number of tiles.
inline ClusterGeo make_cluster_geo(const Geo &g) {
  ClusterGeo c;
  c.tiles_per_part = (uint32_t)(g.part_elems / kCTile);
  c.n_items = g.P * c.tiles_per_part;
  return c;
}

// Splits a gradient into the part the single-pass kernels take (whole partitions that are a
// whole number of tiles) and the ragged last partition, if any.
struct SplitGeo {
  bool single_pass;   // false: the partition size is not a multiple of the tile
  Geo head;           // the full partitions (head.D may be 0)
  Geo tail;           // the last, shorter partition as a one-partition gradient (tail.D may be 0)
};
inline SplitGeo split_geo(const Geo &g) {
  SplitGeo s;
  s.single_pass = g.part_elems % kCTile == 0;
  const uint32_t p_full = (uint32_t)(g.D / g.part_elems);
  s.head = g;
  s.head.D = (uint64_t)p_full * g.part_elems;
  s.head.P = p_full;
  s.head.n_tiles = p_full * g.tiles_per_part;
  s.tail = g;
  s.tail.D = g.D - s.head.D;
  s.tail.P = s.tail.D ? 1 : 0;
  s.tail.n_tiles = (uint32_t)cdiv(s.tail.D, kTile);
  s.tail.part0 = g.part0 + p_full;
  return s;
}

// Host side: cluster kernels are launched as ordinary kernels whose grid never exceeds what
// the device can hold at once.  Two of them running concurrently (different streams) could
// each end up partly resident and wait for each other's slots, so launches are chained:
// every launch records an event, and a launch on another stream first waits for it.
hipError_t cluster_launch_begin(hipStream_t stream);
hipError_t cluster_launch_end(hipStream_t stream);
// Number of workgroups of `kernel` (kCThreads threads, `dyn_lds` bytes of dynamic LDS) resident at once.
int cluster_capacity(const void *kernel, size_t dyn_lds = 0);

#if defined(__HIPCC__)
__global__ void slots_reset_kernel(double *slots, uint32_t n, uint32_t *status);

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
    for (int off = kCThreads / 128; off > 0; off >>= 1) {
      double o = __shfl_xor(t, off, 64);
      t = MAX ? fmax(t, o) : t + o;
    }
  }
  return t;
}

// Persistent, software-pipelined driver over the tiles of the full partitions (a ragged last
// partition is left to the multi-pass kernels).  `Op` supplies:
//   struct Raw, struct Held, struct Ctx;         raw loads of a tile / what is kept for phase 2
//   uint32_t n_items() const;
//   void   issue_row(item, row, Raw&) const;     start the loads of one row of a tile
//   double phase1(item, Raw&, Held&, table) const;   consume the loads, return the tile's partial
//   void   early(item, Held&) const;             stores that do not need the norm
//   Ctx    begin2(item, total, table) / row2(item, row, Held&, Ctx) const;   outputs of one row
//   void   slots_of(item, first, count)          the partition's slots
//   static constexpr int kRowsPerTile; static constexpr bool kMax (maximum instead of sum)
//   static constexpr Prefetch kPrefetch; static constexpr int kTableFloats (LDS scratch, `table`)
// The operator is passed by value in the kernel arguments and never modified, so it stays in
// the kernel-argument segment (a modified copy would live in scratch memory).
// The loads of a workgroup's next tile overlap its work on the current one (see Prefetch).
// When a tile's loads are issued relative to the work on the previous tile.
enum class Prefetch {
  kEarly,        // all of them right after phase 1 of the previous tile (phase 2 is mostly stores)
  kInterleaved,  // row by row between the rows of output of the previous tile (phase 2 is
                 // arithmetic-heavy: loads, arithmetic and stores of the CU interleave)
  kNone          // not ahead of time: phase 1 issues its own loads and hides them behind its
                 // arithmetic
};

template <class Op>
__device__ inline void cluster_run(const Op &op, float *table, double *slots, uint32_t *status) {
  __shared__ double red[kCThreads / 64];
  __shared__ double total_sh;
  const uint32_t n_items = op.n_items();
  // item numbers are the same for every lane: keeping them in scalar registers makes all
  // tile addresses scalar
  uint32_t item = __builtin_amdgcn_readfirstlane(blockIdx.x);
  if (item >= n_items) return;
  typename Op::Raw raw;
  if (Op::kPrefetch != Prefetch::kNone) {
#pragma unroll
    for (int u = 0; u < Op::kRowsPerTile; ++u) op.issue_row(item, u, raw);
  }
  for (;;) {
    typename Op::Held held;
    double part = op.phase1(item, raw, held, table);
    const uint32_t next = __builtin_amdgcn_readfirstlane(item + gridDim.x);
    const bool have_next = next < n_items;
    if (Op::kPrefetch == Prefetch::kEarly && have_next) {
#pragma unroll
      for (int u = 0; u < Op::kRowsPerTile; ++u) op.issue_row(next, u, raw);
    }
    part = cluster_block_reduce<Op::kMax>(part, red);
    if (threadIdx.x < 64) {
      uint32_t first, count;
      op.slots_of(item, &first, &count);
      if (op.needs_total()) {
        if (threadIdx.x == 0) slot_publish(slots + item, part);
        double total = slots_collect<Op::kMax>(slots + first, count, status);
        if (threadIdx.x == 0) total_sh = total;
      }
    }
    op.early(item, held);
    __syncthreads();
    const double total = total_sh;
    const typename Op::Ctx ctx = op.begin2(item, total, table);
#pragma unroll
    for (int u = 0; u < Op::kRowsPerTile; ++u) {
      op.row2(item, u, held, ctx);
      if (Op::kPrefetch == Prefetch::kInterleaved && have_next) op.issue_row(next, u, raw);
    }
    if (!have_next) break;
    item = next;
    __syncthreads();
  }
}
#endif

}  // namespace bpc
