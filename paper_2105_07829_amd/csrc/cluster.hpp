// Single-pass kernels that need a partition-wide reduction (a norm) between reading their
// inputs and writing their outputs keep each tile in registers and synchronise the
// workgroups that share a partition through global memory:
//
//   - every tile (partition, tile), numbered partition-major, owns one slot (an f64).  It is
//     preset to -1 and the workgroup that has the tile publishes its non-negative partial
//     with one agent-scope atomic store.  The value is its own flag: readers poll the slots
//     of their partition with agent-scope atomic loads until none is negative, so no fence
//     (and no L2 write-back) is involved;
//   - the poll is bounded: after kSpinLimit rounds the workgroup records the failure in a
//     status word and carries on with the values it has, so the kernel always terminates;
//   - partial results are combined in slot order, so the total does not depend on timing.
//
// Two drivers share this exchange.  Both are LAGGED: a workgroup publishes the partial of
// tile k, then finishes tile k-1 (collects its partition's total and writes its outputs), then
// goes on to tile k+1.  Tile k-1 was published a whole phase 1 earlier, so the other tiles of
// its partition have had that long to publish too, and collecting the total is as a rule one
// read of the slots instead of a wait; the price is a second copy of what a tile keeps for
// its phase 2.  A workgroup never waits while it holds a tile it has not published, so the
// oldest unpublished tile is always being worked on, and every wait ends provided the grid is
// resident as a whole and a partition has no more tiles than the grid (the launcher checks
// both).  They differ in how tiles get to workgroups:
//
//   PERSISTENT (cluster_run_persistent): workgroup w takes tiles w, w+G, w+2G, ... and
//     requests the loads of its next tile right after phase 1 of the current one, so the
//     memory pipeline of a compute unit stays busy across the exchange.  Used on the worker
//     side (two input streams per tile, one large workgroup per compute unit).
//   TICKETED (cluster_run_ticketed): a workgroup takes the number of its next tile from a
//     counter, so tiles are handed out in the order in which workgroups become free, and phase
//     1 issues its own loads.  There are C = min(kTicketClasses, grid) counters: workgroup w
//     draws from counter c = w % C, whose ticket t stands for tile t * C + c.  (Atomics on one
//     address are served one after the other, about 11 ns each: with a single counter the
//     13 K tiles of a 110 M element gradient were 0.15 ms of that unit's time, which a kernel
//     with little else to do -- few workers, no residual -- then took: 0.17 against 0.10 ms.)
//     Within a class tiles are taken in index order, and every class has at least
//     floor(grid / C) workgroups, so the argument below holds class by class: the lowest tile
//     never published would belong to a class all of whose workgroups hold two earlier tiles
//     of that class each, which puts it 2 C floor(grid / C) tiles past the oldest of them,
//     further than a partition reaches.  Used on the server side (n + 1 input streams and n-term sums
//     per tile): several workgroups per compute unit overlap each other's loads and
//     arithmetic, with no prefetch to keep in registers.
//   (Launching one workgroup per tile instead of a resident grid would tie each workgroup to
//   the XCD its index maps to; near the end of the grid the tiles still to come would all
//   belong to the one or two XCDs that are behind, too few workgroups to hold a partition.)
#pragma once
#include "device_utils.hpp"
#include "geometry.hpp"
#include <hip/hip_runtime.h>
#include <type_traits>
#include <utility>

namespace bpc {

constexpr int kSpinLimit = 1 << 22;

struct ClusterGeo {
  uint32_t tiles_per_part;  // tiles of a full partition
  uint32_t n_items;         // tiles over all partitions
};

// A full partition must be a whole number of tiles of `tile` elements; a shorter last
// partition has the tiles it needs, the last of them possibly ragged.
inline ClusterGeo make_cluster_geo(const Geo &g, uint32_t tile) {
  ClusterGeo c;
  c.tiles_per_part = (uint32_t)(g.part_elems / tile);
  const uint32_t p_full = (uint32_t)(g.D / g.part_elems);
  c.n_items = p_full * c.tiles_per_part + (uint32_t)cdiv(g.D - (uint64_t)p_full * g.part_elems, tile);
  return c;
}

// Splits a gradient into the part the single-pass kernels take and the part left to the
// multi-pass kernels.  `ragged_ok`: the single-pass kernel bounds its accesses to a shorter
// last partition itself; otherwise it gets the full partitions only.
struct SplitGeo {
  bool single_pass;   // false: the partition size is not a multiple of the tile
  Geo head;           // what the single-pass kernel takes (head.D may be 0)
  Geo tail;           // the last, shorter partition as a one-partition gradient (tail.D may be 0)
};
inline SplitGeo split_geo(const Geo &g, uint32_t tile, bool ragged_ok) {
  SplitGeo s;
  s.single_pass = g.part_elems % tile == 0;
  if (ragged_ok) {
    s.head = g;
    s.tail = g;
    s.tail.D = 0;
    s.tail.P = 0;
    s.tail.n_tiles = 0;
    return s;
  }
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

// Host side: the arguments above count the resident workgroups of ONE kernel.  Two cluster
// kernels running concurrently (different streams) would share the device, so launches are
// chained: a launch on another stream than the one before first waits for an event recorded
// on that earlier stream.
hipError_t cluster_launch_begin(hipStream_t stream);
hipError_t cluster_launch_end(hipStream_t stream);
// Creates the current device's event now rather than at the first launch that needs it.
hipError_t cluster_prepare_device();
// Number of workgroups of `kernel` (`threads` threads, `dyn_lds` bytes of dynamic LDS) resident at once
// on the current device; 0 if the query failed.
int cluster_capacity(const void *kernel, int threads, size_t dyn_lds = 0);

// 1 if `kernel` may now be launched with up to `bytes` of dynamic LDS on the current device, else 0.
int lds_limit_raised(const void *kernel, size_t bytes);

// A positive integer per device that is found out once (an occupancy figure, "this function
// attribute is set").  One zero-initialised static instance per kernel.  Answers <= 0 (a failed
// query) are handed back but never kept, so the next call asks again.
constexpr int kMaxDevices = 64;
struct PerDevice {
  int v[kMaxDevices];
  template <class F>
  int get(F query) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return query();
    int cur = __atomic_load_n(&v[dev], __ATOMIC_ACQUIRE);
    if (cur > 0) return cur;
    cur = query();
    if (cur > 0) __atomic_store_n(&v[dev], cur, __ATOMIC_RELEASE);
    return cur;
  }
};

#if defined(__HIPCC__)
// Presets the slots to "not published", clears the status word and (if given) the ticket counters.
__global__ void slots_reset_kernel(double *slots, uint32_t n, uint32_t *status, uint32_t *tickets);

// A slot is unpublished while it holds exactly the preset -1.0.  Partials are sums of
// magnitudes or squares, so no published value has that bit pattern, whatever the inputs
// (a NaN partial from non-finite inputs still counts as published: no wait depends on the data).
constexpr long long kSlotUnpublished = (long long)0xBFF0000000000000ull;
__device__ inline bool slot_published(double x) { return __double_as_longlong(x) != kSlotUnpublished; }
__device__ inline void slot_publish(double *slot, double value) {
  __hip_atomic_store(slot, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Two neighbouring slots in one 16-byte load that goes to the memory side like the atomic loads
// (each slot is written with one 8-byte store, so either half is a whole old or new value);
// slots past `bytes` read as 0.0, a published nothing.  Reading a partition's 256 slots with
// four 8-byte loads a lane instead was 6 % of the dithering worker with 8192-element tiles.
constexpr int kMemorySide = 16;   // cache policy of a buffer access: coherent at the level of the device
__device__ inline void slot_pair(const TileBuf &b, uint32_t pair, double *x0, double *x1) {
  const u32x4 w = b.load16<kMemorySide>(pair * 16, 0);
  *x0 = __longlong_as_double((long long)(((unsigned long long)w.y << 32) | w.x));
  *x1 = __longlong_as_double((long long)(((unsigned long long)w.w << 32) | w.z));
}

// Called by the first wave of a workgroup.  Polls the `count` slots starting at `slots`
// until all are published, then returns their sum (MAX = false) or maximum (MAX = true),
// combined in a fixed order, in every lane.
template <bool MAX>
__device__ inline double slots_collect(const double *slots, uint32_t count, uint32_t *status) {
  const uint32_t lane = threadIdx.x & 63;
  const TileBuf b(slots, count * 8);
  double v;
  int spins = 0;
  for (;;) {
    bool ok = true;
    v = 0.0;
    for (uint32_t s = lane; 2 * s < count; s += 64) {
      double x[2];
      slot_pair(b, s, &x[0], &x[1]);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bool pub = slot_published(x[h]);
        ok = ok && pub;
        const double y = pub ? x[h] : 0.0;
        v = MAX ? fmax(v, y) : v + y;
      }
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

// The same in two steps for the persistent driver: slots_probe() reads every slot once without
// waiting for the values (the loads stay in flight under whatever the caller does next), and
// slots_finish() uses them if all were published, else falls back to slots_collect().  Both
// combine in the same order, so the result does not depend on which one produced it.  A probe
// covers partitions of up to 256 tiles.
struct SlotProbe { double v; bool ok; };
template <bool MAX>
__device__ inline SlotProbe slots_probe(const double *slots, uint32_t count) {
  const uint32_t lane = threadIdx.x & 63;
  SlotProbe r{0.0, count <= 256u};
  if (count <= 256u) {
    const TileBuf b(slots, count * 8);
#pragma unroll
    for (uint32_t j = 0; j < 2; ++j) {
      double x[2];
      slot_pair(b, lane + 64 * j, &x[0], &x[1]);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bool pub = slot_published(x[h]);
        r.ok = r.ok && pub;
        const double y = pub ? x[h] : 0.0;
        r.v = MAX ? fmax(r.v, y) : r.v + y;
      }
    }
  }
  return r;
}
template <bool MAX>
__device__ inline double slots_finish(const SlotProbe &probe, const double *slots, uint32_t count, uint32_t *status) {
  if (!__all(probe.ok)) return slots_collect<MAX>(slots, count, status);
  double v = probe.v;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    double o = __shfl_xor(v, off, 64);
    v = MAX ? fmax(v, o) : v + o;
  }
  return v;
}

// Workgroup-wide sum / max of per-thread values (fixed order); result valid in wave 0.
template <bool MAX, int THREADS>
__device__ inline double cluster_block_reduce(double x, double *red /*THREADS/64*/) {
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
    t = lane < THREADS / 64 ? red[lane] : 0.0;
#pragma unroll
    for (int off = THREADS / 128; off > 0; off >>= 1) {
      double o = __shfl_xor(t, off, 64);
      t = MAX ? fmax(t, o) : t + o;
    }
  }
  return t;
}

// What the drivers ask of an operator `Op`:
//   struct Raw, struct Held, struct Ctx;         raw loads of a tile / what is kept for phase 2
//   static constexpr int kThreads;               workgroup size
//   static constexpr bool kPersistent;           which driver
//   uint32_t n_items() const;  bool needs_total() const;
//   void   issue_row(item, row, Raw&) const;     (persistent) request a row of the tile's inputs
//   double phase1(item, Raw&, Held&, table) const;   consume the loads (ticketed: request them
//                                                first), return the tile's partial
//   void   early(item, Held&) const;             stores that do not need the norm
//   float  scale_of(item, total) const;         the partition's scale from the total (one thread
//                                                forms it: a division or a root of doubles per
//                                                thread and tile was a sixth of the sign kernels'
//                                                instructions)
//   Ctx    begin2(item, scale, table) / row2(item, row, Held&, Ctx) const;   outputs of one row
//   void   slots_of(item, first, count)          the partition's slots
//   static constexpr int kRowsPerTile; static constexpr bool kMax (maximum instead of sum)
//   static constexpr int kTableFloats (LDS scratch, `table`)
// The operator is passed by value in the kernel arguments and never modified, so it stays in
// the kernel-argument segment (a modified copy would live in scratch memory).

// An operator may have `void init(table) const`, called once per workgroup before its first tile
// (tables in the LDS scratch that do not depend on the tile; the first barrier of the loop
// orders them before their use).
template <class Op, class = void>
struct has_init { static constexpr bool value = false; };
template <class Op>
struct has_init<Op, std::void_t<decltype(std::declval<const Op &>().init((float *)nullptr))>> { static constexpr bool value = true; };

// Ticketed driver.
template <class Op>
__device__ inline void cluster_run_ticketed(const Op &op, float *table, double *slots, uint32_t *status, uint32_t *tickets) {
  constexpr int kT = Op::kThreads;
  constexpr uint32_t kNone = 0xffffffffu;
  __shared__ double red[kT / 64];
  __shared__ float scale_sh;
  __shared__ uint32_t item_sh;
  const uint32_t n_items = op.n_items();
  typename Op::Held held_prev;
  uint32_t prev = kNone;
  const uint32_t n_classes = gridDim.x < (uint32_t)kTicketClasses ? gridDim.x : (uint32_t)kTicketClasses;
  const uint32_t cls = blockIdx.x % n_classes;
  uint32_t *counter = tickets + cls * (kTicketStride / 4);
  if (threadIdx.x == 0) item_sh = atomicAdd(counter, 1u) * n_classes + cls;
  if constexpr (has_init<Op>::value) op.init(table);
  __syncthreads();
  uint32_t item = __builtin_amdgcn_readfirstlane(item_sh);
  for (;;) {
    const bool have = item < n_items;
    if (!have && prev == kNone) break;
    typename Op::Held held;
    if (have) {
      typename Op::Raw raw;
      double part = op.phase1(item, raw, held, table);
      part = cluster_block_reduce<Op::kMax, kT>(part, red);
      if (threadIdx.x == 0 && op.needs_total()) slot_publish(slots + item, part);
    }
    uint32_t ticket = kNone;
    // (reading the older tile's slots before phase 1, as the persistent driver does,
    // was slower here: phase 1 of these operators has no registers to spare for the values)
    if (prev != kNone && threadIdx.x < 64) {
      double total = 0.0;
      if (op.needs_total()) {
        uint32_t first, count;
        op.slots_of(prev, &first, &count);
        total = slots_collect<Op::kMax>(slots + first, count, status);
      }
      if (threadIdx.x == 0) scale_sh = op.scale_of(prev, total);
    }
    // the next ticket is on its way while the older tile is written out
    if (have && threadIdx.x == 0) ticket = atomicAdd(counter, 1u) * n_classes + cls;
    if (have) op.early(item, held);
    __syncthreads();
    if (prev != kNone) {
      const typename Op::Ctx ctx = op.begin2(prev, scale_sh, table);
#pragma unroll
      for (int u = 0; u < Op::kRowsPerTile; ++u) op.row2(prev, u, held_prev, ctx);
    }
    if (!have) break;
    held_prev = held;
    prev = item;
    if (threadIdx.x == 0) item_sh = ticket;
    __syncthreads();
    item = __builtin_amdgcn_readfirstlane(item_sh);
  }
}

// Persistent driver.  The older tile's slots are read before phase 1 of the current tile and
// looked at after it, so that read is off the critical path as well.
template <class Op>
__device__ inline void cluster_run_persistent(const Op &op, float *table, double *slots, uint32_t *status, uint32_t *) {
  constexpr int kT = Op::kThreads;
  constexpr uint32_t kNone = 0xffffffffu;
  __shared__ double red[kT / 64];
  __shared__ float scale_sh;
  const uint32_t n_items = op.n_items();
  uint32_t item = __builtin_amdgcn_readfirstlane(blockIdx.x);
  if (item >= n_items) return;
  typename Op::Raw raw;
#pragma unroll
  for (int u = 0; u < Op::kRowsPerTile; ++u) op.issue_row(item, u, raw);
  __builtin_amdgcn_s_waitcnt(0x0F70);
  typename Op::Held held_prev;
  uint32_t prev = kNone;
  for (;;) {
    typename Op::Held held;
    // the older tile's slots are read now and looked at after phase 1
    SlotProbe probe{0.0, false};
    const bool collects = prev != kNone && threadIdx.x < 64 && op.needs_total();
    uint32_t first = 0, count = 0;
    if (collects) {
      op.slots_of(prev, &first, &count);
      probe = slots_probe<Op::kMax>(slots + first, count);
    }
    double part = op.phase1(item, raw, held, table);
    const uint32_t next = __builtin_amdgcn_readfirstlane(item + gridDim.x);
    const bool have_next = next < n_items;
    if (have_next) {
#pragma unroll
      for (int u = 0; u < Op::kRowsPerTile; ++u) op.issue_row(next, u, raw);
    }
    part = cluster_block_reduce<Op::kMax, kT>(part, red);
    if (threadIdx.x == 0 && op.needs_total()) slot_publish(slots + item, part);
    if (prev != kNone && threadIdx.x < 64) {
      double total = 0.0;
      if (collects) total = slots_finish<Op::kMax>(probe, slots + first, count, status);
      if (threadIdx.x == 0) scale_sh = op.scale_of(prev, total);
    }
    op.early(item, held);
    __syncthreads();
    if (prev != kNone) {
      const typename Op::Ctx ctx = op.begin2(prev, scale_sh, table);
#pragma unroll
      for (int u = 0; u < Op::kRowsPerTile; ++u) op.row2(prev, u, held_prev, ctx);
    }
    held_prev = held;
    prev = item;
    if (!have_next) break;
    item = next;
    __syncthreads();
  }
  // the last tile
  __syncthreads();
  if (threadIdx.x < 64) {
    double total = 0.0;
    if (op.needs_total()) {
      uint32_t first, count;
      op.slots_of(prev, &first, &count);
      total = slots_collect<Op::kMax>(slots + first, count, status);
    }
    if (threadIdx.x == 0) scale_sh = op.scale_of(prev, total);
  }
  __syncthreads();
  const typename Op::Ctx ctx = op.begin2(prev, scale_sh, table);
#pragma unroll
  for (int u = 0; u < Op::kRowsPerTile; ++u) op.row2(prev, u, held_prev, ctx);
}
#endif

}  // namespace bpc
