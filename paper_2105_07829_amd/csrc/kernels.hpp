// Launchers of the HIP kernels, one group per compressor.  Every launcher only
// enqueues work on `stream` and returns the first HIP error it saw.
#pragma once
#include <hip/hip_runtime.h>
#include "geometry.hpp"

namespace bpc {

// The n worker messages of an aggregate call, passed by value in the kernel arguments.
struct WorkerMsgs {
  const uint8_t *ptr[kMaxWorkers];
  uint64_t seed[kMaxWorkers];
  uint64_t stream_id[kMaxWorkers];
  int n;
  float inv_n;
  bool shared_scale;    // every worker's params name the same scale array (norm_override): the caller's
                        // statement that the workers compressed with one common scale per partition
};

// Where the worker-side q = g + e or the server-side Delta comes from.
struct Source {
  // worker: grad (+ residual); server: msgs (+ residual)
  const void *grad;     // NULL on the server
  int dtype;            // bpc_dtype_t of grad
  float *residual;      // e (worker) or e~ (server); NULL: no error feedback
  WorkerMsgs msgs;      // used when grad == NULL
};

struct Workspace {
  uint8_t *base;
  WsLayout lay;
  uint32_t run = 0;   // which run of partitions of the call this is: selects the status slot
  template <class T> T *at(size_t off) const { return reinterpret_cast<T *>(base + off); }
  uint32_t *status() const { return reinterpret_cast<uint32_t *>(base + lay.status) + 4 * run; }
  uint32_t *tickets() const { return reinterpret_cast<uint32_t *>(base + lay.tickets); }
};

hipError_t fill_zero(void *ptr, size_t bytes, hipStream_t stream);
// Streaming kernels with a stage's memory traffic and no arithmetic (bpc_stream_probe).
hipError_t stream_probe(int mix, const void *a, const void *b, void *c, uint64_t n, hipStream_t stream);

// The same call restricted to the ragged last partition: every pointer advanced past the
// `full_parts` full partitions that another kernel has taken.
inline void advance_to_tail(uint32_t full_parts, const Geo &g, Source *src, uint8_t **payload,
                            bpc_params_t *prm) {
  const uint64_t elems = (uint64_t)full_parts * g.part_elems;
  if (src->grad) src->grad = (const uint8_t *)src->grad + elems * (src->dtype == BPC_F16 ? 2 : 4);
  if (src->residual) src->residual += elems;
  for (int i = 0; i < src->msgs.n; ++i) src->msgs.ptr[i] += (uint64_t)full_parts * g.stride;
  *payload += (uint64_t)full_parts * g.stride;
  if (prm->norm_override) prm->norm_override += full_parts;
}

// C(q) and the residual update for each kind; the same entry serves worker and server.
hipError_t sign_encode(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                       const Workspace &ws, hipStream_t stream);
hipError_t dither_encode(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                         const Workspace &ws, hipStream_t stream);
hipError_t fp16_encode(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                       const Workspace &ws, hipStream_t stream);
hipError_t identity_encode(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                           const Workspace &ws, hipStream_t stream);
hipError_t topk_encode(const Geo &g, const bpc_params_t &prm, const bpc_params_t *in_prm, const Source &src,
                       uint8_t *payload, const Workspace &ws, hipStream_t stream);
hipError_t randk_encode(const Geo &g, const bpc_params_t &prm, const bpc_params_t *in_prm, const Source &src,
                        uint8_t *payload, const Workspace &ws, hipStream_t stream);

// out[idx] += decoded sparse entries (TOPK: plain store).  `out` holds the running sum.
hipError_t scatter_add_randk_shared(const Geo &g, const bpc_params_t &prm, const WorkerMsgs &msgs, float *out,
                                    hipStream_t stream);
hipError_t scatter_add_sparse(const Geo &g, const bpc_params_t &prm, const uint8_t *payload, float *out,
                              hipStream_t stream);

// Single-pass (register-resident, cluster-synchronised) variants.  *used = false means the
// shape is outside what they handle and nothing was enqueued.
hipError_t sign_worker_single_pass(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                                   const Workspace &ws, hipStream_t stream, bool *used);

hipError_t sign_server_single_pass(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                                   const Workspace &ws, hipStream_t stream, bool *used);
hipError_t dither_server_single_pass(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                                     const Workspace &ws, hipStream_t stream, bool *used);
hipError_t dither_worker_single_pass(const Geo &g, const bpc_params_t &prm, const Source &src, uint8_t *payload,
                                     const Workspace &ws, hipStream_t stream, bool *used);

// out = decode(payload), dense.
// Tables for the update kernel's sparse decoder (see update.hip).
constexpr uint32_t kRandkTableStride = 1025;
hipError_t topk_tile_starts(const Geo &g, const uint8_t *payload, bool half, uint32_t *table, uint32_t tile_shift,
                            hipStream_t stream);
hipError_t randk_bin_tiles(const Geo &g, const bpc_params_t &prm, const uint8_t *payload, uint2 *lists, uint32_t *table,
                           uint32_t tile_shift, hipStream_t stream);
hipError_t decode_dense(const Geo &g, const bpc_params_t &prm, const uint8_t *payload, float *out,
                        hipStream_t stream);

// Algorithm 5 update lines fused with the decode of bit-packed messages; sparse kinds are
// decoded into the workspace first.
hipError_t adaptive_update(const Geo &g, const bpc_params_t &prm, const uint8_t *payload, float *x, float *m,
                           float *v, const bpc_opt_t &opt, const Workspace &ws, hipStream_t stream);

}  // namespace bpc
