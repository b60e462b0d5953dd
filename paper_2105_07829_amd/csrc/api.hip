// C ABI (include/bpc.h): argument validation on the host, then dispatch to the kernel
// launchers.  Nothing here allocates, and only bpc_workspace_check() synchronises.
#include <hip/hip_runtime.h>
#include <mutex>
#include "cluster.hpp"
#include "kernels.hpp"

using namespace bpc;

// Workspace of bpc_compress_static_ws(): each device the library runs on holds this array until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress();
// the address kernels and copies are given is the one that call returned for the device.
static __device__ __align__(256) unsigned char scratch[BPC_STATIC_WS_BYTES];

static thread_local int g_last_hip_error = 0;

static bpc_status_t hip_status(hipError_t e) {
  if (e == hipSuccess) return BPC_OK;
  g_last_hip_error = (int)e;
  return BPC_ERR_HIP;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Device address of `scratch` on the current device, looked up once per device (together with
// the event that orders single-pass kernels across streams, so that no later call creates one).
static hipError_t static_workspace(uint8_t **ptr) {
  static std::mutex mu;
  static uint8_t *addr[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    e = cluster_prepare_device();
    if (e != hipSuccess) return e;
    addr[dev] = static_cast<uint8_t *>(p);
  }
  *ptr = addr[dev];
  return hipSuccess;
}

// A call whose params carry a bypass mask (Section 4.2: tensors under a size threshold are not
// compressed) is carried out run by run: a run is a maximal stretch of partitions of one class,
// compressed by the params' kind or carried as they are (identity records).  Without a mask
// the whole gradient is one run.
struct Run {
  uint32_t p0, n_parts;   // partitions [p0, p0 + n_parts)
  bool bypass;
  uint64_t elem0, elems;  // their elements [elem0, elem0 + elems)
  size_t pay_off;         // byte offset of record p0 in a payload
};
struct Runs {
  int n;
  Run r[kMaxRuns];
  size_t payload_bytes;
};
static size_t identity_stride(uint64_t part_elems) { return kHeaderBytes + 4 * ru4(part_elems); }
// false: more runs than a call accepts.
static bool make_runs(const bpc_params_t *prm, uint64_t D, Runs *out) {
  const uint64_t P = cdiv(D, prm->part_elems);
  out->n = 0;
  size_t off = 0;
  for (uint64_t p = 0; p < P;) {
    const bool by = prm->bypass && prm->bypass[p] != 0;
    uint64_t q = p + 1;
    while (q < P && (prm->bypass && prm->bypass[q] != 0) == by) ++q;
    if (out->n == kMaxRuns) return false;
    Run &r = out->r[out->n++];
    r.p0 = (uint32_t)p;
    r.n_parts = (uint32_t)(q - p);
    r.bypass = by;
    r.elem0 = p * prm->part_elems;
    r.elems = (q * prm->part_elems < D ? q * prm->part_elems : D) - r.elem0;
    r.pay_off = off;
    off += (size_t)(q - p) * (by ? identity_stride(prm->part_elems) : stride_of(prm));
    p = q;
  }
  out->payload_bytes = off;
  return true;
}
// The params of one run as a call of its own.
static bpc_params_t run_params(const bpc_params_t *prm, const Run &r) {
  bpc_params_t s = *prm;
  s.bypass = nullptr;
  if (r.bypass) s.kind = BPC_IDENTITY;
  if (s.norm_override) s.norm_override += r.p0;
  return s;
}
static Geo run_geo(const bpc_params_t &sub, const Run &r) {
  Geo g = make_geo(&sub, r.elems);
  g.part0 = r.p0;
  return g;
}

// Every run's own workspace layout fits in ws_bytes (they all do when ws_bytes covers the layout
// of the whole call, which is what the entry points ask for; checked all the same).
static bool runs_fit(const bpc_params_t *prm, const Runs &runs, size_t ws_bytes) {
  for (int k = 0; k < runs.n; ++k) {
    const bpc_params_t sub = run_params(prm, runs.r[k]);
    if (ws_layout(&sub, runs.r[k].elems).total > ws_bytes) return false;
  }
  return true;
}

extern "C" {

uint64_t bpc_partition_k(const bpc_params_t *params, uint64_t d) {
  if (!params_valid(params) || d == 0) return 0;
  if (params->kind != BPC_TOPK && params->kind != BPC_TOPK16 && params->kind != BPC_RANDK) return 0;
  return k_rule(params->k_ratio, d);
}

size_t bpc_partition_stride(const bpc_params_t *params) {
  if (!params_valid(params)) return 0;
  return stride_of(params);
}

size_t bpc_payload_bytes(const bpc_params_t *params, uint64_t D) {
  if (!params_valid(params) || D == 0) return 0;
  Runs runs;
  if (!make_runs(params, D, &runs)) return 0;
  return runs.payload_bytes;
}

size_t bpc_partition_offset(const bpc_params_t *params, uint64_t D, uint64_t p) {
  if (!params_valid(params) || p >= cdiv(D, params->part_elems)) return (size_t)-1;
  Runs runs;
  if (!make_runs(params, D, &runs)) return (size_t)-1;
  for (int k = 0; k < runs.n; ++k) {
    const Run &r = runs.r[k];
    if (p < (uint64_t)r.p0 + r.n_parts)
      return r.pay_off + (size_t)(p - r.p0) * (r.bypass ? identity_stride(params->part_elems) : stride_of(params));
  }
  return (size_t)-1;
}

size_t bpc_workspace_bytes(const bpc_params_t *params, uint64_t D, int n) {
  if (!params_valid(params) || n < 1 || n > kMaxWorkers) return 0;
  if (D == 0) return 256;
  return ws_layout(params, D).total;
}

size_t bpc_workspace_status_offset(const bpc_params_t *params, uint64_t D) {
  if (!params_valid(params)) return (size_t)-1;
  if (D == 0) return 0;
  return ws_layout(params, D).status;
}

// Workspace of an update call: LANS with caller-defined blocks keeps three f64 sums per block
// where the layout has room for three per partition.
static size_t update_ws_bytes(const WsLayout &lay, bool caller_blocks, uint64_t n_blocks, uint64_t D) {
  size_t need = lay.total;
  if (caller_blocks) {
    // three f64 sums per block (the two-launch form) or the tables of the one-pass form
    size_t with_blocks = lay.norms + (sizeof(double) * 3 * (size_t)n_blocks + 255) / 256 * 256;
    const size_t one_pass = lay.norms + block_ws(nullptr, n_blocks, cdiv(D, kSTile)).bytes;
    if (one_pass > with_blocks) with_blocks = one_pass;
    if (with_blocks > need) need = with_blocks;
  }
  return need;
}

size_t bpc_update_workspace_bytes(const bpc_params_t *params, uint64_t D, uint64_t n_blocks) {
  if (!params_valid(params) || n_blocks > (1ull << 40)) return 0;
  if (D == 0) return 256;
  return update_ws_bytes(ws_layout(params, D), n_blocks != 0, n_blocks, D);
}

bpc_status_t bpc_workspace_check(const bpc_params_t *params, uint64_t D, const void *ws, void *hip_stream) {
  if (!params_valid(params)) return BPC_ERR_INVALID_ARG;
  if (D != 0 && !ws) {
    // the static workspace of the current device
    if (ws_layout(params, D).total > BPC_STATIC_WS_BYTES) return BPC_ERR_WORKSPACE;
    uint8_t *st = nullptr;
    hipError_t e0 = static_workspace(&st);
    if (e0 != hipSuccess) return hip_status(e0);
    ws = st;
  }
  Runs runs;
  runs.n = 1;
  if (D != 0 && !make_runs(params, D, &runs)) return BPC_ERR_UNSUPPORTED;
  hipError_t e = hipStreamSynchronize((hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_status(e);
  if (D == 0) return BPC_OK;
  // one slot of four words per run; word 0 of a slot is the run's flag
  uint32_t words[4 * kMaxRuns];
  e = hipMemcpy(words, (const uint8_t *)ws + ws_layout(params, D).status, 16 * (size_t)runs.n, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_status(e);
  for (int k = 0; k < runs.n; ++k)
    if (words[4 * k] != 0) return BPC_ERR_WAIT;
  return BPC_OK;
}

static bpc_status_t check_size(const bpc_params_t *p, uint64_t D) {
  // element offsets inside kernels are 64 bit, tile and partition counts 32 bit
  if (D / kTile >= 0x7fffffffull) return BPC_ERR_UNSUPPORTED;
  // the sparse kinds have launches with the partition number in the second grid dimension
  const bool sparse = p->kind == BPC_TOPK || p->kind == BPC_TOPK16 || p->kind == BPC_RANDK;
  if (sparse && cdiv(D, p->part_elems) > 65535) return BPC_ERR_UNSUPPORTED;
  return BPC_OK;
}

static hipError_t encode(const Geo &g, const bpc_params_t &prm, const bpc_params_t *in_prm, const Source &src,
                         uint8_t *payload, const Workspace &ws, hipStream_t stream) {
  switch (prm.kind) {
    case BPC_IDENTITY: return identity_encode(g, prm, src, payload, ws, stream);
    case BPC_FP16: return fp16_encode(g, prm, src, payload, ws, stream);
    case BPC_SIGN: return sign_encode(g, prm, src, payload, ws, stream);
    case BPC_TOPK: case BPC_TOPK16: return topk_encode(g, prm, in_prm, src, payload, ws, stream);
    case BPC_RANDK: return randk_encode(g, prm, in_prm, src, payload, ws, stream);
    default: return dither_encode(g, prm, src, payload, ws, stream);
  }
}

bpc_status_t bpc_compress(const bpc_params_t *params, const void *grad, bpc_dtype_t dtype, float *residual,
                          uint64_t D, void *payload, void *ws, size_t ws_bytes, void *hip_stream) {
  if (!params_valid(params)) return BPC_ERR_INVALID_ARG;
  if (dtype != BPC_F32 && dtype != BPC_F16) return BPC_ERR_INVALID_ARG;
  if (D == 0) return BPC_OK;
  if (!grad || !payload) return BPC_ERR_INVALID_ARG;
  if (check_size(params, D) != BPC_OK) return BPC_ERR_UNSUPPORTED;
  if (!aligned16(grad) || !aligned16(residual) || !aligned16(payload) || !aligned16(ws) ||
      !aligned16(params->norm_override))
    return BPC_ERR_ALIGNMENT;
  WsLayout lay = ws_layout(params, D);
  if (!ws || ws_bytes < lay.total) return BPC_ERR_WORKSPACE;
  Runs runs;
  if (!make_runs(params, D, &runs)) return BPC_ERR_UNSUPPORTED;
  if (!runs_fit(params, runs, ws_bytes)) return BPC_ERR_WORKSPACE;
  const size_t gbytes = dtype == BPC_F16 ? 2 : 4;
  for (int k = 0; k < runs.n; ++k) {
    const Run &r = runs.r[k];
    const bpc_params_t sub = run_params(params, r);
    const WsLayout sub_lay = ws_layout(&sub, r.elems);
    Source src{};
    src.grad = (const uint8_t *)grad + r.elem0 * gbytes;
    src.dtype = (int)dtype;
    src.residual = residual ? residual + r.elem0 : nullptr;
    Workspace w{(uint8_t *)ws, sub_lay, (uint32_t)k};
    const hipError_t e = encode(run_geo(sub, r), sub, nullptr, src, (uint8_t *)payload + r.pay_off, w, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_status(e);
  }
  return BPC_OK;
}

bpc_status_t bpc_compress_static_ws(const bpc_params_t *params, const void *grad, bpc_dtype_t dtype, float *residual,
                                    uint64_t D, void *payload, void *hip_stream) {
  if (!params_valid(params)) return BPC_ERR_INVALID_ARG;
  if (dtype != BPC_F32 && dtype != BPC_F16) return BPC_ERR_INVALID_ARG;
  if (D == 0) return BPC_OK;
  if (!grad || !payload) return BPC_ERR_INVALID_ARG;
  if (check_size(params, D) != BPC_OK) return BPC_ERR_UNSUPPORTED;
  if (!aligned16(grad) || !aligned16(residual) || !aligned16(payload) || !aligned16(params->norm_override))
    return BPC_ERR_ALIGNMENT;
  if (ws_layout(params, D).total > BPC_STATIC_WS_BYTES) return BPC_ERR_WORKSPACE;
  uint8_t *ws = nullptr;
  hipError_t e = static_workspace(&ws);
  if (e != hipSuccess) return hip_status(e);
  // from here on the call is bpc_compress on that workspace (whose kernels clear the parts of it
  // that must start from a known value: slots, status word, histograms)
  return bpc_compress(params, grad, dtype, residual, D, payload, ws, BPC_STATIC_WS_BYTES, hip_stream);
}

bpc_status_t bpc_decompress(const bpc_params_t *params, const void *payload, uint64_t D, float *out,
                            void *hip_stream) {
  if (!params_valid(params)) return BPC_ERR_INVALID_ARG;
  if (D == 0) return BPC_OK;
  if (!payload || !out) return BPC_ERR_INVALID_ARG;
  if (check_size(params, D) != BPC_OK) return BPC_ERR_UNSUPPORTED;
  if (!aligned16(payload) || !aligned16(out)) return BPC_ERR_ALIGNMENT;
  Runs runs;
  if (!make_runs(params, D, &runs)) return BPC_ERR_UNSUPPORTED;
  for (int k = 0; k < runs.n; ++k) {
    const Run &r = runs.r[k];
    const bpc_params_t sub = run_params(params, r);
    const hipError_t e = decode_dense(run_geo(sub, r), sub, (const uint8_t *)payload + r.pay_off, out + r.elem0,
                                      (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_status(e);
  }
  return BPC_OK;
}

bpc_status_t bpc_server_aggregate(const bpc_params_t *in, const void *const *payloads, int n,
                                  const bpc_params_t *out, float *server_residual, uint64_t D,
                                  void *out_payload, void *ws, size_t ws_bytes, void *hip_stream) {
  if (!params_valid(out) || !in || n < 1) return BPC_ERR_INVALID_ARG;
  if (n > kMaxWorkers) return BPC_ERR_UNSUPPORTED;
  for (int i = 0; i < n; ++i) {
    if (!params_valid(&in[i])) return BPC_ERR_INVALID_ARG;
    if (in[i].kind != out->kind || in[i].part_elems != out->part_elems) return BPC_ERR_INVALID_ARG;
    if ((out->kind == BPC_TOPK || out->kind == BPC_TOPK16 || out->kind == BPC_RANDK) && in[i].k_ratio != out->k_ratio)
      return BPC_ERR_INVALID_ARG;
    if ((out->kind == BPC_DITHER || out->kind == BPC_NATDITHER) && in[i].levels != out->levels) return BPC_ERR_INVALID_ARG;
  }
  if (D == 0) return BPC_OK;
  if (!payloads || !out_payload) return BPC_ERR_INVALID_ARG;
  for (int i = 0; i < n; ++i)
    if (!payloads[i]) return BPC_ERR_INVALID_ARG;
  if (check_size(out, D) != BPC_OK) return BPC_ERR_UNSUPPORTED;
  if (!aligned16(server_residual) || !aligned16(out_payload) || !aligned16(ws) || !aligned16(out->norm_override))
    return BPC_ERR_ALIGNMENT;
  for (int i = 0; i < n; ++i)
    if (!aligned16(payloads[i])) return BPC_ERR_ALIGNMENT;
  WsLayout lay = ws_layout(out, D);
  if (!ws || ws_bytes < lay.total) return BPC_ERR_WORKSPACE;
  Runs runs;
  if (!make_runs(out, D, &runs)) return BPC_ERR_UNSUPPORTED;
  if (!runs_fit(out, runs, ws_bytes)) return BPC_ERR_WORKSPACE;
  // the workers' messages have the layout of the outgoing one: the same partitions bypass
  const uint64_t P = cdiv(D, out->part_elems);
  for (int i = 0; i < n; ++i) {
    if ((in[i].bypass != nullptr) != (out->bypass != nullptr)) return BPC_ERR_INVALID_ARG;
    if (out->bypass && in[i].bypass != out->bypass)
      for (uint64_t p = 0; p < P; ++p)
        if ((in[i].bypass[p] != 0) != (out->bypass[p] != 0)) return BPC_ERR_INVALID_ARG;
  }
  for (int k = 0; k < runs.n; ++k) {
    const Run &r = runs.r[k];
    const bpc_params_t sub = run_params(out, r);
    bpc_params_t sub_in[kMaxWorkers];
    Source src{};
    src.grad = nullptr;
    src.residual = server_residual ? server_residual + r.elem0 : nullptr;
    src.msgs.n = n;
    src.msgs.inv_n = 1.0f / (float)n;
    for (int i = 0; i < n; ++i) {
      sub_in[i] = run_params(&in[i], r);
      src.msgs.ptr[i] = (const uint8_t *)payloads[i] + r.pay_off;
      src.msgs.seed[i] = in[i].seed;
      src.msgs.stream_id[i] = in[i].stream_id;
    }
    src.msgs.shared_scale = in[0].norm_override != nullptr;
    for (int i = 1; i < n; ++i) src.msgs.shared_scale = src.msgs.shared_scale && in[i].norm_override == in[0].norm_override;
    Workspace w{(uint8_t *)ws, ws_layout(&sub, r.elems), (uint32_t)k};
    const hipError_t e = encode(run_geo(sub, r), sub, sub_in, src, (uint8_t *)out_payload + r.pay_off, w, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_status(e);
  }
  return BPC_OK;
}

bpc_status_t bpc_adaptive_update(const bpc_params_t *params, const void *payload, uint64_t D, float *param,
                                 float *m, float *v, const bpc_opt_t *opt, void *ws, size_t ws_bytes,
                                 void *hip_stream) {
  if (!params_valid(params) || !opt) return BPC_ERR_INVALID_ARG;
  if (opt->kind != BPC_OPT_LANS && opt->kind != BPC_OPT_ADAM) return BPC_ERR_INVALID_ARG;
  if (!(opt->beta1 > 0.0f && opt->beta1 < 1.0f) || !(opt->beta2 > 0.0f && opt->beta2 < 1.0f) ||
      !(opt->eps > 0.0f) || !(opt->bias_corr1 > 0.0f) || !(opt->bias_corr2 > 0.0f) ||
      !(opt->phi_lo <= opt->phi_hi))
    return BPC_ERR_INVALID_ARG;
  if (opt->kind == BPC_OPT_LANS && opt->block_offsets && opt->n_blocks == 0) return BPC_ERR_INVALID_ARG;
  if (D == 0) return BPC_OK;
  if (!payload || !param || !m || !v) return BPC_ERR_INVALID_ARG;
  if (check_size(params, D) != BPC_OK) return BPC_ERR_UNSUPPORTED;
  if (!aligned16(payload) || !aligned16(param) || !aligned16(m) || !aligned16(v) || !aligned16(ws) ||
      !aligned16(opt->block_offsets))
    return BPC_ERR_ALIGNMENT;
  WsLayout lay = ws_layout(params, D);
  const size_t need = update_ws_bytes(lay, opt->kind == BPC_OPT_LANS && opt->block_offsets, opt->n_blocks, D);
  if (!ws || ws_bytes < need) return BPC_ERR_WORKSPACE;
  Runs runs;
  if (!make_runs(params, D, &runs)) return BPC_ERR_UNSUPPORTED;
  // (caller-defined LANS blocks may reach from one run into the next: not built)
  if (runs.n > 1 && opt->kind == BPC_OPT_LANS && opt->block_offsets) return BPC_ERR_UNSUPPORTED;
  if (!runs_fit(params, runs, ws_bytes)) return BPC_ERR_WORKSPACE;
  for (int k = 0; k < runs.n; ++k) {
    const Run &r = runs.r[k];
    const bpc_params_t sub = run_params(params, r);
    Workspace w{(uint8_t *)ws, ws_layout(&sub, r.elems), (uint32_t)k};
    const hipError_t e = adaptive_update(run_geo(sub, r), sub, (const uint8_t *)payload + r.pay_off, param + r.elem0, m + r.elem0,
                                         v + r.elem0, *opt, w, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_status(e);
  }
  return BPC_OK;
}

bpc_status_t bpc_stream_probe(bpc_probe_t mix, const void *a, const void *b, void *c, uint64_t n, void *hip_stream) {
  if (mix != BPC_PROBE_COPY && mix != BPC_PROBE_WORKER_MIX && mix != BPC_PROBE_UPDATE_MIX) return BPC_ERR_INVALID_ARG;
  if (n == 0) return BPC_OK;
  if (!a || !c || (mix != BPC_PROBE_COPY && !b)) return BPC_ERR_INVALID_ARG;
  if (n / kTile >= 0x7fffffffull) return BPC_ERR_UNSUPPORTED;
  if (!aligned16(a) || !aligned16(b) || !aligned16(c)) return BPC_ERR_ALIGNMENT;
  return hip_status(stream_probe((int)mix, a, b, c, n, (hipStream_t)hip_stream));
}

const char *bpc_status_string(bpc_status_t status) {
  switch (status) {
    case BPC_OK: return "ok";
    case BPC_ERR_INVALID_ARG: return "invalid argument";
    case BPC_ERR_UNSUPPORTED: return "unsupported configuration";
    case BPC_ERR_WORKSPACE: return "workspace missing or too small";
    case BPC_ERR_ALIGNMENT: return "device pointer not 16-byte aligned";
    case BPC_ERR_HIP: return "HIP call failed";
    case BPC_ERR_WAIT: return "a device-side wait gave up: outputs of the call are undefined";
    default: return "unknown status";
  }
}

int bpc_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
