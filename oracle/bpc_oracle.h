/*
 * CPU oracle for the two-way error-feedback gradient-compression path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition the GPU library
 * is checked against; nothing in the product path may call it.  It shares no
 * code with the HIP library (own structs, own Philox, own message writer).
 *
 * Follows the paper step by step: Algorithm 4 (two-way compression with error
 * feedback), Algorithm 3 (without), the compressors of Section 3.2 /
 * Definitions 1-2, and the update lines of Algorithm 5.  Element-wise
 * arithmetic is IEEE binary32 in the order written, because the state the
 * method carries (residuals, moments, parameters) is binary32 and the packed
 * bits are decided from those values; every reduction (L1/L2 norms) is
 * accumulated in binary64 in index order and rounded once.  Build with
 * -ffp-contract=off.
 *
 * Parity pins (tests/test_oracle_*.py): sign closed form, top-k brute force,
 * random-k / dithering unbiasedness, error-feedback identity, identity
 * compressor == plain mean, textbook Adam, LANS norm bound, Philox known
 * answers.  No function here is parity-unpinned.
 */
#ifndef BPC_ORACLE_H_
#define BPC_ORACLE_H_

#include <stddef.h>
#include <stdint.h>

enum { ORC_IDENTITY = 0, ORC_SIGN = 1, ORC_TOPK = 2, ORC_RANDK = 3, ORC_DITHER = 4, ORC_NATDITHER = 5,
       ORC_FP16 = 6, ORC_TOPK16 = 7 };
enum { ORC_F32 = 0, ORC_F16 = 1 };
enum { ORC_NORM_L2 = 0, ORC_NORM_LINF = 1 };
enum { ORC_OPT_LANS = 0, ORC_OPT_ADAM = 1 };

typedef struct {
  int kind;
  int norm;
  uint64_t part_elems;
  double k_ratio;
  unsigned levels;
  float value_scale;       /* < 0: d/k */
  uint64_t seed;
  uint64_t stream_id;
  uint64_t first_partition; /* partition number of the first partition of this call */
  const float *norm_override; /* host, one per partition of this call, or NULL */
} orc_params;

typedef struct {
  int kind;
  float lr, beta1, beta2, eps, weight_decay, bias_corr1, bias_corr2, phi_lo, phi_hi;
  const uint64_t *block_offsets; /* host, n_blocks+1 entries, or NULL: one block per partition */
  uint64_t n_blocks;
} orc_opt;

void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
float orc_half_to_float(uint16_t h);
uint16_t orc_float_to_half(float x);

uint64_t orc_partition_k(const orc_params *p, uint64_t d);
size_t orc_partition_stride(const orc_params *p);
size_t orc_payload_bytes(const orc_params *p, uint64_t D);

/* Single-partition encoder / decoder, exposed so tests can pin them directly. */
void orc_encode_partition(const orc_params *p, uint64_t part_no, const float *norm_override1,
                          const float *q, uint64_t d, unsigned char *rec);
void orc_decode_partition(const orc_params *p, uint64_t part_no, const unsigned char *rec,
                          uint64_t d, float *out);

/* Algorithm 4 worker lines (residual != NULL) / Algorithm 3 worker line (NULL). */
int orc_compress(const orc_params *p, const void *grad, int dtype, float *residual, uint64_t D,
                 unsigned char *payload);
int orc_decompress(const orc_params *p, const unsigned char *payload, uint64_t D, float *out);
/* Algorithm 4 server lines (server_residual != NULL) / Algorithm 3 (NULL). */
int orc_server_aggregate(const orc_params *in, const unsigned char *const *payloads, int n,
                         const orc_params *out, float *server_residual, uint64_t D,
                         unsigned char *out_payload);
/* Algorithm 5 update lines on the decoded message. */
int orc_adaptive_update(const orc_params *p, const unsigned char *payload, uint64_t D,
                        float *param, float *m, float *v, const orc_opt *opt);

#endif
