/*
 * CPU oracle -- see bpc_oracle.h.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain C, scalar loops, one obvious statement per step of the paper.  No
 * blocking, no fusion: the residual really is "q minus the decoded message"
 * (Algorithm 4), even where a shortcut exists (Section 4.2, operator fusion).
 */
#include "bpc_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Philox4x32-10, Salmon, Moraes, Dror, Shaw (SC'11).                  */
/* ------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Random word number t of partition `part_no` in the stream (seed, stream_id). */
static uint32_t draw_word(const orc_params *p, uint64_t part_no, uint64_t t) {
  uint32_t ctr[4], key[2], out[4];
  ctr[0] = (uint32_t)(t / 4);
  ctr[1] = (uint32_t)part_no;
  ctr[2] = (uint32_t)(p->stream_id & 0xffffffffu);
  ctr[3] = (uint32_t)(p->stream_id >> 32);
  key[0] = (uint32_t)(p->seed & 0xffffffffu);
  key[1] = (uint32_t)(p->seed >> 32);
  orc_philox4x32_10(ctr, key, out);
  return out[t % 4];
}

/* IEEE binary16 -> binary32, exact (every half value is a float value). */
float orc_half_to_float(uint16_t h) {
  uint32_t sign = (uint32_t)(h >> 15) & 1u;
  uint32_t expo = (uint32_t)(h >> 10) & 0x1fu;
  uint32_t frac = (uint32_t)h & 0x3ffu;
  float mag;
  if (expo == 0) {
    mag = ldexpf((float)frac, -24);               /* zero and subnormals */
  } else if (expo == 31) {
    mag = frac ? NAN : INFINITY;
  } else {
    mag = ldexpf((float)(frac | 0x400u), (int)expo - 25);
  }
  return sign ? -mag : mag;
}

static uint32_t float_bits(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }

/* IEEE binary32 -> binary16, round to nearest, ties to even; magnitudes that round past the
 * largest half (65504) become infinity, NaN stays NaN.  Done on the exact value: the float is
 * m * 2^e with an integer m < 2^24, a half is an integer multiple of 2^max(e_h - 10, -24). */
uint16_t orc_float_to_half(float x) {
  uint32_t u = float_bits(x);
  uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  uint32_t expo = (u >> 23) & 0xffu, frac = u & 0x7fffffu;
  if (expo == 255) return (uint16_t)(sign | 0x7c00u | (frac ? 0x200u : 0u));
  if (expo == 0) return sign;                       /* float zero/subnormal: below half the smallest half */
  int e = (int)expo - 127;                          /* |x| = (1.frac) * 2^e */
  uint64_t m = (uint64_t)(frac | 0x800000u);        /* |x| = m * 2^(e-23) */
  /* spacing of the halves around |x|: 2^(e-10) for normal halves (e >= -14), else 2^-24 */
  int unit = e >= -14 ? e - 10 : -24;
  int shift = unit - (e - 23);                      /* |x| / 2^unit = m / 2^shift, shift >= 13 */
  uint64_t q, rem, half_way;
  if (shift >= 40) { q = 0; rem = 1; half_way = 2; }   /* far below half a unit */
  else {
    q = m >> shift;
    rem = m & (((uint64_t)1 << shift) - 1);
    half_way = (uint64_t)1 << (shift - 1);
  }
  if (rem > half_way || (rem == half_way && (q & 1u))) ++q;
  /* q units of 2^unit: q < 2048 at entry; a carry to 2048 moves to the next exponent by itself
   * because the half encoding is monotone in (exponent, fraction) */
  uint32_t bits;
  if (e >= -14) bits = ((uint32_t)(e + 15) << 10) + (uint32_t)(q - 1024);   /* q in [1024, 2048] */
  else bits = (uint32_t)q;                                                    /* subnormal, or 1024 = smallest normal */
  if (bits >= 0x7c00u) bits = 0x7c00u;              /* past 65504: infinity */
  return (uint16_t)(sign | bits);
}

/* ------------------------------------------------------------------ */
/* Sizes                                                               */
/* ------------------------------------------------------------------ */
static uint64_t ru4(uint64_t x) { return (x + 3) / 4 * 4; }

static int params_ok(const orc_params *p) {
  if (!p) return 0;
  if (p->part_elems == 0 || p->part_elems % 1024 != 0) return 0;
  switch (p->kind) {
    case ORC_IDENTITY: case ORC_SIGN: case ORC_FP16: return 1;
    case ORC_TOPK: case ORC_TOPK16: case ORC_RANDK: return p->k_ratio > 0.0 && p->k_ratio <= 1.0;
    case ORC_DITHER:
      return p->levels >= 1 && p->levels <= 63 && (p->norm == ORC_NORM_L2 || p->norm == ORC_NORM_LINF);
    case ORC_NATDITHER:
      return p->levels >= 1 && p->levels <= 7 && (p->norm == ORC_NORM_L2 || p->norm == ORC_NORM_LINF);
    default: return 0;
  }
}

/* Linear dithering with more than 7 levels (the 5- and 7-bit forms of Section 5's list): the
 * level bits above the third go into bit planes after the nibbles, one bit per element and
 * plane, so a message costs 4 + planes bits per element.  s <= 7: 0, <= 15: 1, <= 31: 2,
 * <= 63: 3 planes. */
static unsigned dither_planes(unsigned levels) {
  unsigned planes = 0;
  while ((levels >> (3 + planes)) != 0) ++planes;
  return planes;
}

/* k = max(1, floor(ratio*d)), never above d. */
uint64_t orc_partition_k(const orc_params *p, uint64_t d) {
  if (!params_ok(p) || d == 0) return 0;
  if (p->kind != ORC_TOPK && p->kind != ORC_TOPK16 && p->kind != ORC_RANDK) return 0;
  uint64_t k = (uint64_t)floor(p->k_ratio * (double)d);
  if (k < 1) k = 1;
  if (k > d) k = d;
  return k;
}

size_t orc_partition_stride(const orc_params *p) {
  if (!params_ok(p)) return 0;
  uint64_t d = p->part_elems, words = 0;
  switch (p->kind) {
    case ORC_IDENTITY: words = ru4(d); break;
    case ORC_SIGN:     words = ru4((d + 31) / 32); break;
    case ORC_DITHER:   words = ru4((d + 7) / 8) + dither_planes(p->levels) * ru4((d + 31) / 32); break;
    case ORC_NATDITHER: words = ru4((d + 7) / 8); break;
    case ORC_TOPK:     words = 2 * ru4(orc_partition_k(p, d)); break;
    case ORC_TOPK16:   words = ru4(orc_partition_k(p, d)) + ru4((orc_partition_k(p, d) + 1) / 2); break;
    case ORC_RANDK:    words = ru4(orc_partition_k(p, d)); break;
    case ORC_FP16:     words = ru4((d + 1) / 2); break;
  }
  return (size_t)(16 + 4 * words);
}

static uint64_t n_partitions(const orc_params *p, uint64_t D) {
  return (D + p->part_elems - 1) / p->part_elems;
}

size_t orc_payload_bytes(const orc_params *p, uint64_t D) {
  if (!params_ok(p)) return 0;
  return (size_t)n_partitions(p, D) * orc_partition_stride(p);
}

/* ------------------------------------------------------------------ */
/* Encoders: q (d floats) -> one partition record                      */
/* ------------------------------------------------------------------ */
static void put_u32(unsigned char *rec, uint64_t word, uint32_t x) { memcpy(rec + 4 * word, &x, 4); }
static uint32_t get_u32(const unsigned char *rec, uint64_t word) { uint32_t x; memcpy(&x, rec + 4 * word, 4); return x; }
static void put_f32(unsigned char *rec, uint64_t word, float x) { memcpy(rec + 4 * word, &x, 4); }
static float get_f32(const unsigned char *rec, uint64_t word) { float x; memcpy(&x, rec + 4 * word, 4); return x; }

/* Scaled sign (Definition 2 example): sigma = ||q||_1 / d, one bit per element. */
static void encode_sign(const float *q, uint64_t d, const float *sigma_given, unsigned char *rec) {
  float sigma;
  if (sigma_given) {
    sigma = *sigma_given;
  } else {
    double l1 = 0.0;
    for (uint64_t j = 0; j < d; ++j) l1 += (double)fabsf(q[j]);
    sigma = (float)(l1 / (double)d);
  }
  uint64_t words = ru4((d + 31) / 32);
  put_f32(rec, 0, sigma);
  put_u32(rec, 1, 0); put_u32(rec, 2, 0); put_u32(rec, 3, 0);
  for (uint64_t w = 0; w < words; ++w) put_u32(rec, 4 + w, 0);
  for (uint64_t j = 0; j < d; ++j) {
    if (q[j] < 0.0f) {
      uint32_t w = get_u32(rec, 4 + j / 32);
      w |= (uint32_t)1 << (j % 32);
      put_u32(rec, 4 + j / 32, w);
    }
  }
}

static void decode_sign(const unsigned char *rec, uint64_t d, float *out) {
  float sigma = get_f32(rec, 0);
  for (uint64_t j = 0; j < d; ++j) {
    uint32_t bit = (get_u32(rec, 4 + j / 32) >> (j % 32)) & 1u;
    out[j] = bit ? -sigma : sigma;
  }
}

/* Top-k: order by (magnitude key descending, index ascending), keep the first k,
 * write them in ascending index order. */
typedef struct { uint32_t key; uint32_t idx; } key_idx;

static int by_key_desc_idx_asc(const void *a, const void *b) {
  const key_idx *x = (const key_idx *)a, *y = (const key_idx *)b;
  if (x->key != y->key) return x->key > y->key ? -1 : 1;
  if (x->idx != y->idx) return x->idx < y->idx ? -1 : 1;
  return 0;
}
static int by_idx_asc(const void *a, const void *b) {
  const key_idx *x = (const key_idx *)a, *y = (const key_idx *)b;
  return (x->idx > y->idx) - (x->idx < y->idx);
}

static void encode_topk(const orc_params *p, const float *q, uint64_t d, unsigned char *rec) {
  uint64_t k = orc_partition_k(p, d);
  uint64_t kcap4 = ru4(orc_partition_k(p, p->part_elems));
  key_idx *all = (key_idx *)malloc(sizeof(key_idx) * (size_t)d);
  for (uint64_t j = 0; j < d; ++j) {
    all[j].key = float_bits(q[j]) & 0x7fffffffu;
    all[j].idx = (uint32_t)j;
  }
  qsort(all, (size_t)d, sizeof(key_idx), by_key_desc_idx_asc);
  qsort(all, (size_t)k, sizeof(key_idx), by_idx_asc);
  put_u32(rec, 0, (uint32_t)k);
  put_u32(rec, 1, 0); put_u32(rec, 2, 0); put_u32(rec, 3, 0);
  if (p->kind == ORC_TOPK16) {
    /* the message format behind the compression rate quoted in Section 5.2: a 32-bit index
     * and a half-precision value per kept element */
    for (uint64_t w = 0; w < ru4((k + 1) / 2); ++w) put_u32(rec, 4 + kcap4 + w, 0);
    for (uint64_t t = 0; t < k; ++t) {
      put_u32(rec, 4 + t, all[t].idx);
      uint32_t w = get_u32(rec, 4 + kcap4 + t / 2);
      w |= (uint32_t)orc_float_to_half(q[all[t].idx]) << (16 * (t % 2));
      put_u32(rec, 4 + kcap4 + t / 2, w);
    }
    free(all);
    return;
  }
  for (uint64_t t = 0; t < k; ++t) {
    put_u32(rec, 4 + t, all[t].idx);
    put_f32(rec, 4 + kcap4 + t, q[all[t].idx]);
  }
  free(all);
}

static void decode_topk(const orc_params *p, const unsigned char *rec, uint64_t d, float *out) {
  uint64_t k = get_u32(rec, 0);
  uint64_t kcap4 = ru4(orc_partition_k(p, p->part_elems));
  for (uint64_t j = 0; j < d; ++j) out[j] = 0.0f;
  for (uint64_t t = 0; t < k; ++t) {
    uint32_t idx = get_u32(rec, 4 + t);
    if (idx >= d) continue;
    if (p->kind == ORC_TOPK16)
      out[idx] = orc_half_to_float((uint16_t)(get_u32(rec, 4 + kcap4 + t / 2) >> (16 * (t % 2))));
    else
      out[idx] = get_f32(rec, 4 + kcap4 + t);
  }
}

/* Random-k: k indices uniform on [0,d) with replacement, idx = (word*d) >> 32. */
static uint64_t randk_index(const orc_params *p, uint64_t part_no, uint64_t t, uint64_t d) {
  uint64_t r = draw_word(p, part_no, t);
  return (r * d) >> 32;
}

static float randk_scale(const orc_params *p, uint64_t d, uint64_t k) {
  if (p->value_scale >= 0.0f) return p->value_scale;
  return (float)d / (float)k;
}

static void encode_randk(const orc_params *p, uint64_t part_no, const float *q, uint64_t d,
                         unsigned char *rec) {
  uint64_t k = orc_partition_k(p, d);
  put_u32(rec, 0, (uint32_t)k);
  put_u32(rec, 1, 0); put_u32(rec, 2, 0); put_u32(rec, 3, 0);
  for (uint64_t t = 0; t < k; ++t) put_f32(rec, 4 + t, q[randk_index(p, part_no, t, d)]);
}

static void decode_randk(const orc_params *p, uint64_t part_no, const unsigned char *rec, uint64_t d,
                         float *out) {
  uint64_t k = get_u32(rec, 0);
  float scale = randk_scale(p, d, k);
  for (uint64_t j = 0; j < d; ++j) out[j] = 0.0f;
  for (uint64_t t = 0; t < k; ++t) {
    uint64_t idx = randk_index(p, part_no, t, d);
    out[idx] = out[idx] + scale * get_f32(rec, 4 + t);
  }
}

/* Linear dithering in the form of the quantiser the paper cites for it (QSGD):
 * with a = s|q_j|/nu, the level is floor(a) + 1 with probability a - floor(a),
 * else floor(a); the message holds the sign and the level, the norm nu once. */
static void encode_dither(const orc_params *p, uint64_t part_no, const float *q, uint64_t d,
                          const float *nu_given, unsigned char *rec) {
  float nu;
  if (nu_given) {
    nu = *nu_given;
  } else if (p->norm == ORC_NORM_L2) {
    double ss = 0.0;
    for (uint64_t j = 0; j < d; ++j) ss += (double)q[j] * (double)q[j];
    nu = (float)sqrt(ss);
  } else {
    nu = 0.0f;
    for (uint64_t j = 0; j < d; ++j) if (fabsf(q[j]) > nu) nu = fabsf(q[j]);
  }
  uint64_t words = ru4((d + 7) / 8);
  /* plane t starts after the nibbles of a full partition, whatever d is */
  unsigned planes = dither_planes(p->levels);
  uint64_t plane0 = 4 + ru4((p->part_elems + 7) / 8), plane_words = ru4((p->part_elems + 31) / 32);
  put_f32(rec, 0, nu);
  put_u32(rec, 1, 0); put_u32(rec, 2, 0); put_u32(rec, 3, 0);
  for (uint64_t w = 0; w < words; ++w) put_u32(rec, 4 + w, 0);
  for (unsigned t = 0; t < planes; ++t)
    for (uint64_t w = 0; w < ru4((d + 31) / 32); ++w) put_u32(rec, plane0 + t * plane_words + w, 0);
  if (!(nu > 0.0f)) return;
  unsigned s = p->levels;
  /* a = s|q_j|/nu is evaluated as |q_j| * (s/nu), the quotient formed once per partition;
   * if s/nu overflows (nu below about 1e-38) the division is done per element instead. */
  float s_over_nu = (float)s / nu;
  for (uint64_t j = 0; j < d; ++j) {
    float a = isfinite(s_over_nu) ? fabsf(q[j]) * s_over_nu : (fabsf(q[j]) * (float)s) / nu;
    float l = floorf(a);
    float f = a - l;
    float u = (float)(draw_word(p, part_no, j) >> 8) * 0x1p-24f;
    unsigned level = (unsigned)l + (u < f ? 1u : 0u);
    if (level > s) level = s;
    uint32_t nibble = (q[j] < 0.0f ? 8u : 0u) | (level & 7u);
    uint32_t w = get_u32(rec, 4 + j / 8);
    w |= nibble << (4 * (j % 8));
    put_u32(rec, 4 + j / 8, w);
    for (unsigned t = 0; t < planes; ++t) {
      uint64_t at = plane0 + t * plane_words + j / 32;
      put_u32(rec, at, get_u32(rec, at) | (((level >> (3 + t)) & 1u) << (j % 32)));
    }
  }
}

static void decode_dither(const orc_params *p, const unsigned char *rec, uint64_t d, float *out) {
  float nu = get_f32(rec, 0);
  float s = (float)p->levels;
  unsigned planes = dither_planes(p->levels);
  uint64_t plane0 = 4 + ru4((p->part_elems + 7) / 8), plane_words = ru4((p->part_elems + 31) / 32);
  for (uint64_t j = 0; j < d; ++j) {
    uint32_t nibble = (get_u32(rec, 4 + j / 8) >> (4 * (j % 8))) & 0xfu;
    uint32_t level = nibble & 7u;
    for (unsigned t = 0; t < planes; ++t)
      level |= ((get_u32(rec, plane0 + t * plane_words + j / 32) >> (j % 32)) & 1u) << (3 + t);
    float mag = (nu * (float)level) / s;
    out[j] = (nibble & 8u) ? -mag : mag;
  }
}

/* Natural dithering, the power-of-two sibling of the quantiser above that the paper lists
 * among its compressors (Section 5, "natural dithering"): the levels l = 1..s stand for the
 * magnitudes nu * 2^(l-s), level 0 for zero, and |q_j| is rounded to one of its two
 * neighbouring levels at random so that the expectation is |q_j|.
 * With y = |q_j| * 2^(s-1) / nu (levels sit at y = 0, 1, 2, 4, ..., 2^(s-1)):
 *   y < 1        : lower level 0, upper level 1, P(up) = y
 *   2^e <= y     : lower level e+1, P(up) = y / 2^e - 1 (the fraction bits of y, exact)
 * Same record as linear dithering: norm, then one nibble (sign, level) per element. */
static void encode_natdither(const orc_params *p, uint64_t part_no, const float *q, uint64_t d,
                             const float *nu_given, unsigned char *rec) {
  float nu;
  if (nu_given) {
    nu = *nu_given;
  } else if (p->norm == ORC_NORM_L2) {
    double ss = 0.0;
    for (uint64_t j = 0; j < d; ++j) ss += (double)q[j] * (double)q[j];
    nu = (float)sqrt(ss);
  } else {
    nu = 0.0f;
    for (uint64_t j = 0; j < d; ++j) if (fabsf(q[j]) > nu) nu = fabsf(q[j]);
  }
  uint64_t words = ru4((d + 7) / 8);
  put_f32(rec, 0, nu);
  put_u32(rec, 1, 0); put_u32(rec, 2, 0); put_u32(rec, 3, 0);
  for (uint64_t w = 0; w < words; ++w) put_u32(rec, 4 + w, 0);
  if (!(nu > 0.0f)) return;
  unsigned s = p->levels;
  float top = (float)(1u << (s - 1));        /* y of the highest level */
  /* the quotient is formed once per partition; per element only if it overflows */
  float top_over_nu = top / nu;
  for (uint64_t j = 0; j < d; ++j) {
    float y = isfinite(top_over_nu) ? fabsf(q[j]) * top_over_nu : (fabsf(q[j]) * top) / nu;
    unsigned lower;
    float up;
    if (y < 1.0f) {
      lower = 0;
      up = y;
    } else {
      uint32_t bits = float_bits(y);
      lower = (unsigned)(bits >> 23) - 127u + 1u;          /* floor(log2 y) + 1 */
      uint32_t frac = (bits & 0x007fffffu) | 0x3f800000u;  /* y / 2^floor(log2 y), in [1, 2) */
      float m; memcpy(&m, &frac, 4);
      up = m - 1.0f;
    }
    float u = (float)(draw_word(p, part_no, j) >> 8) * 0x1p-24f;
    unsigned level = lower + (u < up ? 1u : 0u);
    if (level > s) level = s;
    uint32_t nibble = (q[j] < 0.0f ? 8u : 0u) | level;
    uint32_t w = get_u32(rec, 4 + j / 8);
    w |= nibble << (4 * (j % 8));
    put_u32(rec, 4 + j / 8, w);
  }
}

static void decode_natdither(const orc_params *p, const unsigned char *rec, uint64_t d, float *out) {
  float nu = get_f32(rec, 0);
  float top = (float)(1u << (p->levels - 1));
  for (uint64_t j = 0; j < d; ++j) {
    uint32_t nibble = (get_u32(rec, 4 + j / 8) >> (4 * (j % 8))) & 0xfu;
    unsigned level = nibble & 7u;
    float mag = level == 0 ? 0.0f : (nu * (float)(1u << (level - 1))) / top;
    out[j] = (nibble & 8u) ? -mag : mag;
  }
}

static void encode_identity(const float *q, uint64_t d, unsigned char *rec) {
  put_u32(rec, 0, 0); put_u32(rec, 1, 0); put_u32(rec, 2, 0); put_u32(rec, 3, 0);
  for (uint64_t j = 0; j < d; ++j) put_f32(rec, 4 + j, q[j]);
}
static void decode_identity(const unsigned char *rec, uint64_t d, float *out) {
  for (uint64_t j = 0; j < d; ++j) out[j] = get_f32(rec, 4 + j);
}

/* The data type conversion the paper uses where anything heavier would not pay (Section 4.1:
 * FP32 to FP16 inside a node; Section 5.1 lists the half-precision baseline): every element is
 * rounded to the nearest half, ties to even. */
static void encode_fp16(const float *q, uint64_t d, unsigned char *rec) {
  put_u32(rec, 0, 0); put_u32(rec, 1, 0); put_u32(rec, 2, 0); put_u32(rec, 3, 0);
  uint64_t words = ru4((d + 1) / 2);
  for (uint64_t w = 0; w < words; ++w) put_u32(rec, 4 + w, 0);
  for (uint64_t j = 0; j < d; ++j) {
    uint32_t w = get_u32(rec, 4 + j / 2);
    w |= (uint32_t)orc_float_to_half(q[j]) << (16 * (j % 2));
    put_u32(rec, 4 + j / 2, w);
  }
}
static void decode_fp16(const unsigned char *rec, uint64_t d, float *out) {
  for (uint64_t j = 0; j < d; ++j)
    out[j] = orc_half_to_float((uint16_t)(get_u32(rec, 4 + j / 2) >> (16 * (j % 2))));
}

void orc_encode_partition(const orc_params *p, uint64_t part_no, const float *norm_override1,
                          const float *q, uint64_t d, unsigned char *rec) {
  switch (p->kind) {
    case ORC_IDENTITY: encode_identity(q, d, rec); break;
    case ORC_SIGN:     encode_sign(q, d, norm_override1, rec); break;
    case ORC_TOPK: case ORC_TOPK16: encode_topk(p, q, d, rec); break;
    case ORC_RANDK:    encode_randk(p, part_no, q, d, rec); break;
    case ORC_DITHER:   encode_dither(p, part_no, q, d, norm_override1, rec); break;
    case ORC_NATDITHER: encode_natdither(p, part_no, q, d, norm_override1, rec); break;
    case ORC_FP16:     encode_fp16(q, d, rec); break;
  }
}

void orc_decode_partition(const orc_params *p, uint64_t part_no, const unsigned char *rec,
                          uint64_t d, float *out) {
  switch (p->kind) {
    case ORC_IDENTITY: decode_identity(rec, d, out); break;
    case ORC_SIGN:     decode_sign(rec, d, out); break;
    case ORC_TOPK: case ORC_TOPK16: decode_topk(p, rec, d, out); break;
    case ORC_RANDK:    decode_randk(p, part_no, rec, d, out); break;
    case ORC_DITHER:   decode_dither(p, rec, d, out); break;
    case ORC_NATDITHER: decode_natdither(p, rec, d, out); break;
    case ORC_FP16:     decode_fp16(rec, d, out); break;
  }
}

/* ------------------------------------------------------------------ */
/* Algorithm 4 / 3, worker                                             */
/* ------------------------------------------------------------------ */
int orc_compress(const orc_params *p, const void *grad, int dtype, float *residual, uint64_t D,
                 unsigned char *payload) {
  if (!params_ok(p) || (D && (!grad || !payload))) return 1;
  if (dtype != ORC_F32 && dtype != ORC_F16) return 1;
  size_t stride = orc_partition_stride(p);
  uint64_t P = n_partitions(p, D);
  float *q = (float *)malloc(sizeof(float) * (size_t)p->part_elems);
  float *dec = (float *)malloc(sizeof(float) * (size_t)p->part_elems);
  for (uint64_t pi = 0; pi < P; ++pi) {
    uint64_t base = pi * p->part_elems;
    uint64_t d = D - base < p->part_elems ? D - base : p->part_elems;
    uint64_t part_no = p->first_partition + pi;
    unsigned char *rec = payload + pi * stride;
    /* q = g + e */
    for (uint64_t j = 0; j < d; ++j) {
      float g = dtype == ORC_F32 ? ((const float *)grad)[base + j]
                                 : orc_half_to_float(((const uint16_t *)grad)[base + j]);
      q[j] = residual ? g + residual[base + j] : g;
    }
    /* delta = C(q) */
    orc_encode_partition(p, part_no, p->norm_override ? p->norm_override + pi : NULL, q, d, rec);
    /* e' = q - delta */
    if (residual) {
      orc_decode_partition(p, part_no, rec, d, dec);
      for (uint64_t j = 0; j < d; ++j) residual[base + j] = q[j] - dec[j];
    }
  }
  free(q); free(dec);
  return 0;
}

int orc_decompress(const orc_params *p, const unsigned char *payload, uint64_t D, float *out) {
  if (!params_ok(p) || (D && (!payload || !out))) return 1;
  size_t stride = orc_partition_stride(p);
  uint64_t P = n_partitions(p, D);
  for (uint64_t pi = 0; pi < P; ++pi) {
    uint64_t base = pi * p->part_elems;
    uint64_t d = D - base < p->part_elems ? D - base : p->part_elems;
    orc_decode_partition(p, p->first_partition + pi, payload + pi * stride, d, out + base);
  }
  return 0;
}

/* ------------------------------------------------------------------ */
/* Algorithm 4 / 3, server                                             */
/* ------------------------------------------------------------------ */
int orc_server_aggregate(const orc_params *in, const unsigned char *const *payloads, int n,
                         const orc_params *out, float *server_residual, uint64_t D,
                         unsigned char *out_payload) {
  if (n < 1 || !in || !params_ok(out) || (D && (!payloads || !out_payload))) return 1;
  for (int i = 0; i < n; ++i)
    if (!params_ok(&in[i]) || in[i].kind != out->kind || in[i].part_elems != out->part_elems) return 1;
  size_t stride_in = orc_partition_stride(&in[0]);
  size_t stride_out = orc_partition_stride(out);
  uint64_t P = n_partitions(out, D);
  float inv_n = 1.0f / (float)n;
  float *acc = (float *)malloc(sizeof(float) * (size_t)out->part_elems);
  float *dec = (float *)malloc(sizeof(float) * (size_t)out->part_elems);
  float *delta = (float *)malloc(sizeof(float) * (size_t)out->part_elems);
  for (uint64_t pi = 0; pi < P; ++pi) {
    uint64_t base = pi * out->part_elems;
    uint64_t d = D - base < out->part_elems ? D - base : out->part_elems;
    /* sum of the n decoded worker messages, in worker order */
    for (uint64_t j = 0; j < d; ++j) acc[j] = 0.0f;
    for (int i = 0; i < n; ++i) {
      orc_decode_partition(&in[i], in[i].first_partition + pi, payloads[i] + pi * stride_in, d, dec);
      for (uint64_t j = 0; j < d; ++j) acc[j] = acc[j] + dec[j];
    }
    /* Delta = (1/n) sum + e~ */
    for (uint64_t j = 0; j < d; ++j) {
      float mean = acc[j] * inv_n;
      delta[j] = server_residual ? mean + server_residual[base + j] : mean;
    }
    /* p = C(Delta);  e~' = Delta - p */
    uint64_t part_no = out->first_partition + pi;
    unsigned char *rec = out_payload + pi * stride_out;
    orc_encode_partition(out, part_no, out->norm_override ? out->norm_override + pi : NULL, delta, d, rec);
    if (server_residual) {
      orc_decode_partition(out, part_no, rec, d, dec);
      for (uint64_t j = 0; j < d; ++j) server_residual[base + j] = delta[j] - dec[j];
    }
  }
  free(acc); free(dec); free(delta);
  return 0;
}

/* ------------------------------------------------------------------ */
/* Algorithm 5, update lines                                           */
/* ------------------------------------------------------------------ */
static float l2_norm(const float *x, uint64_t n) {
  double ss = 0.0;
  for (uint64_t j = 0; j < n; ++j) ss += (double)x[j] * (double)x[j];
  return (float)sqrt(ss);
}

static void update_block(const orc_opt *o, const float *g, float *x, float *m, float *v, uint64_t n) {
  float one_minus_b1 = 1.0f - o->beta1;
  float one_minus_b2 = 1.0f - o->beta2;
  float *u_r = (float *)malloc(sizeof(float) * (size_t)(n ? n : 1)); /* r + lambda x */
  float *u_c = (float *)malloc(sizeof(float) * (size_t)(n ? n : 1)); /* c + lambda x */
  for (uint64_t j = 0; j < n; ++j) {
    m[j] = o->beta1 * m[j] + one_minus_b1 * g[j];
    v[j] = o->beta2 * v[j] + one_minus_b2 * (g[j] * g[j]);
    float m_hat = m[j] / o->bias_corr1;
    float v_hat = v[j] / o->bias_corr2;
    float denom = sqrtf(v_hat) + o->eps;
    float r = m_hat / denom;
    float c = g[j] / denom;
    float decay = o->weight_decay * x[j];
    u_r[j] = r + decay;
    u_c[j] = c + decay;
  }
  if (o->kind == ORC_OPT_ADAM) {
    for (uint64_t j = 0; j < n; ++j) x[j] = x[j] - o->lr * u_r[j];
  } else {
    float norm_x = l2_norm(x, n);
    float norm_r = l2_norm(u_r, n);
    float norm_c = l2_norm(u_c, n);
    float phi = norm_x;
    if (phi < o->phi_lo) phi = o->phi_lo;
    if (phi > o->phi_hi) phi = o->phi_hi;
    float w_r = norm_r > 0.0f ? o->beta1 / norm_r : 0.0f;
    float w_c = norm_c > 0.0f ? one_minus_b1 / norm_c : 0.0f;
    for (uint64_t j = 0; j < n; ++j) {
      float dir = phi * (w_r * u_r[j] + w_c * u_c[j]);
      x[j] = x[j] - o->lr * dir;
    }
  }
  free(u_r); free(u_c);
}

int orc_adaptive_update(const orc_params *p, const unsigned char *payload, uint64_t D,
                        float *param, float *m, float *v, const orc_opt *opt) {
  if (!params_ok(p) || !opt || (D && (!payload || !param || !m || !v))) return 1;
  float *g = (float *)malloc(sizeof(float) * (size_t)(D ? D : 1));
  orc_decompress(p, payload, D, g);
  if (opt->block_offsets) {
    for (uint64_t b = 0; b < opt->n_blocks; ++b) {
      uint64_t lo = opt->block_offsets[b], hi = opt->block_offsets[b + 1];
      update_block(opt, g + lo, param + lo, m + lo, v + lo, hi - lo);
    }
  } else {
    for (uint64_t lo = 0; lo < D; lo += p->part_elems) {
      uint64_t n = D - lo < p->part_elems ? D - lo : p->part_elems;
      update_block(opt, g + lo, param + lo, m + lo, v + lo, n);
    }
  }
  free(g);
  return 0;
}
