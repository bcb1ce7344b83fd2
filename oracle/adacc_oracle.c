/*
 * CPU oracle for outlier-separated activation compression (Adacc, arXiv 2508.00806).
 * TEST INFRASTRUCTURE ONLY - see adacc_oracle.h.
 *
 * What is computed, in the order Section 3.2 and Fig. 3(c) give it:
 *   1. choose the outliers                      ("Outlier-separated activation compression")
 *   2. keep them, value and index, uncompressed
 *   3. set them to zero in the activation
 *   4. quantise what is left, group by group, in its original memory order
 *      (Eq. 2 symmetric, Eq. 3 asymmetric)
 *   5. decompression: code * S (+ O), then the outliers are put back.
 *
 * Readings taken where the paper is silent (each is listed in the design notes):
 *   - input is bf16 or (the paper's own format) binary16, arithmetic is binary32, the bit width b
 *     generalises the paper's 4 (divisor 8 -> 2^(b-1), divisor 16 -> 2^b, clip [-2^(b-1), 2^(b-1)-1]);
 *   - the tensor is one flat array cut into groups from its start; when the group length does not
 *     divide the number of elements, the last group is the shorter one and is treated like any
 *     other group over the elements it has (its own scale; its own mean and variance, divided by
 *     its own count; at most as many largest values as it has elements);
 *   - outliers are single elements picked by |x| > tau, by x^2 > k^2 * var of the
 *     statistics group, or as the k largest magnitudes of the group (the paper
 *     picks whole channels by Z-score; same extract / zero / quantise structure);
 *   - X / S is evaluated as X * (D / max): one binary32 division per group, one binary32
 *     multiplication per element, and that product is then rounded to the nearest integer;
 *   - "nearest rounding" is round-half-to-even;
 *   - sums for the variance are canonical pairwise (binary tree) binary32 sums;
 *   - Inf and NaN are always outliers when outliers are kept; they never enter
 *     a scale; a negative zero counts as zero.
 *
 * Build: gcc -std=c11 -O2 -ffp-contract=off -fno-fast-math (x86-64 SSE2: strict binary32).
 */
#include "adacc_oracle.h"

#include <float.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---------- 16-bit formats <-> binary32 ---------- */

static float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

static uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN stays NaN */
  u += 0x7FFFu + ((u >> 16) & 1u); /* ties go to the even 16-bit pattern */
  return (uint16_t)(u >> 16);
}

/* binary16: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits.  Every value is a binary32 value. */
static float f16_to_f32(uint16_t b) {
  const int e = (b >> 10) & 0x1F;
  const int frac = b & 0x3FF;
  float mag;
  if (e == 0x1F)
    mag = frac ? NAN : INFINITY;
  else if (e == 0)
    mag = ldexpf((float)frac, -24); /* subnormal: frac * 2^-24 */
  else
    mag = ldexpf((float)(frac + 1024), e - 25); /* (1 + frac/1024) * 2^(e-15) */
  return (b & 0x8000u) ? -mag : mag;
}

/* Round to nearest, ties to even.  Values of magnitude 65520 and above (half a step past the largest
 * finite value, 65504) become infinite. */
static uint16_t f32_to_f16_rne(float f) {
  const uint16_t sign = signbit(f) ? 0x8000u : 0u;
  if (isnan(f)) return (uint16_t)(sign | 0x7E00u);
  const double a = fabs((double)f);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u);
  int e2;
  frexp(a, &e2);                                 /* a = frac * 2^e2 with frac in [0.5, 1): a in [2^(e2-1), 2^e2) */
  int e = (a == 0.0) ? -14 : e2 - 1;
  if (e < -14) e = -14;                          /* subnormal range: fixed spacing 2^-24 */
  const double steps = rint(ldexp(a, 10 - e));   /* a in units of the spacing 2^(e-10): exact scaling, one rounding */
  /* steps is in [0, 2048]; 2048 means the value rounded up into the next binade, 1024 .. 2047 is a
   * normal number of exponent e, below 1024 (only when e == -14) a subnormal */
  uint32_t bits;
  if (steps >= 2048.0)
    bits = (uint32_t)(e + 1 + 15) << 10;
  else if (steps >= 1024.0)
    bits = ((uint32_t)(e + 15) << 10) | ((uint32_t)steps - 1024u);
  else
    bits = (uint32_t)steps;
  return (uint16_t)(sign | bits);
}

static float to_f32(const oracle_method *m, uint16_t b) {
  return m->dtype == ORACLE_DT_F16 ? f16_to_f32(b) : bf16_to_f32(b);
}

static uint16_t from_f32(const oracle_method *m, float f) {
  return m->dtype == ORACLE_DT_F16 ? f32_to_f16_rne(f) : f32_to_bf16_rne(f);
}

/* Inf or NaN: the exponent field is all ones.  In both formats the 15 low bits, read as an integer,
 * grow with |x|, and the patterns that are not finite are the largest. */
static int is_nonfinite(const oracle_method *m, uint16_t b) {
  return (b & 0x7FFFu) >= (m->dtype == ORACLE_DT_F16 ? 0x7C00u : 0x7F80u);
}

float oracle_to_f32(const oracle_method *m, uint16_t b) { return to_f32(m, b); }
uint16_t oracle_from_f32(const oracle_method *m, float f) { return from_f32(m, f); }

/* ---------- canonical pairwise sum ----------
 * Pad with +0 to the next power of two, then add neighbours until one value is left:
 * level 1 adds (v0,v1), (v2,v3), ...; level 2 adds those sums two by two; and so on. */
float oracle_pairwise_sum(const float *v, size_t n) {
  size_t p = 1;
  while (p < n) p <<= 1;
  float *s = (float *)malloc(p * sizeof(float));
  for (size_t i = 0; i < p; ++i) s[i] = (i < n) ? v[i] : 0.0f;
  while (p > 1) {
    for (size_t j = 0; j < p / 2; ++j) s[j] = s[2 * j] + s[2 * j + 1];
    p /= 2;
  }
  float r = s[0];
  free(s);
  return r;
}

static int method_ok(const oracle_method *m, size_t n) {
  if (m->bits != 4 && m->bits != 8) return 0;
  (void)n; /* any length: the last group of either kind may be short */
  if (m->dtype > ORACLE_DT_F16) return 0;
  if (m->quant_group == 0) return 0;
  if (m->outlier_mode > ORACLE_OUT_TOPK) return 0;
  if (m->outlier_mode == ORACLE_OUT_STD || m->outlier_mode == ORACLE_OUT_TOPK) {
    if (m->stat_group == 0) return 0;
  }
  if (m->outlier_mode == ORACLE_OUT_TOPK && (m->topk == 0 || m->topk > m->stat_group)) return 0;
  return 1;
}

/* ---------- step 1: outlier selection ---------- */

/* |x| > tau, compared in binary32. */
static void select_abs(const oracle_method *m, const uint16_t *x, size_t n, uint8_t *out) {
  for (size_t i = 0; i < n; ++i) out[i] = fabsf(to_f32(m, x[i])) > m->thresh;
}

/* x^2 > k^2 * var, var = population variance of the statistics group about its mean.
 * The group's own outliers are part of the statistics (one pass, nothing is removed first). */
static void select_std(const oracle_method *m, const uint16_t *x, size_t n, uint8_t *out) {
  const size_t gs = m->stat_group;
  const float k2 = m->thresh * m->thresh;
  float *v = (float *)malloc(gs * sizeof(float));
  float *v2 = (float *)malloc(gs * sizeof(float));
  for (size_t g0 = 0; g0 < n; g0 += gs) {
    const size_t cnt = (n - g0 < gs) ? n - g0 : gs; /* the last group may be short */
    const uint16_t *xg = x + g0;
    for (size_t i = 0; i < cnt; ++i) {
      v[i] = to_f32(m, xg[i]);
      v2[i] = v[i] * v[i]; /* exact: two significands of at most 11 bits */
    }
    float s1 = oracle_pairwise_sum(v, cnt);
    float s2 = oracle_pairwise_sum(v2, cnt);
    float mean = s1 / (float)cnt;
    float var = fmaf(-mean, mean, s2 / (float)cnt);
    if (var < 0.0f) var = 0.0f; /* a NaN (non-finite input) stays NaN: nothing then passes the test */
    float limit = k2 * var;
    for (size_t i = 0; i < cnt; ++i) out[g0 + i] = v2[i] > limit;
  }
  free(v);
  free(v2);
}

/* The k largest magnitudes of each statistics group (all of a group that has no more than k).
 * Magnitudes are compared as the 15 low bits of the pattern (monotone in |x| in both formats);
 * equal magnitudes are ranked by position, the earlier one first. */
static void select_topk(const oracle_method *m, const uint16_t *x, size_t n, uint8_t *out) {
  const size_t gs = m->stat_group;
  for (size_t g0 = 0; g0 < n; g0 += gs) {
    const size_t cnt = (n - g0 < gs) ? n - g0 : gs; /* the last group may be short */
    const uint16_t *xg = x + g0;
    uint8_t *og = out + g0;
    memset(og, 0, cnt);
    for (uint32_t r = 0; r < m->topk && r < cnt; ++r) {
      size_t best = cnt;
      for (size_t i = 0; i < cnt; ++i) {
        if (og[i]) continue;
        if (best == cnt || (xg[i] & 0x7FFFu) > (xg[best] & 0x7FFFu)) best = i;
      }
      og[best] = 1;
    }
  }
}

int oracle_select_outliers(const oracle_method *m, const uint16_t *x, size_t n, uint8_t *out) {
  if (!method_ok(m, n)) return -1;
  switch (m->outlier_mode) {
    case ORACLE_OUT_NONE: memset(out, 0, n); return 0; /* nothing is kept aside */
    case ORACLE_OUT_ABS: select_abs(m, x, n, out); break;
    case ORACLE_OUT_STD: select_std(m, x, n, out); break;
    case ORACLE_OUT_TOPK: select_topk(m, x, n, out); break;
  }
  /* a value that cannot be quantised at all is always kept exactly */
  for (size_t i = 0; i < n; ++i)
    if (is_nonfinite(m, x[i])) out[i] = 1;
  return 0;
}

/* ---------- step 4: quantisation of one group ---------- */

static int8_t clip_code(float r, int q) {
  /* written so that a NaN lands on the lower bound */
  if (!(r >= (float)(-q))) r = (float)(-q);
  if (r > (float)(q - 1)) r = (float)(q - 1);
  return (int8_t)r;
}

/* Eq. 2:  S = max|X| / D,  code = clip(round(X / S), -Q, Q-1),  D = Q (paper) or Q-1. */
static void quant_sym(const oracle_method *m, const float *y, size_t g, int8_t *codes, float *scale) {
  const int q = 1 << (m->bits - 1);
  const float d = (m->scale_rule == ORACLE_RULE_PAPER) ? (float)q : (float)(q - 1);
  float a = 0.0f;
  for (size_t i = 0; i < g; ++i)
    if (fabsf(y[i]) > a) a = fabsf(y[i]);
  *scale = a / d;
  float inv = 0.0f;
  if (a != 0.0f) {
    inv = d / a;
    if (inv > FLT_MAX) inv = FLT_MAX; /* a is so small that D/a overflows */
  }
  for (size_t i = 0; i < g; ++i) codes[i] = clip_code(rintf(y[i] * inv), q);
}

/* Eq. 3:  O = (max+min)/2,  S = (max-min)/D2,  code = clip(round((X-O)/S), -Q, Q-1),
 * D2 = 2Q (paper: 16 for 4 bits) or 2Q-1. */
static void quant_asym(const oracle_method *m, const float *y, size_t g, int8_t *codes, float *scale,
                       float *zp) {
  const int q = 1 << (m->bits - 1);
  const float d2 = (m->scale_rule == ORACLE_RULE_PAPER) ? (float)(2 * q) : (float)(2 * q - 1);
  float hi = y[0], lo = y[0];
  for (size_t i = 1; i < g; ++i) {
    if (y[i] > hi) hi = y[i];
    if (y[i] < lo) lo = y[i];
  }
  float o = (hi + lo) * 0.5f;
  float r = hi - lo;
  *zp = o;
  *scale = r / d2;
  float inv = 0.0f;
  if (r != 0.0f) {
    inv = d2 / r;
    if (inv > FLT_MAX) inv = FLT_MAX;
  }
  for (size_t i = 0; i < g; ++i) codes[i] = clip_code(rintf((y[i] - o) * inv), q);
}

/* Steps 3 and 4 for a given outlier mask, then the packing of the codes. */
static void quantise_rest(const oracle_method *m, const uint16_t *x, const uint8_t *out, size_t n,
                          int8_t *codes, uint8_t *packed, float *scale, float *zp) {
  float *y = (float *)malloc((n ? n : 1) * sizeof(float));

  /* 3. zero them in the activation; a value that is not finite, or a negative
   *    zero, also counts as zero from here on */
  for (size_t i = 0; i < n; ++i) {
    float f = to_f32(m, x[i]);
    if (out[i] || is_nonfinite(m, x[i]) || f == 0.0f) f = 0.0f;
    y[i] = f;
  }

  /* 4. quantise every group of the flat array; the last one may be short */
  const size_t gq = m->quant_group;
  for (size_t h = 0; h * gq < n; ++h) {
    const size_t cnt = (n - h * gq < gq) ? n - h * gq : gq;
    if (m->asym)
      quant_asym(m, y + h * gq, cnt, codes + h * gq, scale + h, zp + h);
    else
      quant_sym(m, y + h * gq, cnt, codes + h * gq, scale + h);
  }

  /* pack */
  if (packed) {
    if (m->bits == 8) {
      for (size_t i = 0; i < n; ++i) packed[i] = (uint8_t)codes[i];
    } else {
      for (size_t j = 0; j < (n + 1) / 2; ++j) {
        int lo = codes[2 * j] & 0xF;
        int hi = (2 * j + 1 < n) ? (codes[2 * j + 1] & 0xF) : 0; /* odd n: last high nibble is 0 */
        packed[j] = (uint8_t)(lo | (hi << 4));
      }
    }
  }
  free(y);
}

/* ---------- steps 1-4 ---------- */

int oracle_compress(const oracle_method *m, const uint16_t *x, size_t n, int8_t *codes, uint8_t *packed,
                    float *scale, float *zp, int32_t *out_idx, uint16_t *out_val, size_t cap,
                    size_t *n_out) {
  if (!method_ok(m, n)) return -1;
  if (m->asym && !zp) return -1;
  uint8_t *out = (uint8_t *)malloc(n ? n : 1);

  /* 1. which elements are outliers */
  oracle_select_outliers(m, x, n, out);

  /* 2. keep them, in ascending index order, exactly as they are */
  size_t cnt = 0;
  for (size_t i = 0; i < n; ++i) {
    if (!out[i]) continue;
    if (cnt < cap) {
      out_idx[cnt] = (int32_t)i;
      out_val[cnt] = x[i];
    }
    ++cnt;
  }
  if (n_out) *n_out = cnt;

  quantise_rest(m, x, out, n, codes, packed, scale, zp);
  free(out);
  return 0;
}

/* ---------- step 5 ---------- */

static int unpack_code(const oracle_method *m, const uint8_t *packed, size_t i) {
  if (m->bits == 8) return (int8_t)packed[i];
  int nib = (packed[i / 2] >> ((i & 1) ? 4 : 0)) & 0xF;
  return (nib >= 8) ? nib - 16 : nib;
}

/* X^ = code * S (+ O) for every element */
static void dequantise_all(const oracle_method *m, const uint8_t *packed, const float *scale, const float *zp,
                           size_t n, float *xhat_f32, uint16_t *xhat_bf16) {
  const size_t gq = m->quant_group;
  for (size_t i = 0; i < n; ++i) {
    float c = (float)unpack_code(m, packed, i);
    float s = scale[i / gq];
    float v = m->asym ? fmaf(c, s, zp[i / gq]) : c * s; /* X^ = code * S (+ O) */
    if (xhat_f32) xhat_f32[i] = v;
    if (xhat_bf16) xhat_bf16[i] = from_f32(m, v);
  }
}

int oracle_decompress(const oracle_method *m, const uint8_t *packed, const float *scale, const float *zp,
                      const int32_t *out_idx, const uint16_t *out_val, size_t n_out, size_t n,
                      float *xhat_f32, uint16_t *xhat_bf16) {
  if (!method_ok(m, n)) return -1;
  if (m->asym && !zp) return -1;
  dequantise_all(m, packed, scale, zp, n, xhat_f32, xhat_bf16);
  for (size_t j = 0; j < n_out; ++j) {
    size_t i = (size_t)out_idx[j];
    if (i >= n) return -1;
    if (xhat_f32) xhat_f32[i] = to_f32(m, out_val[j]);
    if (xhat_bf16) xhat_bf16[i] = out_val[j];
  }
  return 0;
}

uint64_t oracle_logical_bytes(const oracle_method *m, size_t n, size_t n_out) {
  uint64_t groups = (n + m->quant_group - 1) / m->quant_group;
  return ((uint64_t)n * m->bits + 7) / 8 + 4ull * groups * (m->asym ? 2 : 1) + 6ull * n_out;
}

/* ====================================================================================
 * Outlier CHANNELS (Section 3.2, Eq. 1): the paper's own selection rule.
 *
 * The activation is a matrix of `tokens` rows and `hidden` channels, row-major.  For channel h,
 * S_h is the sum over the tokens of |x|; mu and sigma are mean and standard deviation of S_h over
 * the channels; Z_h = (S_h - mu) / sigma; channels with Z_h above the threshold (3 in the paper)
 * are kept whole and uncompressed, with their indices, are zeroed in the activation, and the rest
 * is quantised as before.
 *
 * Readings (the printed Eq. 1 has a slipped subscript; the text after it defines the terms):
 *   - sigma is the population standard deviation (divide by the number of channels);
 *   - the threshold is compared against Z itself, formed by one binary64 division;
 *   - a channel whose sum is not finite is always an outlier and takes no part in mu and sigma;
 *   - if sigma is zero or not a number (all channels alike, or none left), nothing else is selected.
 * S_h is the exact sum, rounded once to binary64 (the magnitude of a finite value of either 16-bit
 * format is an integer multiple of 2^-133 below 2^128, so the sum is kept as a 320-bit integer); mu and sigma
 * are the textbook two-pass mean and standard deviation, plain binary64 loops in channel order.
 * ==================================================================================== */

/* sum of magnitudes as an integer count of 2^-133, five 64-bit limbs, least significant first */
typedef struct exact_sum { uint64_t limb[5]; } exact_sum;

/* adds the magnitude of the finite 16-bit pattern b */
static void exact_add(exact_sum *a, uint32_t dtype, uint16_t b) {
  uint64_t sig;
  uint32_t shift; /* |x| = sig * 2^shift * 2^-133 */
  if (dtype == ORACLE_DT_F16) {
    const uint32_t e = (b >> 10) & 0x1Fu;
    sig = e ? ((b & 0x3FFu) | 0x400u) : (b & 0x3FFu); /* |x| = sig * 2^(max(e,1) - 25) */
    shift = (e ? e : 1u) + 108u;
  } else {
    const uint32_t e = (b >> 7) & 0xFFu;
    sig = e ? ((b & 0x7Fu) | 0x80u) : (b & 0x7Fu); /* |x| = sig * 2^(max(e,1) - 134) */
    shift = e ? e - 1u : 0u;
  }
  const unsigned __int128 v = (unsigned __int128)sig << (shift % 64u);
  uint64_t add[2] = {(uint64_t)v, (uint64_t)(v >> 64)};
  uint64_t carry = 0;
  for (uint32_t i = shift / 64u, k = 0; i < 5; ++i, ++k) {
    const unsigned __int128 t = (unsigned __int128)a->limb[i] + (k < 2 ? add[k] : 0u) + carry;
    a->limb[i] = (uint64_t)t;
    carry = (uint64_t)(t >> 64);
  }
}

/* the 320-bit integer times 2^-133, rounded to the nearest binary64, ties to even */
static double exact_round(const exact_sum *a) {
  int top = -1; /* position of the highest set bit */
  for (int i = 4; i >= 0 && top < 0; --i)
    if (a->limb[i])
      for (int j = 63; j >= 0; --j)
        if ((a->limb[i] >> j) & 1u) { top = 64 * i + j; break; }
  if (top < 0) return 0.0;
  uint64_t mant = 0; /* the 53 bits from `top` down (fewer if the number is shorter) */
  int low = top - 52;
  if (low < 0) low = 0;
  for (int p = top; p >= low; --p) mant = (mant << 1) | ((a->limb[p / 64] >> (p % 64)) & 1u);
  if (low > 0) {
    const int guard = (int)((a->limb[(low - 1) / 64] >> ((low - 1) % 64)) & 1u);
    int sticky = 0;
    for (int p = low - 2; p >= 0 && !sticky; --p) sticky = (int)((a->limb[p / 64] >> (p % 64)) & 1u);
    if (guard && (sticky || (mant & 1u))) ++mant; /* 2^53 is still exact as a double */
  }
  return ldexp((double)mant, low - 133);
}

/* S_h = sum over the tokens of |x|, for every channel. */
void oracle_channel_scores(uint32_t dtype, const uint16_t *x, size_t tokens, size_t hidden, double *S) {
  const uint16_t inf = (dtype == ORACLE_DT_F16) ? 0x7C00u : 0x7F80u;
  for (size_t h = 0; h < hidden; ++h) {
    exact_sum acc;
    memset(&acc, 0, sizeof acc);
    int inf_seen = 0, nan_seen = 0;
    for (size_t t = 0; t < tokens; ++t) {
      const uint16_t b = x[t * hidden + h];
      if ((b & 0x7FFFu) > inf) nan_seen = 1;
      else if ((b & 0x7FFFu) == inf) inf_seen = 1;
      else exact_add(&acc, dtype, b);
    }
    S[h] = nan_seen ? (double)NAN : inf_seen ? (double)INFINITY : exact_round(&acc);
  }
}

/* Eq. 1.  is_out[h] = 1 for an outlier channel.  stats (may be NULL) receives mu, sigma. */
void oracle_channel_select(const double *S, size_t hidden, float z_thresh, uint8_t *is_out, double *stats) {
  size_t finite = 0;
  double sum = 0.0;
  for (size_t h = 0; h < hidden; ++h)
    if (isfinite(S[h])) {
      sum = sum + S[h];
      ++finite;
    }
  const double mu = sum / (double)finite;
  double ss = 0.0;
  for (size_t h = 0; h < hidden; ++h)
    if (isfinite(S[h])) {
      const double d = S[h] - mu;
      ss = ss + d * d;
    }
  const double sigma = sqrt(ss / (double)finite);
  for (size_t h = 0; h < hidden; ++h) {
    const double z = (S[h] - mu) / sigma;
    is_out[h] = !isfinite(S[h]) || z > (double)z_thresh; /* a NaN z selects nothing */
  }
  if (stats) {
    stats[0] = mu;
    stats[1] = sigma;
  }
}

static int channel_method_ok(const oracle_method *m, size_t tokens, size_t hidden) {
  if (hidden == 0 || m->outlier_mode != ORACLE_OUT_NONE) return 0;
  return method_ok(m, tokens * hidden);
}

/* Compression with outlier channels.  Outputs as oracle_compress, except for the outliers:
 *   ch_idx [cap]            the outlier channels, ascending (at most cap are written)
 *   ch_val [tokens * n_ch]  their values, token by token: ch_val[t * n_ch + r] is channel ch_idx[r]
 *                           of token t, the original bf16 bit pattern
 *   n_ch                    the number of outlier channels
 * If n_ch exceeds cap only ch_idx and n_ch are produced. */
int oracle_channel_compress(const oracle_method *m, const uint16_t *x, size_t tokens, size_t hidden,
                            float z_thresh, int8_t *codes, uint8_t *packed, float *scale, float *zp,
                            int32_t *ch_idx, uint16_t *ch_val, size_t cap, size_t *n_ch) {
  if (!channel_method_ok(m, tokens, hidden)) return -1;
  if (m->asym && !zp) return -1;
  const size_t n = tokens * hidden;
  double *S = (double *)malloc(hidden * sizeof(double));
  uint8_t *is_out = (uint8_t *)malloc(hidden);
  oracle_channel_scores(m->dtype, x, tokens, hidden, S);
  oracle_channel_select(S, hidden, z_thresh, is_out, NULL);
  size_t cnt = 0;
  for (size_t h = 0; h < hidden; ++h)
    if (is_out[h]) {
      if (cnt < cap) ch_idx[cnt] = (int32_t)h;
      ++cnt;
    }
  if (n_ch) *n_ch = cnt;
  if (cnt <= cap) {
    /* the outlier channels are kept as they are ... */
    for (size_t t = 0; t < tokens; ++t)
      for (size_t r = 0; r < cnt; ++r) ch_val[t * cnt + r] = x[t * hidden + (size_t)ch_idx[r]];
    /* ... and count as zero when the rest is quantised */
    uint8_t *out = (uint8_t *)malloc(n ? n : 1);
    for (size_t i = 0; i < n; ++i) out[i] = is_out[i % hidden];
    quantise_rest(m, x, out, n, codes, packed, scale, zp);
    free(out);
  }
  free(S);
  free(is_out);
  return 0;
}

/* Dequantise, then put the outlier channels back. */
int oracle_channel_decompress(const oracle_method *m, const uint8_t *packed, const float *scale, const float *zp,
                              const int32_t *ch_idx, const uint16_t *ch_val, size_t n_ch, size_t tokens,
                              size_t hidden, float *xhat_f32, uint16_t *xhat_bf16) {
  if (!channel_method_ok(m, tokens, hidden)) return -1;
  if (m->asym && !zp) return -1;
  dequantise_all(m, packed, scale, zp, tokens * hidden, xhat_f32, xhat_bf16);
  for (size_t t = 0; t < tokens; ++t)
    for (size_t r = 0; r < n_ch; ++r) {
      const size_t h = (size_t)ch_idx[r];
      if (h >= hidden) return -1;
      if (xhat_f32) xhat_f32[t * hidden + h] = to_f32(m, ch_val[t * n_ch + r]);
      if (xhat_bf16) xhat_bf16[t * hidden + h] = ch_val[t * n_ch + r];
    }
  return 0;
}

/* ====================================================================================
 * Dropout mask (Section 3.2, list of layer-specific schemes): the mask of an attention layer is
 * kept in bit format instead of byte format, without loss.  Element i of the mask (a byte, zero =
 * dropped, anything else = kept) becomes bit (i mod 8) of byte i / 8; unused bits of the last
 * byte are zero.  Unpacking yields bytes 0 and 1.
 * ==================================================================================== */
void oracle_mask_pack(const uint8_t *mask, size_t n, uint8_t *bits) {
  for (size_t j = 0; j < (n + 7) / 8; ++j) bits[j] = 0;
  for (size_t i = 0; i < n; ++i)
    if (mask[i] != 0) bits[i / 8] = (uint8_t)(bits[i / 8] | (1u << (i % 8)));
}

void oracle_mask_unpack(const uint8_t *bits, size_t n, uint8_t *mask) {
  for (size_t i = 0; i < n; ++i) mask[i] = (uint8_t)((bits[i / 8] >> (i % 8)) & 1u);
}

/* ====================================================================================
 * Channel-wise symmetric quantisation (Section 3.2, list of layer-specific schemes: the scheme for
 * the Query, Key and Value matrices).  The tensor is a row-major matrix of `tokens` rows and
 * `hidden` channels; every channel (column) is one quantisation group of Eq. 2: S_h = max over the
 * tokens of |x| / D, code = clip(round(x / S_h)).  The codes stay in the tensor's own memory order
 * (no transposition, "no extra memory alignment is needed").  No outliers are separated; as in
 * the other schemes a value that is not finite, or a negative zero, counts as zero.
 * ==================================================================================== */
int oracle_channelwise_compress(const oracle_method *m, const uint16_t *x, size_t tokens, size_t hidden,
                                int8_t *codes, uint8_t *packed, float *scale) {
  if ((m->bits != 4 && m->bits != 8) || m->asym || m->outlier_mode != ORACLE_OUT_NONE || hidden == 0) return -1;
  const size_t n = tokens * hidden;
  float *col = (float *)malloc((tokens ? tokens : 1) * sizeof(float));
  int8_t *ccol = (int8_t *)malloc(tokens ? tokens : 1);
  for (size_t h = 0; h < hidden; ++h) {
    for (size_t t = 0; t < tokens; ++t) {
      float f = to_f32(m, x[t * hidden + h]);
      if (is_nonfinite(m, x[t * hidden + h]) || f == 0.0f) f = 0.0f;
      col[t] = f;
    }
    quant_sym(m, col, tokens, ccol, scale + h); /* Eq. 2 with the channel as the group */
    for (size_t t = 0; t < tokens; ++t) codes[t * hidden + h] = ccol[t];
  }
  if (packed) {
    if (m->bits == 8) {
      for (size_t i = 0; i < n; ++i) packed[i] = (uint8_t)codes[i];
    } else {
      for (size_t j = 0; j < (n + 1) / 2; ++j) {
        int lo = codes[2 * j] & 0xF;
        int hi = (2 * j + 1 < n) ? (codes[2 * j + 1] & 0xF) : 0;
        packed[j] = (uint8_t)(lo | (hi << 4));
      }
    }
  }
  free(col);
  free(ccol);
  return 0;
}

/* X^ = code * S_h */
int oracle_channelwise_decompress(const oracle_method *m, const uint8_t *packed, const float *scale, size_t tokens,
                                  size_t hidden, float *xhat_f32, uint16_t *xhat_bf16) {
  if ((m->bits != 4 && m->bits != 8) || m->asym || hidden == 0) return -1;
  for (size_t i = 0; i < tokens * hidden; ++i) {
    float v = (float)unpack_code(m, packed, i) * scale[i % hidden];
    if (xhat_f32) xhat_f32[i] = v;
    if (xhat_bf16) xhat_bf16[i] = from_f32(m, v);
  }
  return 0;
}
