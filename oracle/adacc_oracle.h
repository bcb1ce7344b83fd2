/*
 * CPU oracle for outlier-separated activation compression (Adacc, arXiv 2508.00806, Section 3.2).
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain reference that the GPU
 * library is checked against.  Nothing in the product path may call it; it
 * shares no code, header, table or constant with the HIP implementation.
 *
 * The oracle works on logical arrays (one code per element, one scale per
 * quantisation group, a sorted outlier list).  It knows nothing about tiles,
 * lanes, blobs or any other device-side layout.
 *
 * Arithmetic: every floating-point step is IEEE-754 binary32 in the order
 * written in adacc_oracle.c (the scale is stored as a 32-bit float in
 * Section 3.2, and each code is an integer decided by that arithmetic, so the
 * precision is fixed rather than widened to binary64).
 */
#ifndef ADACC_ORACLE_H
#define ADACC_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_OUT_NONE = 0, ORACLE_OUT_ABS = 1, ORACLE_OUT_STD = 2, ORACLE_OUT_TOPK = 3 };
enum { ORACLE_RULE_PAPER = 0, ORACLE_RULE_FULLRANGE = 1 };
enum { ORACLE_DT_BF16 = 0, ORACLE_DT_F16 = 1 }; /* the 16-bit format of the tensor: bfloat16 or IEEE binary16 */

typedef struct oracle_method {
  uint32_t bits;         /* 4 or 8                                                  */
  uint32_t quant_group;  /* elements per scale (Section 3.2, "group the activations") */
  uint32_t asym;         /* 0: Eq. 2 (symmetric)   1: Eq. 3 (asymmetric)            */
  uint32_t scale_rule;   /* PAPER: divisor 2^(b-1) resp. 2^b;  FULLRANGE: 2^(b-1)-1 resp. 2^b-1 */
  uint32_t outlier_mode; /* ORACLE_OUT_*                                            */
  uint32_t stat_group;   /* elements per statistics group (STD, TOPK)               */
  float    thresh;       /* ABS: tau     STD: k (multiples of the group's std)      */
  uint32_t topk;         /* TOPK: outliers kept per statistics group                */
  uint32_t dtype;        /* ORACLE_DT_*: format of the input, of the kept outliers and of the 16-bit output */
} oracle_method;

/* The two conversions every other function uses, exported so that they can be pinned on their own:
 * a 16-bit pattern of the method's format as binary32 (exact), and binary32 rounded to that format
 * (to nearest, ties to even; NaN stays NaN; too large becomes infinite). */
float oracle_to_f32(const oracle_method *m, uint16_t b);
uint16_t oracle_from_f32(const oracle_method *m, float f);

/* Step 1: which elements are outliers.  out[i] = 1 for an outlier, else 0.
 * x holds n bf16 bit patterns.  Returns 0, or -1 on a malformed method. */
int oracle_select_outliers(const oracle_method *m, const uint16_t *x, size_t n, uint8_t *out);

/* Steps 1-4 together.  Outputs (all caller-allocated):
 *   codes   [n]        one signed code per element, in [-2^(b-1), 2^(b-1)-1]
 *   packed  [ceil(n*b/8)] the same codes packed (b=8: one byte each; b=4: element 2j
 *                      in the low nibble of byte j, element 2j+1 in the high nibble)
 *   scale   [n/Gq]     S per quantisation group (binary32)
 *   zp      [n/Gq]     O per quantisation group (asym only; may be NULL otherwise)
 *   out_idx [cap], out_val [cap]   outliers in ascending index order, values as the
 *                      original bf16 bit patterns; at most cap are written
 *   n_out              the true number of outliers (may exceed cap)
 * Returns 0, or -1 on a malformed method. */
int oracle_compress(const oracle_method *m, const uint16_t *x, size_t n,
                    int8_t *codes, uint8_t *packed, float *scale, float *zp,
                    int32_t *out_idx, uint16_t *out_val, size_t cap, size_t *n_out);

/* Step 5: dequantise, then put the outliers back.
 *   xhat_f32  [n]  binary32 result          (may be NULL)
 *   xhat_bf16 [n]  its round-to-nearest-even bf16 image; outlier positions carry
 *                  the stored bit pattern unchanged  (may be NULL) */
int oracle_decompress(const oracle_method *m, const uint8_t *packed, const float *scale,
                      const float *zp, const int32_t *out_idx, const uint16_t *out_val,
                      size_t n_out, size_t n, float *xhat_f32, uint16_t *xhat_bf16);

/* Bytes a compressed tensor needs, without any padding:
 * codes + scales (+ offsets) + 6 bytes per outlier (4-byte index, 2-byte value). */
uint64_t oracle_logical_bytes(const oracle_method *m, size_t n, size_t n_out);

/* Canonical pairwise sum (exposed so tests can pin it on its own). */
float oracle_pairwise_sum(const float *v, size_t n);

/* ---- outlier channels (Section 3.2, Eq. 1) ----
 * x is a row-major matrix of `tokens` rows and `hidden` channels.  S_h is the exact sum rounded once
 * to binary64; mu and sigma are plain two-pass binary64 loops over the channels. */

/* S_h = sum over the tokens of |x|, for every channel. */
void oracle_channel_scores(uint32_t dtype, const uint16_t *x, size_t tokens, size_t hidden, double *S);

/* Eq. 1: is_out[h] = 1 where Z_h = (S_h - mu) / sigma exceeds z_thresh (or S_h is not finite).
 * stats (may be NULL) receives mu and sigma. */
void oracle_channel_select(const double *S, size_t hidden, float z_thresh, uint8_t *is_out, double *stats);

/* Compression with whole outlier channels; m->outlier_mode must be ORACLE_OUT_NONE.
 *   ch_idx [cap]            the outlier channels, ascending (at most cap are written)
 *   ch_val [tokens * n_ch]  ch_val[t * n_ch + r] = channel ch_idx[r] of token t (bf16 bits)
 * codes, packed, scale, zp as oracle_compress, with the outlier channels counted as zero.
 * If *n_ch exceeds cap only ch_idx and *n_ch are produced. */
int oracle_channel_compress(const oracle_method *m, const uint16_t *x, size_t tokens, size_t hidden,
                            float z_thresh, int8_t *codes, uint8_t *packed, float *scale, float *zp,
                            int32_t *ch_idx, uint16_t *ch_val, size_t cap, size_t *n_ch);

int oracle_channel_decompress(const oracle_method *m, const uint8_t *packed, const float *scale, const float *zp,
                              const int32_t *ch_idx, const uint16_t *ch_val, size_t n_ch, size_t tokens,
                              size_t hidden, float *xhat_f32, uint16_t *xhat_bf16);

/* ---- channel-wise symmetric quantisation (Section 3.2: the scheme for Query, Key and Value) ----
 * x: row-major [tokens][hidden]; one scale per channel, S_h = max_t |x| / D (Eq. 2 with the channel as
 * the group); codes in the tensor's own order.  m: bits, scale_rule; asym must be 0, outlier_mode NONE;
 * quant_group is ignored.  scale [hidden]. */
int oracle_channelwise_compress(const oracle_method *m, const uint16_t *x, size_t tokens, size_t hidden,
                                int8_t *codes, uint8_t *packed, float *scale);
int oracle_channelwise_decompress(const oracle_method *m, const uint8_t *packed, const float *scale, size_t tokens,
                                  size_t hidden, float *xhat_f32, uint16_t *xhat_bf16);

/* ---- dropout mask: byte format <-> bit format (Section 3.2), lossless ----
 * mask: n bytes, zero = dropped, non-zero = kept.  bits: ceil(n/8) bytes, element i in bit i%8 of
 * byte i/8, unused bits zero.  Unpacking writes bytes 0 and 1. */
void oracle_mask_pack(const uint8_t *mask, size_t n, uint8_t *bits);
void oracle_mask_unpack(const uint8_t *bits, size_t n, uint8_t *mask);

#ifdef __cplusplus
}
#endif
#endif
