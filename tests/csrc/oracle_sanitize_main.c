/* Drives every entry point of the oracle on small seeded inputs; built with
 * -fsanitize=address,undefined by tests/test_oracle_sanitizers.py: any out-of-bounds access, use after
 * free, signed overflow or misaligned access in the oracle ends the run with a report. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "adacc_oracle.h"

static uint32_t state = 12345u;
static uint32_t next(void) { state = state * 1664525u + 1013904223u; return state; }

static void fill(uint16_t *x, size_t n, uint32_t dtype) {
  for (size_t i = 0; i < n; ++i) {
    uint32_t r = next();
    /* mostly moderate magnitudes, now and then anything at all (Inf, NaN, subnormals) */
    if ((r & 63u) == 0) x[i] = (uint16_t)(r >> 16);
    else if (dtype == ORACLE_DT_F16) x[i] = (uint16_t)(((r >> 16) & 0x8000u) | (0x3000u + ((r >> 8) & 0x0FFFu)));
    else x[i] = (uint16_t)(((r >> 16) & 0x8000u) | (0x3E00u + ((r >> 8) & 0x03FFu)));
  }
}

static int run(const oracle_method *m, size_t n) {
  uint16_t *x = malloc(n * 2 + 2), *ov = malloc(n * 2 + 2), *b16 = malloc(n * 2 + 2);
  int8_t *codes = malloc(n + 1);
  uint8_t *packed = malloc((n * m->bits + 7) / 8 + 1), *sel = malloc(n + 1);
  size_t groups = (n + m->quant_group - 1) / m->quant_group;
  float *scale = malloc(groups * 4 + 4), *zp = malloc(groups * 4 + 4), *f32 = malloc(n * 4 + 4);
  int32_t *oi = malloc(n * 4 + 4);
  size_t n_out = 0;
  fill(x, n, m->dtype);
  int rc = oracle_select_outliers(m, x, n, sel);
  rc |= oracle_compress(m, x, n, codes, packed, scale, zp, oi, ov, n, &n_out);
  rc |= oracle_decompress(m, packed, scale, zp, oi, ov, n_out, n, f32, b16);
  /* a capacity smaller than the count */
  size_t n2 = 0;
  rc |= oracle_compress(m, x, n, codes, packed, scale, zp, oi, ov, n_out / 2, &n2);
  if (n2 != n_out) rc |= 1;
  (void)oracle_logical_bytes(m, n, n_out);
  free(x); free(ov); free(b16); free(codes); free(packed); free(sel); free(scale); free(zp); free(f32); free(oi);
  return rc;
}

static int run_channels(uint32_t dtype, size_t tokens, size_t hidden) {
  const size_t n = tokens * hidden;
  oracle_method m;
  memset(&m, 0, sizeof m);
  m.bits = 4; m.quant_group = 8; m.dtype = dtype;
  uint16_t *x = malloc(n * 2), *cv = malloc(n * 2), *b16 = malloc(n * 2);
  int8_t *codes = malloc(n);
  uint8_t *packed = malloc((n + 1) / 2), *mask = malloc(n), *bits = malloc((n + 7) / 8), *back = malloc(n);
  float *scale = malloc((n / 8 + 1) * 4 + hidden * 4), *f32 = malloc(n * 4);
  int32_t *ci = malloc(hidden * 4);
  double *S = malloc(hidden * 8), stats[2];
  size_t n_ch = 0;
  fill(x, n, dtype);
  for (size_t t = 0; t < tokens; ++t) x[t * hidden + 3] = (dtype == ORACLE_DT_F16) ? 0x5640 : 0x42C8; /* a channel that stands out */
  oracle_channel_scores(dtype, x, tokens, hidden, S);
  oracle_channel_select(S, hidden, 2.0f, mask, stats);
  int rc = oracle_channel_compress(&m, x, tokens, hidden, 2.0f, codes, packed, scale, NULL, ci, cv, hidden, &n_ch);
  rc |= oracle_channel_decompress(&m, packed, scale, NULL, ci, cv, n_ch, tokens, hidden, f32, b16);
  rc |= oracle_channelwise_compress(&m, x, tokens, hidden, codes, packed, scale);
  rc |= oracle_channelwise_decompress(&m, packed, scale, tokens, hidden, f32, b16);
  for (size_t i = 0; i < n; ++i) mask[i] = (uint8_t)(next() & 1u);
  oracle_mask_pack(mask, n, bits);
  oracle_mask_unpack(bits, n, back);
  if (memcmp(mask, back, n) != 0) rc |= 1;
  free(x); free(cv); free(b16); free(codes); free(packed); free(mask); free(bits); free(back); free(scale); free(f32);
  free(ci); free(S);
  return rc;
}

int main(void) {
  int rc = 0;
  for (uint32_t dtype = 0; dtype < 2; ++dtype)
    for (uint32_t mode = 0; mode < 4; ++mode)
      for (uint32_t bits = 4; bits <= 8; bits += 4)
        for (uint32_t asym = 0; asym < 2; ++asym) {
          static const size_t sizes[] = {1, 7, 64, 333, 1000};
          static const uint32_t groups[][2] = {{8, 8}, {8, 64}, {24, 72}, {64, 64}};
          for (size_t s = 0; s < 5; ++s)
            for (size_t g = 0; g < 4; ++g) {
              oracle_method m;
              memset(&m, 0, sizeof m);
              m.bits = bits; m.quant_group = groups[g][0]; m.asym = asym; m.scale_rule = (uint32_t)(s & 1);
              m.outlier_mode = mode; m.stat_group = groups[g][1]; m.thresh = mode == ORACLE_OUT_ABS ? 0.75f : 1.5f;
              m.topk = 3; m.dtype = dtype;
              rc |= run(&m, sizes[s]);
            }
        }
  for (uint32_t dtype = 0; dtype < 2; ++dtype) {
    rc |= run_channels(dtype, 37, 16);
    rc |= run_channels(dtype, 1, 8);
  }
  float v[5] = {1e8f, 3.0f, -1e8f, 3.0f, 1.0f};
  (void)oracle_pairwise_sum(v, 5);
  printf("oracle sanitizer run: rc=%d\n", rc);
  return rc;
}
