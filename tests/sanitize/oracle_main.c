/* Exercises every function of the oracle on small inputs; built with
 * -fsanitize=address,undefined by tests/test_sanitizers_cpu.py.  Prints a few totals that
 * the test compares with the hand-derived golden values. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int64_t lvo_seq_len(int32_t, const int32_t*);
int lvo_allowed(int32_t, const int32_t*, const int32_t*, int32_t, int32_t, int64_t, int64_t);
int lvo_mask_dense(int32_t, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, uint8_t*);
int lvo_row_counts(int32_t, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, int64_t*);
int lvo_index_sets(int32_t, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, const int64_t*, int32_t*, int64_t);
int lvo_attn(int32_t, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, int32_t, const void*, const void*,
             const void*, int32_t, int32_t, int32_t, int32_t, double, int64_t, const int64_t*, int64_t, int64_t, double*);
int lvo_attn_probs(int32_t, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, const void*, const void*,
                   const void*, int32_t, int32_t, int32_t, int32_t, double, int64_t, int64_t, double*, double*);
int lvo_cfg_share(int32_t, const int32_t*, int32_t, int32_t, const uint8_t*, int32_t, int32_t, int32_t, double*);
int lvo_calibrate(int32_t, const int32_t*, const double*, int32_t, int32_t, double, int32_t*, double*, int32_t);
int lvo_quantize_rows(const void*, int32_t, int64_t, int32_t, int32_t, int32_t*, double*, double*);
int lvo_dequantize_rows(const int32_t*, const double*, const double*, int64_t, int32_t, double*);
int lvo_attn_qkv8(int32_t, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, const void*, const void*,
                  const void*, int32_t, int32_t, int32_t, int32_t, double, int32_t, int64_t, int64_t, double*);

#define CHECK(x) do { int rc_ = (x); if (rc_) { fprintf(stderr, "failed (%d): %s\n", rc_, #x); return 1; } } while (0)

int main(void) {
  const int32_t scales[4] = {1, 2, 3, 4};
  int32_t radii[16];
  for (int i = 0; i < 16; ++i) radii[i] = 1;
  const int64_t L = lvo_seq_len(4, scales);
  enum { B = 2, H = 2, D = 8 };
  uint8_t* mask = malloc((size_t)(L * L));
  int64_t* cnt = malloc((size_t)L * sizeof *cnt);
  int64_t* rowptr = malloc((size_t)(L + 1) * sizeof *rowptr);
  for (int mode = 0; mode < 2; ++mode) {
    CHECK(lvo_mask_dense(4, scales, radii, mode, 0, 0, 4, mask));
    CHECK(lvo_row_counts(4, scales, radii, mode, 0, 0, 4, cnt));
    rowptr[0] = 0;
    for (int64_t i = 0; i < L; ++i) rowptr[i + 1] = rowptr[i] + cnt[i];
    int32_t* cols = malloc((size_t)rowptr[L] * sizeof *cols);
    CHECK(lvo_index_sets(4, scales, radii, mode, 0, 0, 4, rowptr, cols, rowptr[L]));
    printf("pairs mode %d: %lld\n", mode, (long long)rowptr[L]);
    if (lvo_allowed(4, scales, radii, 0, mode, 29, 29) != 1 || lvo_allowed(4, scales, radii, 0, mode, 0, 29) != 0) return 1;
    free(cols);
  }
  float* q = malloc(sizeof(float) * B * H * L * D);
  float* k = malloc(sizeof(float) * B * H * L * D);
  float* v = malloc(sizeof(float) * B * H * L * D);
  unsigned s = 12345;
  for (int64_t i = 0; i < B * H * L * D; ++i) {
    s = s * 1664525u + 1013904223u; q[i] = (float)(s >> 8) / 8388608.f - 1.f;
    s = s * 1664525u + 1013904223u; k[i] = (float)(s >> 8) / 8388608.f - 1.f;
    s = s * 1664525u + 1013904223u; v[i] = (float)(s >> 8) / 8388608.f - 1.f;
  }
  double* out = malloc(sizeof(double) * B * H * L * D);
  double* probs = malloc(sizeof(double) * L);
  double orow[D];
  int32_t per_head[2 * 16];
  for (int i = 0; i < 32; ++i) per_head[i] = i < 16 ? 0 : -1;
  const int64_t rows[3] = {0, 14, 29};
  for (int mode = 0; mode < 2; ++mode) {
    CHECK(lvo_attn(4, scales, radii, 0, mode, 0, 0, 4, q, k, v, 1, B, H, D, 0.3, 0, NULL, 0, B * H, out));
    CHECK(lvo_attn(4, scales, per_head, 1, mode, 1, 0, 4, q, k, v, 1, B, H, D, 0.3, 3, rows, 1, 3, out));
    CHECK(lvo_attn(4, scales, radii, 0, mode, 0, 3, 4, q, k, v, 1, B, H, D, 0.3, 0, NULL, 0, B * H, out));   /* a KV-cache step */
    CHECK(lvo_attn_probs(4, scales, radii, 0, mode, 0, 4, q, k, v, 1, B, H, D, 0.3, 3, 29, probs, orow));
    double sum = 0;
    for (int64_t t = 0; t < L; ++t) sum += probs[t];
    printf("probs sum mode %d: %.12f\n", mode, sum);
    CHECK(lvo_attn_qkv8(4, scales, radii, 0, mode, 0, 4, q, k, v, 1, B, H, D, 0.3, 8, 0, B * H, out));
  }
  const uint8_t share[8] = {1, 0, 1, 0, 0, 1, 0, 1};
  CHECK(lvo_cfg_share(4, scales, 0, 4, share, B, H, D, out));
  int32_t* codes = malloc(sizeof(int32_t) * B * H * L * D);
  double* sc = malloc(sizeof(double) * B * H * L);
  double* zp = malloc(sizeof(double) * B * H * L);
  CHECK(lvo_quantize_rows(q, 1, B * H * L, D, 8, codes, sc, zp));
  CHECK(lvo_dequantize_rows(codes, sc, zp, B * H * L, D, out));
  double* map = calloc((size_t)(L * L), sizeof *map);
  for (int64_t i = 0; i < L; ++i) for (int64_t t = 0; t <= i; ++t) map[i * L + t] = 1.0 / (double)(i + 1);
  int32_t rad[16];
  double mass[16 * 4];
  CHECK(lvo_calibrate(4, scales, map, 1, 1, 0.9, rad, mass, 4));
  printf("calibrated radius of the last part: %d\n", rad[15]);
  free(mask); free(cnt); free(rowptr); free(q); free(k); free(v); free(out); free(probs); free(codes); free(sc); free(zp); free(map);
  return 0;
}
