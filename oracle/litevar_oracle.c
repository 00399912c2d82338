/*
 * litevar_oracle.c -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * Plain, slow, fp64 CPU statement of LiteVAR's multi-diagonal windowed
 * attention (MDWA) with the optional CFG shared-output step (ASC).  Only the
 * test-suite, the smoke check and the benchmark's cpu_baseline leg may call
 * it.  It shares no code, header, table or helper with the HIP library.
 *
 * Everything here is written as the definition: a predicate allowed(q, t)
 * evaluated for every key t, a max-subtracted softmax over the allowed keys,
 * and a weighted sum of V rows.  No window tables, no tiling, no fusion.
 *
 * What the paper fixes (Section 2, "Multi-Diagonal Window Attention"):
 *   - K scales, scale k holds s_k^2 tokens; a query of scale k sees the
 *     tokens of scales 1..k (block-causal; same-scale tokens are mutually
 *     visible).  Worked shape: k = 2 gives a [4, 5] attention map.
 *   - the map is cut into per-key-scale parts and a local window of some
 *     width is kept inside each part; a threshold of 1 means full attention.
 *   - Section 2, "MDWA implementation details": the leading parts stay dense
 *     (attention sinks) -> parameter n_sink.
 *   - Section 3 (ASC): the unconditional branch reuses the conditional
 *     branch's attention output.
 * What the paper leaves open and the reading taken here:
 *   - window geometry: a square (Chebyshev) window of radius r_j around the
 *     query's position mapped into key scale j's s_j x s_j grid;
 *   - position map: centre = floor((2c+1) s_j / (2 s_k)) per axis (integer);
 *   - tokens of a scale are stored row-major (y major, x minor);
 *   - masking happens before the softmax, so kept weights renormalise to 1;
 *   - CFG layout: batch rows [0, B/2) conditional, b + B/2 the partner.
 * A second reading of the window, mode LVO_BAND (Section 2, step (2), taken
 * literally): the attention map of query scale k, [s_k^2, sum_{i<=k} s_i^2], is
 * cut into parts -- the first spans the first three key scales (those of them the
 * query sees), every later key scale is a part -- and in a part of n columns the
 * query with flattened index i keeps the columns within radius r of the part's
 * diagonal, floor((2i+1) n / (2 s_k^2)).  The radius of a part is the table entry
 * of its last key scale; a part whose last key scale is below n_sink stays dense.
 * Section 2, step (3) determines the window size for each scale, part and head:
 * the attention functions take one radius table per head when asked to.
 *
 * Parity pins live in tests/ (golden worked example, closed-form pair
 * counts, brute force in numpy, reduction to dense scaled-dot-product
 * attention, softmax invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define LVO_OK 0
#define LVO_BAD_ARG (-1)
#define LVO_NO_MEM (-2)
#define LVO_CAP (-3)

enum { LVO_F64 = 0, LVO_F32 = 1, LVO_BF16 = 2 };
enum { LVO_WINDOW = 0, LVO_BAND = 1 };

/* ---- geometry (Section 2: scale k has s_k^2 tokens) -------------------- */

int64_t lvo_seq_len(int32_t K, const int32_t* scales) {
  int64_t L = 0;
  for (int32_t k = 0; k < K; ++k) L += (int64_t)scales[k] * scales[k];
  return L;
}

/* first token of scale k in the flattened sequence */
int64_t lvo_scale_offset(int32_t K, const int32_t* scales, int32_t k) {
  int64_t o = 0;
  for (int32_t i = 0; i < k && i < K; ++i) o += (int64_t)scales[i] * scales[i];
  return o;
}

/* token t -> (scale, row, col); row-major inside the scale */
int lvo_token_coords(int32_t K, const int32_t* scales, int64_t t,
                     int32_t* k_out, int32_t* y_out, int32_t* x_out) {
  if (t < 0) return LVO_BAD_ARG;
  int64_t o = 0;
  for (int32_t k = 0; k < K; ++k) {
    int64_t n = (int64_t)scales[k] * scales[k];
    if (t < o + n) {
      int64_t local = t - o;
      *k_out = k;
      *y_out = (int32_t)(local / scales[k]);
      *x_out = (int32_t)(local % scales[k]);
      return LVO_OK;
    }
    o += n;
  }
  return LVO_BAD_ARG;
}

/* The predicate, on coordinates.  radii is a [K][K] table: radii[k*K + j] is the
 * radius of part j of query scale k's attention map (Section 2, step (3): the
 * window size is determined for each scale and part); < 0 means "no window in
 * that part". */
/* The band reading (LVO_BAND): parts, and a band around each part's diagonal. */
static int allowed_band(int32_t K, const int32_t* scales, const int32_t* radii,
                        int32_t n_sink, int32_t qk, int32_t qy, int32_t qx,
                        int32_t kj, int32_t ky, int32_t kx) {
  if (kj > qk) return 0;                 /* block-causal across scales */
  /* the part that key scale kj belongs to: key scales [first, last] */
  int32_t first = kj < 3 ? 0 : kj;
  int32_t last = kj < 3 ? (qk < 2 ? qk : 2) : kj;
  if (last < n_sink) return 1;           /* leading parts kept dense */
  int32_t r = radii[(int64_t)qk * K + last];
  if (r < 0) return 1;                   /* dense part */
  int64_t n = 0, col = 0;                /* columns of the part; this key's column in it */
  for (int32_t i = first; i <= last; ++i) {
    if (i < kj) col += (int64_t)scales[i] * scales[i];
    n += (int64_t)scales[i] * scales[i];
  }
  col += (int64_t)ky * scales[kj] + kx;
  int64_t nk = (int64_t)scales[qk] * scales[qk];
  int64_t i = (int64_t)qy * scales[qk] + qx;
  int64_t c = ((2 * i + 1) * n) / (2 * nk);     /* the part's diagonal at row i */
  int64_t d = col - c;
  if (d < 0) d = -d;
  return d <= r;
}

static int allowed_window(int32_t K, const int32_t* scales, const int32_t* radii,
                          int32_t n_sink, int32_t qk, int32_t qy, int32_t qx,
                          int32_t kj, int32_t ky, int32_t kx);

static int allowed_coords(int32_t K, const int32_t* scales, const int32_t* radii,
                          int32_t n_sink, int32_t mode, int32_t qk, int32_t qy, int32_t qx,
                          int32_t kj, int32_t ky, int32_t kx) {
  if (mode == LVO_BAND) return allowed_band(K, scales, radii, n_sink, qk, qy, qx, kj, ky, kx);
  return allowed_window(K, scales, radii, n_sink, qk, qy, qx, kj, ky, kx);
}

static int allowed_window(int32_t K, const int32_t* scales, const int32_t* radii,
                          int32_t n_sink, int32_t qk, int32_t qy, int32_t qx,
                          int32_t kj, int32_t ky, int32_t kx) {
  if (kj > qk) return 0;                 /* block-causal across scales */
  if (kj < n_sink) return 1;             /* leading parts kept dense */
  int32_t r = radii[(int64_t)qk * K + kj];
  if (r < 0) return 1;                   /* dense part */
  int64_t sj = scales[kj], sk = scales[qk];
  int64_t cy = ((2 * (int64_t)qy + 1) * sj) / (2 * sk);
  int64_t cx = ((2 * (int64_t)qx + 1) * sj) / (2 * sk);
  int64_t dy = (int64_t)ky - cy, dx = (int64_t)kx - cx;
  if (dy < 0) dy = -dy;
  if (dx < 0) dx = -dx;
  return dy <= r && dx <= r;
}

/* allowed(q, t) on flattened token indices of the full sequence */
int lvo_allowed(int32_t K, const int32_t* scales, const int32_t* radii,
                int32_t n_sink, int32_t mode, int64_t tq, int64_t tk) {
  int32_t qk, qy, qx, kj, ky, kx;
  if (lvo_token_coords(K, scales, tq, &qk, &qy, &qx) != LVO_OK) return LVO_BAD_ARG;
  if (lvo_token_coords(K, scales, tk, &kj, &ky, &kx) != LVO_OK) return LVO_BAD_ARG;
  return allowed_coords(K, scales, radii, n_sink, mode, qk, qy, qx, kj, ky, kx);
}

typedef struct { int32_t k, y, x; } coord_t;

static coord_t* coord_table(int32_t K, const int32_t* scales, int64_t L) {
  coord_t* c = (coord_t*)malloc((size_t)(L > 0 ? L : 1) * sizeof(coord_t));
  if (!c) return NULL;
  for (int64_t t = 0; t < L; ++t)
    lvo_token_coords(K, scales, t, &c[t].k, &c[t].y, &c[t].x);
  return c;
}

static int check_desc(int32_t K, const int32_t* scales, const int32_t* radii,
                      int32_t n_sink, int32_t qb, int32_t qe) {
  if (K < 1 || !scales || !radii) return LVO_BAD_ARG;
  for (int32_t k = 0; k < K; ++k) if (scales[k] < 1) return LVO_BAD_ARG;
  if (n_sink < 0 || qb < 0 || qe > K || qb >= qe) return LVO_BAD_ARG;
  return LVO_OK;
}

/* ---- masks and index sets --------------------------------------------- */

/* dense byte mask [Lq][L]; rows are the queries of scales [qb, qe) */
int lvo_mask_dense(int32_t K, const int32_t* scales, const int32_t* radii, int32_t mode,
                   int32_t n_sink, int32_t qb, int32_t qe, uint8_t* mask) {
  if (check_desc(K, scales, radii, n_sink, qb, qe) || !mask) return LVO_BAD_ARG;
  int64_t L = lvo_seq_len(K, scales);
  int64_t q0 = lvo_scale_offset(K, scales, qb), q1 = lvo_scale_offset(K, scales, qe);
  coord_t* c = coord_table(K, scales, L);
  if (!c) return LVO_NO_MEM;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t q = q0; q < q1; ++q)
    for (int64_t t = 0; t < L; ++t)
      mask[(q - q0) * L + t] = (uint8_t)allowed_coords(
          K, scales, radii, n_sink, mode, c[q].k, c[q].y, c[q].x, c[t].k, c[t].y, c[t].x);
  free(c);
  return LVO_OK;
}

/* per-query count of allowed keys: counts[Lq] */
int lvo_row_counts(int32_t K, const int32_t* scales, const int32_t* radii, int32_t mode,
                   int32_t n_sink, int32_t qb, int32_t qe, int64_t* counts) {
  if (check_desc(K, scales, radii, n_sink, qb, qe) || !counts) return LVO_BAD_ARG;
  int64_t L = lvo_seq_len(K, scales);
  int64_t q0 = lvo_scale_offset(K, scales, qb), q1 = lvo_scale_offset(K, scales, qe);
  coord_t* c = coord_table(K, scales, L);
  if (!c) return LVO_NO_MEM;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t q = q0; q < q1; ++q) {
    int64_t n = 0;
    for (int64_t t = 0; t < L; ++t)
      n += allowed_coords(K, scales, radii, n_sink, mode, c[q].k, c[q].y, c[q].x,
                          c[t].k, c[t].y, c[t].x);
    counts[q - q0] = n;
  }
  free(c);
  return LVO_OK;
}

/* ascending index sets in CSR form: rowptr[Lq+1] (caller-filled from
 * lvo_row_counts by prefix sum), cols[rowptr[Lq]] */
int lvo_index_sets(int32_t K, const int32_t* scales, const int32_t* radii, int32_t mode,
                   int32_t n_sink, int32_t qb, int32_t qe,
                   const int64_t* rowptr, int32_t* cols, int64_t cols_cap) {
  if (check_desc(K, scales, radii, n_sink, qb, qe) || !rowptr || !cols) return LVO_BAD_ARG;
  int64_t L = lvo_seq_len(K, scales);
  int64_t q0 = lvo_scale_offset(K, scales, qb), q1 = lvo_scale_offset(K, scales, qe);
  if (rowptr[q1 - q0] > cols_cap) return LVO_CAP;
  coord_t* c = coord_table(K, scales, L);
  if (!c) return LVO_NO_MEM;
  int bad = 0;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t q = q0; q < q1; ++q) {
    int64_t w = rowptr[q - q0];
    for (int64_t t = 0; t < L; ++t)
      if (allowed_coords(K, scales, radii, n_sink, mode, c[q].k, c[q].y, c[q].x,
                         c[t].k, c[t].y, c[t].x)) {
        if (w < rowptr[q - q0 + 1]) cols[w] = (int32_t)t;
        ++w;
      }
    if (w != rowptr[q - q0 + 1]) {
#pragma omp atomic write
      bad = 1;
    }
  }
  free(c);
  return bad ? LVO_BAD_ARG : LVO_OK;
}

/* ---- attention --------------------------------------------------------- */

static double load_elem(const void* p, int32_t dtype, int64_t i) {
  if (dtype == LVO_F64) return ((const double*)p)[i];
  if (dtype == LVO_F32) return (double)((const float*)p)[i];
  /* bf16: the upper half of an IEEE binary32 */
  uint32_t bits = (uint32_t)((const uint16_t*)p)[i] << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

/*
 * One softmax row, the textbook way: scores over allowed keys, subtract the
 * maximum, exponentiate, normalise, weight V.  probs (optional, length L)
 * receives the normalised weights, 0 for masked keys.
 */
static int attn_row(int32_t K, const int32_t* scales, const int32_t* radii, int32_t n_sink,
                    int32_t mode, const coord_t* c, int64_t L, int64_t tq,
                    const double* qrow, const double* Kd, const double* Vd,
                    int32_t D, double sm_scale, double* z, double* out, double* probs) {
  double m = -INFINITY;
  for (int64_t t = 0; t < L; ++t) {
    if (!allowed_coords(K, scales, radii, n_sink, mode, c[tq].k, c[tq].y, c[tq].x,
                        c[t].k, c[t].y, c[t].x)) { z[t] = NAN; continue; }
    double s = 0.0;
    for (int32_t d = 0; d < D; ++d) s += qrow[d] * Kd[t * D + d];
    z[t] = sm_scale * s;
    if (z[t] > m) m = z[t];
  }
  double denom = 0.0;
  for (int64_t t = 0; t < L; ++t)
    if (!isnan(z[t])) { z[t] = exp(z[t] - m); denom += z[t]; }
  for (int32_t d = 0; d < D; ++d) out[d] = 0.0;
  for (int64_t t = 0; t < L; ++t) {
    double p = isnan(z[t]) ? 0.0 : z[t] / denom;
    if (probs) probs[t] = p;
    if (p != 0.0)
      for (int32_t d = 0; d < D; ++d) out[d] += p * Vd[t * D + d];
  }
  return LVO_OK;
}

/*
 * q: [B,H,Lq,D], k,v: [B,H,L,D] packed, element type `dtype`;
 * rows: optional list of n_rows query indices local to [0, Lq) (NULL = all);
 * out: [B,H,n_rows,D] fp64.  bh_begin/bh_end restrict the (b*H+h) range
 * (used to time or check a sample); rows outside it are left untouched.
 * mode: LVO_WINDOW or LVO_BAND.  radii: one [K][K] table, or, when radii_per_head is
 * non-zero, one per head, [H][K][K].
 */
int lvo_attn(int32_t K, const int32_t* scales, const int32_t* radii, int32_t n_sink,
             int32_t mode, int32_t radii_per_head,
             int32_t qb, int32_t qe, const void* q, const void* k, const void* v,
             int32_t dtype, int32_t B, int32_t H, int32_t D, double sm_scale,
             int64_t n_rows, const int64_t* rows, int64_t bh_begin, int64_t bh_end,
             double* out) {
  if (check_desc(K, scales, radii, n_sink, qb, qe)) return LVO_BAD_ARG;
  if (!q || !k || !v || !out || B < 1 || H < 1 || D < 1) return LVO_BAD_ARG;
  if (dtype != LVO_F64 && dtype != LVO_F32 && dtype != LVO_BF16) return LVO_BAD_ARG;
  int64_t L = lvo_seq_len(K, scales);
  int64_t q0 = lvo_scale_offset(K, scales, qb), q1 = lvo_scale_offset(K, scales, qe);
  int64_t Lq = q1 - q0;
  if (!rows) n_rows = Lq;
  if (n_rows < 0) return LVO_BAD_ARG;
  if (rows) for (int64_t i = 0; i < n_rows; ++i)
    if (rows[i] < 0 || rows[i] >= Lq) return LVO_BAD_ARG;
  if (bh_begin < 0 || bh_end > (int64_t)B * H || bh_begin > bh_end) return LVO_BAD_ARG;
  coord_t* c = coord_table(K, scales, L);
  if (!c) return LVO_NO_MEM;
  int err = 0;
#pragma omp parallel
  {
    double* Kd = (double*)malloc((size_t)L * D * sizeof(double));
    double* Vd = (double*)malloc((size_t)L * D * sizeof(double));
    double* z = (double*)malloc((size_t)L * sizeof(double));
    double* qrow = (double*)malloc((size_t)D * sizeof(double));
    if (!Kd || !Vd || !z || !qrow) {
#pragma omp atomic write
      err = 1;
    }
#pragma omp barrier
    if (!err) {
#pragma omp for schedule(dynamic, 1)
      for (int64_t bh = bh_begin; bh < bh_end; ++bh) {
        for (int64_t i = 0; i < L * D; ++i) {
          Kd[i] = load_elem(k, dtype, bh * L * D + i);
          Vd[i] = load_elem(v, dtype, bh * L * D + i);
        }
        for (int64_t r = 0; r < n_rows; ++r) {
          int64_t ql = rows ? rows[r] : r;
          for (int32_t d = 0; d < D; ++d)
            qrow[d] = load_elem(q, dtype, (bh * Lq + ql) * D + d);
          /* Section 2, step (3): head h may have a radius table of its own, [H][K][K] */
          const int32_t* rad_h = radii_per_head ? radii + (bh % H) * (int64_t)K * K : radii;
          attn_row(K, scales, rad_h, n_sink, mode, c, L, q0 + ql, qrow, Kd, Vd, D, sm_scale,
                   z, out + (bh * n_rows + r) * D, NULL);
        }
      }
    }
    free(Kd); free(Vd); free(z); free(qrow);
  }
  free(c);
  return err ? LVO_NO_MEM : LVO_OK;
}

/* normalised weights of one (b,h,query) over all L keys: probs[L] fp64 */
int lvo_attn_probs(int32_t K, const int32_t* scales, const int32_t* radii, int32_t n_sink,
                   int32_t mode, int32_t qb, int32_t qe, const void* q, const void* k, const void* v,
                   int32_t dtype, int32_t B, int32_t H, int32_t D, double sm_scale,
                   int64_t bh, int64_t ql, double* probs, double* out_row) {
  if (check_desc(K, scales, radii, n_sink, qb, qe)) return LVO_BAD_ARG;
  if (!q || !k || !v || !probs || !out_row) return LVO_BAD_ARG;
  int64_t L = lvo_seq_len(K, scales);
  int64_t q0 = lvo_scale_offset(K, scales, qb), q1 = lvo_scale_offset(K, scales, qe);
  int64_t Lq = q1 - q0;
  if (bh < 0 || bh >= (int64_t)B * H || ql < 0 || ql >= Lq) return LVO_BAD_ARG;
  coord_t* c = coord_table(K, scales, L);
  double* Kd = (double*)malloc((size_t)L * D * sizeof(double));
  double* Vd = (double*)malloc((size_t)L * D * sizeof(double));
  double* z = (double*)malloc((size_t)L * sizeof(double));
  double* qrow = (double*)malloc((size_t)D * sizeof(double));
  int rc = LVO_NO_MEM;
  if (c && Kd && Vd && z && qrow) {
    for (int64_t i = 0; i < L * D; ++i) {
      Kd[i] = load_elem(k, dtype, bh * L * D + i);
      Vd[i] = load_elem(v, dtype, bh * L * D + i);
    }
    for (int32_t d = 0; d < D; ++d) qrow[d] = load_elem(q, dtype, (bh * Lq + ql) * D + d);
    rc = attn_row(K, scales, radii, n_sink, mode, c, L, q0 + ql, qrow, Kd, Vd, D, sm_scale,
                  z, out_row, probs);
  }
  free(c); free(Kd); free(Vd); free(z); free(qrow);
  return rc;
}

/*
 * ASC (Section 3): for every (head h, query scale k) with share[h*K + k] != 0
 * the unconditional row b + B/2 takes the conditional row b's output.
 * o: [B,H,Lq,D] fp64, modified in place; Lq spans query scales [qb, qe).
 */
int lvo_cfg_share(int32_t K, const int32_t* scales, int32_t qb, int32_t qe,
                  const uint8_t* share, int32_t B, int32_t H, int32_t D, double* o) {
  if (K < 1 || !scales || qb < 0 || qe > K || qb >= qe || !share || !o) return LVO_BAD_ARG;
  if (B < 2 || (B & 1)) return LVO_BAD_ARG;
  int64_t q0 = lvo_scale_offset(K, scales, qb), q1 = lvo_scale_offset(K, scales, qe);
  int64_t Lq = q1 - q0;
  int32_t half = B / 2;
  for (int32_t b = 0; b < half; ++b)
    for (int32_t h = 0; h < H; ++h)
      for (int32_t kq = qb; kq < qe; ++kq) {
        if (!share[(int64_t)h * K + kq]) continue;
        int64_t a = lvo_scale_offset(K, scales, kq) - q0;
        int64_t n = (int64_t)scales[kq] * scales[kq];
        double* src = o + (((int64_t)b * H + h) * Lq + a) * D;
        double* dst = o + (((int64_t)(b + half) * H + h) * Lq + a) * D;
        memcpy(dst, src, (size_t)(n * D) * sizeof(double));
      }
  return LVO_OK;
}

/* ---- window calibration (Section 2: the metric R_w and the threshold R_0) ----
 *
 * For every head, query scale k and part j <= k of a post-softmax attention
 * map: R_w = (sum of the map's values inside the window) / (sum of all values
 * of the part); the window grows from zero until R_w reaches R_0.  The map
 * p[N][H][L][L] holds N reference samples; reading taken here: their values
 * are summed (one window per head, scale and part for the whole reference
 * set), a part is one key scale, and "window size zero" is radius 0, the
 * centre key alone (the same square window and centre map as above).
 *
 * radius[h][k][j] = smallest r >= 0 with R_w >= R_0 (0 for a part without
 * mass; entries with j > k are set to -1).  mass[h][k][j][r], optional, is
 * the in-window sum at radius r for r < smax (the whole part's sum once the
 * window covers the part). */
int lvo_calibrate(int32_t K, const int32_t* scales, const double* p, int32_t N, int32_t H,
                  double r0, int32_t* radius, double* mass, int32_t smax) {
  if (K < 1 || !scales || !p || !radius || N < 1 || H < 1) return LVO_BAD_ARG;
  for (int32_t k = 0; k < K; ++k) if (scales[k] < 1 || scales[k] > smax) return LVO_BAD_ARG;
  const int64_t L = lvo_seq_len(K, scales);
  int32_t* rad = (int32_t*)malloc((size_t)K * K * sizeof(int32_t));
  if (!rad) return LVO_NO_MEM;
  for (int32_t h = 0; h < H; ++h)
    for (int32_t k = 0; k < K; ++k)
      for (int32_t j = 0; j < K; ++j) {
        int32_t* out = radius + ((int64_t)h * K + k) * K + j;
        double* mout = mass ? mass + (((int64_t)h * K + k) * K + j) * smax : NULL;
        if (mout) for (int32_t r = 0; r < smax; ++r) mout[r] = 0.0;
        if (j > k) { *out = -1; continue; }
        const int64_t oq = lvo_scale_offset(K, scales, k), ok = lvo_scale_offset(K, scales, j);
        const int32_t sk = scales[k], sj = scales[j];
        int32_t found = -1;
        for (int32_t r = 0; r < smax; ++r) {          /* the window grows from zero */
          for (int32_t i = 0; i < K * K; ++i) rad[i] = r;
          double in = 0.0, all = 0.0;
          for (int32_t n = 0; n < N; ++n)
            for (int32_t qy = 0; qy < sk; ++qy)
              for (int32_t qx = 0; qx < sk; ++qx)
                for (int32_t ky = 0; ky < sj; ++ky)
                  for (int32_t kx = 0; kx < sj; ++kx) {
                    const int64_t q = oq + (int64_t)qy * sk + qx, t = ok + (int64_t)ky * sj + kx;
                    const double v = p[(((int64_t)n * H + h) * L + q) * L + t];
                    all += v;
                    if (allowed_coords(K, scales, rad, 0, LVO_WINDOW, k, qy, qx, j, ky, kx)) in += v;
                  }
          if (mout) mout[r] = in;
          if (found < 0 && (all == 0.0 || in / all >= r0)) found = r;
          if (found >= 0 && !mout) break;
        }
        *out = found < 0 ? sj - 1 : found;
      }
  free(rad);
  return LVO_OK;
}

/* The same procedure with Section 2, step (2) read literally (LVO_BAND): the map of query
 * scale k is cut into parts -- the first three key scales together, then one part per key
 * scale -- and the window of a part is the band of radius r around the part's diagonal; for
 * each part the band grows from radius zero until it holds the fraction r0 of the part's
 * values (n - 1 at the latest, n = the part's columns).  radius[h][k][j] receives the radius of
 * the part that key scale j belongs to (the same value for every key scale of the merged
 * part; -1 for j > k), i.e. a table that the band predicate reads back.  mass[h][k][j][r],
 * optional, r < mcols: the in-band sum at radius r (the part's sum from r = n - 1 on). */
int lvo_calibrate_band(int32_t K, const int32_t* scales, const double* p, int32_t N, int32_t H,
                       double r0, int32_t* radius, double* mass, int32_t mcols) {
  if (K < 1 || !scales || !p || !radius || N < 1 || H < 1) return LVO_BAD_ARG;
  const int64_t L = lvo_seq_len(K, scales);
  int32_t* rad = (int32_t*)malloc((size_t)K * K * sizeof(int32_t));
  if (!rad) return LVO_NO_MEM;
  for (int32_t h = 0; h < H; ++h)
    for (int32_t k = 0; k < K; ++k) {
      for (int32_t j = 0; j < K; ++j) {
        radius[((int64_t)h * K + k) * K + j] = -1;
        if (mass) for (int32_t r = 0; r < mcols; ++r) mass[(((int64_t)h * K + k) * K + j) * mcols + r] = 0.0;
      }
      const int64_t oq = lvo_scale_offset(K, scales, k);
      const int32_t sk = scales[k];
      int32_t first = 0;
      while (first <= k) {
        const int32_t last = first < 3 ? (k < 2 ? k : 2) : first;   /* key scales of this part */
        int64_t n = 0;
        for (int32_t j = first; j <= last; ++j) n += (int64_t)scales[j] * scales[j];
        if (mass && n > mcols) { free(rad); return LVO_BAD_ARG; }
        int32_t found = -1;
        for (int64_t r = 0; r < n; ++r) {              /* the band grows from zero */
          for (int32_t i = 0; i < K * K; ++i) rad[i] = (int32_t)r;
          double in = 0.0, all = 0.0;
          for (int32_t s = 0; s < N; ++s)
            for (int32_t qy = 0; qy < sk; ++qy)
              for (int32_t qx = 0; qx < sk; ++qx)
                for (int32_t j = first; j <= last; ++j)
                  for (int32_t ky = 0; ky < scales[j]; ++ky)
                    for (int32_t kx = 0; kx < scales[j]; ++kx) {
                      const int64_t q = oq + (int64_t)qy * sk + qx;
                      const int64_t t = lvo_scale_offset(K, scales, j) + (int64_t)ky * scales[j] + kx;
                      const double v = p[(((int64_t)s * H + h) * L + q) * L + t];
                      all += v;
                      if (allowed_coords(K, scales, rad, 0, LVO_BAND, k, qy, qx, j, ky, kx)) in += v;
                    }
          if (mass)
            for (int32_t j = first; j <= last; ++j) {
              double* m = mass + (((int64_t)h * K + k) * K + j) * mcols;
              m[r] = in;
              if (r == n - 1) for (int64_t rr = n; rr < mcols; ++rr) m[rr] = in;
            }
          if (found < 0 && (all == 0.0 || in / all >= r0)) found = (int32_t)r;
          if (found >= 0 && !mass) break;
        }
        for (int32_t j = first; j <= last; ++j)
          radius[((int64_t)h * K + k) * K + j] = found < 0 ? (int32_t)(n - 1) : found;
        first = last + 1;
      }
    }
  free(rad);
  return LVO_OK;
}

/* ---- QKV8: attention on 8-bit Q, K, V (Section 4, "Quantization Scheme": min-max
 * quantisation with dynamic parameters computed online from the data's maximum and
 * minimum) ----
 *
 * The printed quantiser is x_q = round(clamp((x - z)/s, -2^(B-1), 2^(B-1))) with
 * z = (max + min)/2 and a scale "s = max(abs(x))" that lacks the integer range, and a clamp
 * whose upper bound is not a B-bit code.  Reading taken here (the usual min-max form with
 * the paper's zero point): z = (max + min)/2, s = ((max - min)/2) / (2^(B-1) - 1), codes
 * clamped to [-2^(B-1), 2^(B-1) - 1], rounding to nearest with ties to even; the
 * dequantised value is s x_q + z.  Granularity (the paper does not state one): one (s, z)
 * per token row of D values, computed from that row alone.  A constant row has s = 0: all
 * codes are 0 and the row dequantises to z exactly.
 *
 * A code is an integer decided by a floating-point comparison; the decision is taken in
 * binary32, in the order z = (max + min) * 0.5f, s = ((max - min) * 0.5f) / qmax,
 * t = (x - z) / s, nearest-even, so that an implementation in that precision can produce
 * the same codes bit for bit.  Everything after the codes is fp64. */
int lvo_quantize_rows(const void* x, int32_t dtype, int64_t rows, int32_t D, int32_t bits,
                      int32_t* codes, double* scale, double* zero) {
  if (!x || !codes || !scale || !zero || rows < 0 || D < 1 || bits < 2 || bits > 16) return LVO_BAD_ARG;
  if (dtype != LVO_F64 && dtype != LVO_F32 && dtype != LVO_BF16) return LVO_BAD_ARG;
  const float qmax = (float)((1 << (bits - 1)) - 1), qmin = -(float)(1 << (bits - 1));
  for (int64_t r = 0; r < rows; ++r) {
    float mx = -INFINITY, mn = INFINITY;
    for (int32_t d = 0; d < D; ++d) {
      const float v = (float)load_elem(x, dtype, r * D + d);
      if (v > mx) mx = v;
      if (v < mn) mn = v;
    }
    const float z = (mx + mn) * 0.5f;
    const float s = ((mx - mn) * 0.5f) / qmax;
    for (int32_t d = 0; d < D; ++d) {
      const float v = (float)load_elem(x, dtype, r * D + d);
      float t = 0.0f;
      if (s > 0.0f) {
        t = (v - z) / s;
        if (t < qmin) t = qmin;
        if (t > qmax) t = qmax;
        t = nearbyintf(t);               /* default rounding mode: nearest, ties to even */
      }
      codes[r * D + d] = (int32_t)t;
    }
    scale[r] = (double)s;
    zero[r] = (double)z;
  }
  return LVO_OK;
}

/* s x_q + z, in fp64 */
int lvo_dequantize_rows(const int32_t* codes, const double* scale, const double* zero,
                        int64_t rows, int32_t D, double* out) {
  if (!codes || !scale || !zero || !out || rows < 0 || D < 1) return LVO_BAD_ARG;
  for (int64_t r = 0; r < rows; ++r)
    for (int32_t d = 0; d < D; ++d) out[r * D + d] = scale[r] * (double)codes[r * D + d] + zero[r];
  return LVO_OK;
}

/* Windowed attention with Q, K and V quantised to `bits` bits per token row and
 * dequantised again (the arithmetic of the attention itself stays fp64): the result that an
 * 8-bit Q/K/V implementation approximates.  Arguments as lvo_attn. */
int lvo_attn_qkv8(int32_t K, const int32_t* scales, const int32_t* radii, int32_t n_sink,
                  int32_t mode, int32_t qb, int32_t qe, const void* q, const void* k, const void* v,
                  int32_t dtype, int32_t B, int32_t H, int32_t D, double sm_scale, int32_t bits,
                  int64_t bh_begin, int64_t bh_end, double* out) {
  if (check_desc(K, scales, radii, n_sink, qb, qe)) return LVO_BAD_ARG;
  if (!q || !k || !v || !out || B < 1 || H < 1 || D < 1) return LVO_BAD_ARG;
  const int64_t L = lvo_seq_len(K, scales);
  const int64_t Lq = lvo_scale_offset(K, scales, qe) - lvo_scale_offset(K, scales, qb);
  const int64_t nq = (int64_t)B * H * Lq, nk = (int64_t)B * H * L;
  int32_t* codes = (int32_t*)malloc((size_t)(nk > nq ? nk : nq) * D * sizeof(int32_t));
  double* sc = (double*)malloc((size_t)(nk > nq ? nk : nq) * sizeof(double));
  double* zp = (double*)malloc((size_t)(nk > nq ? nk : nq) * sizeof(double));
  double* qd = (double*)malloc((size_t)nq * D * sizeof(double));
  double* kd = (double*)malloc((size_t)nk * D * sizeof(double));
  double* vd = (double*)malloc((size_t)nk * D * sizeof(double));
  int rc = LVO_NO_MEM;
  if (codes && sc && zp && qd && kd && vd) {
    rc = lvo_quantize_rows(q, dtype, nq, D, bits, codes, sc, zp);
    if (!rc) rc = lvo_dequantize_rows(codes, sc, zp, nq, D, qd);
    if (!rc) rc = lvo_quantize_rows(k, dtype, nk, D, bits, codes, sc, zp);
    if (!rc) rc = lvo_dequantize_rows(codes, sc, zp, nk, D, kd);
    if (!rc) rc = lvo_quantize_rows(v, dtype, nk, D, bits, codes, sc, zp);
    if (!rc) rc = lvo_dequantize_rows(codes, sc, zp, nk, D, vd);
    if (!rc) rc = lvo_attn(K, scales, radii, n_sink, mode, 0, qb, qe, qd, kd, vd, LVO_F64, B, H, D, sm_scale,
                           0, NULL, bh_begin, bh_end, out);
  }
  free(codes); free(sc); free(zp); free(qd); free(kd); free(vd);
  return rc;
}

int lvo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
