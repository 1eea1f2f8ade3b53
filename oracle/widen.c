/*
 * C helpers of the CPU oracle (test infrastructure, not product code).
 *
 *  - oracle_widen_bf16_f64: widen bf16 bit patterns to fp64.  A bf16 value is the
 *    upper 16 bits of an IEEE fp32, so the conversion is exact.
 *  - oracle_linear_bf16w: y[t][n] = sum_k x[t][k] * W[n][k] with W stored as bf16 bit
 *    patterns, every product and the whole sum in fp64.  Each output is the plain dot
 *    product of one input row with one widened weight row; four weight rows are kept
 *    widened at a time only so that an input row is read once for four outputs.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline double bf16_to_f64(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

void oracle_widen_bf16_f64(const uint16_t *src, double *dst, int64_t n) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) dst[i] = bf16_to_f64(src[i]);
}

#define ROWS 4

void oracle_linear_bf16w(const double *x, int64_t T, int64_t Kd, const uint16_t *W, int64_t N,
                         double *y /* [T][N] */) {
#pragma omp parallel
  {
    double *w = (double *)malloc(sizeof(double) * ROWS * Kd);
#pragma omp for schedule(static)
    for (int64_t n0 = 0; n0 < N; n0 += ROWS) {
      const int64_t nr = N - n0 < ROWS ? N - n0 : ROWS;
      for (int64_t r = 0; r < ROWS; ++r)
        for (int64_t k = 0; k < Kd; ++k) w[r * Kd + k] = r < nr ? bf16_to_f64(W[(n0 + r) * Kd + k]) : 0.0;
      const double *w0 = w, *w1 = w + Kd, *w2 = w + 2 * Kd, *w3 = w + 3 * Kd;
      for (int64_t t = 0; t < T; ++t) {
        const double *xt = x + t * Kd;
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma omp simd reduction(+ : a0, a1, a2, a3)
        for (int64_t k = 0; k < Kd; ++k) {
          a0 += xt[k] * w0[k];
          a1 += xt[k] * w1[k];
          a2 += xt[k] * w2[k];
          a3 += xt[k] * w3[k];
        }
        const double a[ROWS] = {a0, a1, a2, a3};
        for (int64_t r = 0; r < nr; ++r) y[t * N + n0 + r] = a[r];
      }
    }
    free(w);
  }
}
