/*
 * CPU oracle helper (test infrastructure, not product code): widen bf16 bit
 * patterns to fp64.  A bf16 value is the upper 16 bits of an IEEE fp32, so the
 * conversion is exact.
 */
#include <stdint.h>
#include <string.h>

void oracle_widen_bf16_f64(const uint16_t *src, double *dst, int64_t n) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint32_t u = (uint32_t)src[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    dst[i] = (double)f;
  }
}
