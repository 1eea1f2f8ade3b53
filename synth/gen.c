/*
 * Seeded, counter-based synthetic input generator (host side).
 *
 * Every element of every tensor is a pure function of (seed, stream id, element
 * index), so any slice can be regenerated on its own and in parallel.  This file
 * holds no arithmetic of the verify step itself: it only draws random numbers and
 * stores them in the formats the inputs are defined in (bf16 bit patterns, fp32,
 * int32).  Both the CPU oracle's tests and the GPU path's tests feed from it.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

/* 64 random bits for (seed, stream, counter). */
static inline uint64_t draw64(uint64_t seed, uint64_t stream, uint64_t ctr) {
  uint64_t k = mix64(seed ^ mix64(stream));
  return mix64(k + ctr * 0xD1342543DE82EF95ull);
}

/* uniform in (0,1): 53 random bits, never 0 */
static inline double u01(uint64_t bits) {
  return ((double)(bits >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

/* Standard normal for element i: elements 2p and 2p+1 share one Box-Muller pair. */
static inline double normal_at(uint64_t seed, uint64_t stream, uint64_t i) {
  uint64_t p = i >> 1;
  double u1 = u01(draw64(seed, stream, 2 * p));
  double u2 = u01(draw64(seed, stream, 2 * p + 1));
  double r = sqrt(-2.0 * log(u1));
  double a = 6.283185307179586476925286766559 * u2;
  return (i & 1) ? r * sin(a) : r * cos(a);
}

/* round-to-nearest-even fp32 -> bf16 bit pattern (inputs here are finite) */
static inline uint16_t f32_to_bf16_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

void synth_normal_f64(uint64_t seed, uint64_t stream, uint64_t first, uint64_t n,
                      double mean, double std, double *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    out[i] = mean + std * normal_at(seed, stream, first + (uint64_t)i);
}

void synth_normal_f32(uint64_t seed, uint64_t stream, uint64_t first, uint64_t n,
                      double mean, double std, float *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    out[i] = (float)(mean + std * normal_at(seed, stream, first + (uint64_t)i));
}

/* N(mean, std) rounded once to bf16; the bit patterns are the tensor. */
void synth_normal_bf16(uint64_t seed, uint64_t stream, uint64_t first, uint64_t n,
                       double mean, double std, uint16_t *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    out[i] = f32_to_bf16_bits((float)(mean + std * normal_at(seed, stream, first + (uint64_t)i)));
}

/* integers uniform in [lo, hi) */
void synth_uniform_i32(uint64_t seed, uint64_t stream, uint64_t first, uint64_t n,
                       int32_t lo, int32_t hi, int32_t *out) {
  uint64_t span = (uint64_t)((int64_t)hi - (int64_t)lo);
  for (uint64_t i = 0; i < n; ++i) {
    uint64_t b = draw64(seed, stream, first + i);
    /* 64-bit multiply-high range reduction */
    out[i] = lo + (int32_t)(((__uint128_t)b * span) >> 64);
  }
}

/* uniform doubles in (0,1) */
void synth_uniform_f64(uint64_t seed, uint64_t stream, uint64_t first, uint64_t n, double *out) {
  for (uint64_t i = 0; i < n; ++i) out[i] = u01(draw64(seed, stream, first + i));
}
