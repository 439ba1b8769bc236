/*
 * Seeded synthetic-input generator (counter based, integer only).
 *
 * This file holds no arithmetic of the decoding method: it only turns
 * (key, index) into reproducible pseudo-random tensor values, token ids and
 * mask bits.  Both the CPU oracle's tests and the GPU harness fill their
 * buffers from here, so both sides see bit-identical inputs.
 *
 * Value n of a stream with 64-bit key K is derived from mix64(K + n), where
 * mix64 is the SplitMix64 output function (Steele, Lea, Flood 2014).
 *
 * "Normal" values: the eight bytes of the mixed word are summed (Irwin-Hall
 * with 8 terms, range 0..2040, mean 1020, variance 8*(256^2-1)/12), centred,
 * converted to float exactly and multiplied by one float constant so that the
 * standard deviation is `std`.  No libm call is involved, so every platform
 * produces the same bits.  bfloat16 output rounds that float to nearest-even
 * with integer operations.
 */
#include <stdint.h>
#include <stddef.h>

static inline uint64_t mix64(uint64_t x) {
  x += 0x9e3779b97f4a7c15ull;
  x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
  x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
  return x ^ (x >> 31);
}

uint64_t dgen_mix64(uint64_t x) { return mix64(x); }

static inline int32_t byte_sum(uint64_t z) {
  z = (z & 0x00ff00ff00ff00ffull) + ((z >> 8) & 0x00ff00ff00ff00ffull);
  z = (z & 0x0000ffff0000ffffull) + ((z >> 16) & 0x0000ffff0000ffffull);
  z = (z & 0x00000000ffffffffull) + (z >> 32);
  return (int32_t)z;
}

/* sqrt(8 * (256^2 - 1) / 12) */
#define DGEN_IH8_SIGMA 209.02152998196777

static inline float normal_value(uint64_t key, uint64_t n, float scale) {
  return (float)(byte_sum(mix64(key + n)) - 1020) * scale;
}

static inline uint16_t f32_to_bf16_rne(float f) {
  union { float f; uint32_t u; } v;
  v.f = f;
  uint32_t u = v.u;
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  return (uint16_t)(u >> 16);
}

void dgen_normal_f32(uint64_t key, uint64_t first, uint64_t count, double std, float* out) {
  const float scale = (float)(std / DGEN_IH8_SIGMA);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)count; ++i) out[i] = normal_value(key, first + (uint64_t)i, scale);
}

void dgen_normal_bf16(uint64_t key, uint64_t first, uint64_t count, double std, uint16_t* out) {
  const float scale = (float)(std / DGEN_IH8_SIGMA);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)count; ++i)
    out[i] = f32_to_bf16_rne(normal_value(key, first + (uint64_t)i, scale));
}

/* Uniform integers on [0, bound). */
void dgen_uniform_i32(uint64_t key, uint64_t first, uint64_t count, uint32_t bound, int32_t* out) {
  for (uint64_t i = 0; i < count; ++i) out[i] = (int32_t)(mix64(key + first + i) % bound);
}

/* Bernoulli(1/2) bits: bit 0 of the mixed word. */
void dgen_bits(uint64_t key, uint64_t first, uint64_t count, uint8_t* out) {
  for (uint64_t i = 0; i < count; ++i) out[i] = (uint8_t)(mix64(key + first + i) & 1u);
}
