/* Seeded synthetic-input generator (counter based, thread-count independent).
 *
 * Holds no arithmetic of the verifier: it only fills buffers with pseudo-random
 * numbers.  Element i of a stream is a pure function of (seed, stream, i), so the
 * output does not depend on the number of OpenMP threads or on the chunking.
 *
 * normal_bf16: pairs of N(0, std^2) variates by the Box-Muller transform of two
 * 24-bit uniforms taken from one 64-bit hash of the pair's counter, rounded to
 * bf16 (nearest, ties to even).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static inline uint16_t to_bf16(float f) {
  uint32_t b;
  memcpy(&b, &f, 4);
  b += 0x7FFFu + ((b >> 16) & 1u);
  return (uint16_t)(b >> 16);
}

void llm42_synth_normal_bf16(uint64_t seed, uint64_t stream, uint64_t n, float std, uint16_t* out) {
  const uint64_t key = mix64(seed ^ mix64(stream));
  const uint64_t pairs = (n + 1) / 2;
  const float two_pi = 6.28318530717958647692f;
#pragma omp parallel for schedule(static)
  for (uint64_t p = 0; p < pairs; ++p) {
    const uint64_t h = mix64(key + p);
    const float u1 = ((float)(h >> 40) + 0.5f) * (1.0f / 16777216.0f);
    const float u2 = ((float)(h & 0xFFFFFFull) + 0.5f) * (1.0f / 16777216.0f);
    const float r = sqrtf(-2.0f * logf(u1)) * std;
    const float a = two_pi * u2;
    out[2 * p] = to_bf16(r * cosf(a));
    if (2 * p + 1 < n) out[2 * p + 1] = to_bf16(r * sinf(a));
  }
}

/* Uniform integers in [0, bound) (bound < 2^31), one per counter. */
void llm42_synth_uniform_i32(uint64_t seed, uint64_t stream, uint64_t n, int32_t bound, int32_t* out) {
  const uint64_t key = mix64(seed ^ mix64(stream));
#pragma omp parallel for schedule(static)
  for (uint64_t i = 0; i < n; ++i) {
    const uint64_t h = mix64(key + i);
    out[i] = (int32_t)(((h >> 32) * (uint64_t)bound) >> 32);
  }
}
