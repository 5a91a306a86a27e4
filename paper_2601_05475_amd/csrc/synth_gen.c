/*
 * Seeded synthetic-input generator (host only, plain C + OpenMP).
 *
 * Every value is a pure function of (seed, stream, flat index), so arrays can be
 * produced in any order, in parallel, and in pieces.  The generator holds none of
 * the transformer's arithmetic: it only fills buffers with
 *   - normal deviates (mean, std) as fp32 or as bf16 bit patterns,
 *   - token ids uniform in [0, vocab),
 *   - uniforms in [0, 1) with 24 random bits (exactly representable in fp32).
 *
 * Counter-based construction: the 64-bit finaliser of SplitMix64 (Steele, Lea,
 * Flood 2014) applied to   key(seed, stream) + index * golden-ratio increment.
 * Normals come from one 64-bit draw per element by the Box-Muller transform in
 * double precision (u1 from the high 32 bits, u2 from the low 32 bits).
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

static inline uint64_t sm64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

static inline uint64_t stream_key(uint64_t seed, uint64_t stream) {
  return sm64(sm64(seed) ^ (stream * 0xD1B54A32D192ED03ull));
}

static inline uint64_t draw(uint64_t key, uint64_t idx) {
  return sm64(key + idx * 0x9E3779B97F4A7C15ull);
}

static inline double normal_from_bits(uint64_t r) {
  const double two_m32 = 1.0 / 4294967296.0;
  double u1 = ((double)(r >> 32) + 1.0) * two_m32;       /* (0, 1] */
  double u2 = (double)(r & 0xFFFFFFFFull) * two_m32;     /* [0, 1) */
  return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
}

/* round-to-nearest-even fp32 -> bf16 bit pattern (inputs here are always finite) */
static inline uint16_t f32_to_bf16_bits(float f) {
  union { float f; uint32_t u; } v;
  v.f = f;
  uint32_t lsb = (v.u >> 16) & 1u;
  return (uint16_t)((v.u + 0x7FFFu + lsb) >> 16);
}

void synth_normal_f32(uint64_t seed, uint64_t stream, uint64_t first, size_t n,
                      double mean, double std, float *out) {
  const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i)
    out[i] = (float)(mean + std * normal_from_bits(draw(key, first + i)));
}

void synth_normal_bf16(uint64_t seed, uint64_t stream, uint64_t first, size_t n,
                       double mean, double std, uint16_t *out) {
  const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i)
    out[i] = f32_to_bf16_bits((float)(mean + std * normal_from_bits(draw(key, first + i))));
}

void synth_tokens(uint64_t seed, uint64_t stream, uint64_t first, size_t n,
                  int32_t vocab, int32_t *out) {
  const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i)
    out[i] = (int32_t)(draw(key, first + i) % (uint64_t)vocab);
}

void synth_uniform_f32(uint64_t seed, uint64_t stream, uint64_t first, size_t n,
                       float *out) {
  const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i)
    out[i] = (float)(draw(key, first + i) >> 40) * (1.0f / 16777216.0f);
}
