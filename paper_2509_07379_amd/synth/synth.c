/*
 * Seeded synthetic-input generator (counter based, multi-threaded).
 *
 * This file holds no arithmetic of the MoE method: it only fills buffers with
 * Gaussian bf16 values so that the CPU oracle and the HIP path can be fed the
 * very same tensors.  Element i of a stream depends only on (seed, stream, i),
 * so any slice of a tensor can be regenerated on its own.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC synth.c -o libsynth.so -lm
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

static inline uint16_t f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u); /* round to nearest even; inputs are finite */
  return (uint16_t)(u >> 16);
}

/* Two standard normals for pair index p of the keyed stream (Box-Muller). */
static inline void normal_pair(uint64_t key, uint64_t p, float *z0, float *z1) {
  uint64_t r = mix64(key + p * 0xD1342543DE82EF95ull);
  float u1 = (float)((r >> 40) + 1) * (1.0f / 16777216.0f); /* (0,1] */
  float u2 = (float)((r >> 8) & 0xFFFFFFu) * (1.0f / 16777216.0f);
  float rad = sqrtf(-2.0f * logf(u1));
  float ang = 6.28318530717958647692f * u2;
  *z0 = rad * cosf(ang);
  *z1 = rad * sinf(ang);
}

/* out[i] = bf16(sigma * N(0,1)) for i in [first, first+n) of stream (seed, stream). */
void synth_normal_bf16(uint64_t seed, uint64_t stream, int64_t first, int64_t n,
                       float sigma, uint16_t *out) {
  const uint64_t key = mix64(mix64(seed) ^ (stream * 0xA24BAED4963EE407ull));
  const int64_t last = first + n;
  const int64_t p0 = first >> 1, p1 = (last + 1) >> 1;
#pragma omp parallel for schedule(static)
  for (int64_t p = p0; p < p1; ++p) {
    float z0, z1;
    normal_pair(key, (uint64_t)p, &z0, &z1);
    int64_t i0 = 2 * p, i1 = 2 * p + 1;
    if (i0 >= first && i0 < last) out[i0 - first] = f32_to_bf16(sigma * z0);
    if (i1 >= first && i1 < last) out[i1 - first] = f32_to_bf16(sigma * z1);
  }
}

/* Same stream as fp32 (no bf16 rounding), for biases and the like. */
void synth_normal_f32(uint64_t seed, uint64_t stream, int64_t first, int64_t n,
                      float sigma, float *out) {
  const uint64_t key = mix64(mix64(seed) ^ (stream * 0xA24BAED4963EE407ull));
  const int64_t last = first + n;
  const int64_t p0 = first >> 1, p1 = (last + 1) >> 1;
#pragma omp parallel for schedule(static)
  for (int64_t p = p0; p < p1; ++p) {
    float z0, z1;
    normal_pair(key, (uint64_t)p, &z0, &z1);
    int64_t i0 = 2 * p, i1 = 2 * p + 1;
    if (i0 >= first && i0 < last) out[i0 - first] = sigma * z0;
    if (i1 >= first && i1 < last) out[i1 - first] = sigma * z1;
  }
}
