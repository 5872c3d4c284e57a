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

/*
 * Offline 8-bit quantiser for expert blobs that travel over the host link in fp8 (OCP e4m3:
 * 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, largest finite value 448, no infinities).
 * Input preparation only: per row, scale = max|w| / 448 (1 for an all-zero row) and each weight
 * becomes the e4m3 code nearest to w / scale (ties to the even code, saturating at +-448).
 * w_bf16 [rows, cols] bf16 bits -> scales [rows] fp32, q [rows, cols] bytes.
 */
static inline float bf16_to_float(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

static inline float e4m3_value(int code) { /* code 0..126: the non-negative finite values, ascending */
  int e = code >> 3, m = code & 7;
  return e == 0 ? ldexpf((float)m, -9) : ldexpf(1.0f + (float)m / 8.0f, e - 7);
}

static inline uint8_t e4m3_nearest(float x) {
  uint8_t sign = x < 0.0f ? 0x80 : 0;
  float a = fabsf(x);
  if (!(a < 448.0f)) return (uint8_t)(sign | 0x7E);
  int lo = 0, hi = 126; /* largest code with value <= a */
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (e4m3_value(mid) <= a) lo = mid; else hi = mid - 1;
  }
  int code = lo;
  if (lo < 126) {
    float dl = a - e4m3_value(lo), dh = e4m3_value(lo + 1) - a;
    if (dh < dl || (dh == dl && (lo & 1))) code = lo + 1;
  }
  return (uint8_t)(sign | code);
}

void synth_quantize_e4m3_rows(const uint16_t *w_bf16, int64_t rows, int64_t cols, float *scales, uint8_t *q) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    const uint16_t *w = w_bf16 + r * cols;
    float amax = 0.0f;
    for (int64_t c = 0; c < cols; ++c) {
      float a = fabsf(bf16_to_float(w[c]));
      if (a > amax) amax = a;
    }
    float scale = amax > 0.0f ? amax / 448.0f : 1.0f;
    scales[r] = scale;
    for (int64_t c = 0; c < cols; ++c) q[r * cols + c] = e4m3_nearest(bf16_to_float(w[c]) / scale);
  }
}

/*
 * Offline 4-bit quantiser: unsigned 4-bit integers in groups of 128 along a row, one fp32 scale and
 * one zero point (0..15) per group, the storage form of AWQ / GPTQ-style weight quantisation
 * (input preparation only).  Per group: scale = (max - min) / 15 (1 if the group is constant),
 * zero = round(-min / scale) clamped to 0..15, code = round(w / scale) + zero clamped to 0..15;
 * min and max include 0 so that a zero weight is representable.  Two codes per byte, the even
 * column in the low nibble.  cols % 128 == 0.
 * w_bf16 [rows, cols] -> scales [rows, cols/128] fp32, zeros [rows, cols/128] bytes, codes [rows, cols/2] bytes.
 */
void synth_quantize_int4_g128(const uint16_t *w_bf16, int64_t rows, int64_t cols, float *scales, uint8_t *zeros,
                              uint8_t *codes) {
  const int64_t groups = cols / 128;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t g = 0; g < groups; ++g) {
      const uint16_t *w = w_bf16 + r * cols + g * 128;
      float lo = 0.0f, hi = 0.0f;
      for (int i = 0; i < 128; ++i) {
        float v = bf16_to_float(w[i]);
        if (v < lo) lo = v;
        if (v > hi) hi = v;
      }
      float scale = hi > lo ? (hi - lo) / 15.0f : 1.0f;
      float zf = nearbyintf(-lo / scale);
      int zero = zf < 0.0f ? 0 : (zf > 15.0f ? 15 : (int)zf);
      scales[r * groups + g] = scale;
      zeros[r * groups + g] = (uint8_t)zero;
      for (int i = 0; i < 128; i += 2) {
        int q[2];
        for (int j = 0; j < 2; ++j) {
          float t = nearbyintf(bf16_to_float(w[i + j]) / scale) + (float)zero;
          q[j] = t < 0.0f ? 0 : (t > 15.0f ? 15 : (int)t);
        }
        codes[(r * cols + g * 128 + i) / 2] = (uint8_t)(q[0] | (q[1] << 4));
      }
    }
}

/*
 * Offline quantiser to the OCP microscaling format MXFP4 (input preparation only): blocks of 32
 * values along a row share one scale 2^(s - 127) (s = one byte, E8M0), each value is an e2m1 code
 * (1 sign, 2 exponent, 1 mantissa bit: 0, 0.5, 1, 1.5, 2, 3, 4, 6).  Per block: s - 127 =
 * floor(log2(max|w|)) - 2 (the largest e2m1 exponent), clamped to [-126, 127]; an all-zero block gets
 * s = 127; each value is rounded to the nearest code (ties to the even code), saturating at +-6.
 * Two codes per byte, the even column in the low nibble.  cols % 32 == 0.
 * w_bf16 [rows, cols] -> scales [rows, cols/32] bytes, codes [rows, cols/2] bytes.
 */
static const float kE2M1[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

static inline uint8_t e2m1_nearest(float x) {
  uint8_t sign = x < 0.0f ? 8 : 0;
  float a = fabsf(x);
  int best = 0;
  for (int c = 1; c < 8; ++c) {
    float db = fabsf(a - kE2M1[best]), dc = fabsf(a - kE2M1[c]);
    if (dc < db || (dc == db && !(c & 1))) best = c;
  }
  return (uint8_t)(sign | best);
}

void synth_quantize_mxfp4(const uint16_t *w_bf16, int64_t rows, int64_t cols, uint8_t *scales, uint8_t *codes) {
  const int64_t blocks = cols / 32;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t b = 0; b < blocks; ++b) {
      const uint16_t *w = w_bf16 + r * cols + b * 32;
      float amax = 0.0f;
      for (int i = 0; i < 32; ++i) {
        float a = fabsf(bf16_to_float(w[i]));
        if (a > amax) amax = a;
      }
      int e = 0;
      if (amax > 0.0f) {
        (void)frexpf(amax, &e);   /* amax = m * 2^e, m in [0.5, 1): floor(log2(amax)) = e - 1 */
        e = e - 1 - 2;
        if (e < -126) e = -126;
        if (e > 127) e = 127;
      }
      scales[r * blocks + b] = (uint8_t)(e + 127);
      const float inv = ldexpf(1.0f, -e);
      for (int i = 0; i < 32; i += 2) {
        uint8_t lo = e2m1_nearest(bf16_to_float(w[i]) * inv), hi = e2m1_nearest(bf16_to_float(w[i + 1]) * inv);
        codes[(r * cols + b * 32 + i) / 2] = (uint8_t)(lo | (hi << 4));
      }
    }
}
