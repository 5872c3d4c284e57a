/*
 * CPU oracle for one top-k Mixture-of-Experts FFN layer.  TEST INFRASTRUCTURE ONLY:
 * it is the parity reference for the HIP library and shares no code with it.  Only
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * The scheduling side of the method (prefetch, caching, prediction; Section V of the
 * paper) must never change the numbers (Section V-C has the verification step make sure that
 * the right experts' weights are the ones computed with), so the numerical oracle is the plain
 * definition of the layer:
 *   - a softmax gate whose values are non-negative and sum to 1 (Section II-A),
 *   - Top-k selection out of n routed experts (Section II-A, Fig. 1),
 *   - grouping the tokens by assigned expert (Section V-B),
 *   - each expert an FFN block (Section I), here SwiGLU without biases,
 *   - the output a weighted sum of the selected experts' outputs (Section II-A),
 *     with optional shared experts that contribute to every token (Fig. 1).
 *
 * Everything is scalar loops; dot products of the experts accumulate in fp64.  The
 * router logits are ALSO computed in fp32 in one fixed summation order, because the
 * Top-k decision is an integer result that both sides must take in the same
 * precision:
 *     element i of the dot product belongs to bin (i / 8) mod 64; each bin adds its
 *     products in ascending i (the bf16 x bf16 products are exact in fp32); the 64
 *     bins are then summed by a binary tree that pairs bins differing in bit 5,
 *     then bit 4, ... then bit 0; the bias, if any, is added last.
 *
 * bf16 values travel as uint16_t bit patterns.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC
 *            moe_oracle.c -o libmoe_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline float bf16_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* Round a double to the nearest bf16 (ties to even), without passing through fp32. */
static uint16_t bf16_from_f64(double v) {
  if (v != v) return 0x7FC0;
  double a = fabs(v);
  uint16_t sign = (uint16_t)(signbit(v) ? 0x8000 : 0);
  if (a == 0.0) return sign;
  if (isinf(a)) return (uint16_t)(sign | 0x7F80);
  int e = ilogb(a);
  if (e < -126) e = -126;              /* subnormal range shares the smallest exponent */
  double q = rint(ldexp(a, 7 - e));    /* 8 significant bits, ties to even */
  float f = (float)ldexp(q, e - 7);    /* exact in fp32 (may have carried to 2^(e+1)) */
  if (isinf(f)) return (uint16_t)(sign | 0x7F80);
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)(sign | (u >> 16));
}

uint16_t ref_bf16_from_f64(double v) { return bf16_from_f64(v); }

/* fp32 dot product in the fixed order described in the header. */
static float dot_fixed_order(const uint16_t *x, const uint16_t *w, int d) {
  float bin[64];
  for (int b = 0; b < 64; ++b) bin[b] = 0.0f;
  for (int i = 0; i < d; ++i) {
    int b = (i >> 3) & 63;
    float prod = bf16_f32(x[i]) * bf16_f32(w[i]);
    bin[b] = bin[b] + prod;
  }
  for (int m = 32; m >= 1; m >>= 1)
    for (int b = 0; b < 64; ++b)
      if ((b & m) == 0) bin[b] = bin[b] + bin[b | m];
  return bin[0];
}

/*
 * Gate scores (Section II-A): logit[t,e] = sum_i x[t,i] * Wr[e,i] (+ bias).
 * bias may be NULL; otherwise bias[t*bias_stride + e] (stride 0 = one row for all tokens).
 * logits32: fixed-order fp32 (used for selection); logits64 (may be NULL): fp64 value.
 */
void ref_router_logits(const uint16_t *x, const uint16_t *wr, const float *bias, int bias_stride,
                       int T, int d, int E, float *logits32, double *logits64) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    for (int e = 0; e < E; ++e) {
      const uint16_t *xr = x + (size_t)t * d, *wrow = wr + (size_t)e * d;
      float acc = dot_fixed_order(xr, wrow, d);
      if (bias) acc = acc + bias[(size_t)t * bias_stride + e];
      logits32[(size_t)t * E + e] = acc;
      if (logits64) {
        double s = 0.0;
        for (int i = 0; i < d; ++i) s += (double)bf16_f32(xr[i]) * (double)bf16_f32(wrow[i]);
        if (bias) s += (double)bias[(size_t)t * bias_stride + e];
        logits64[(size_t)t * E + e] = s;
      }
    }
  }
}

/*
 * Top-k of n experts per token (Section II-A).  Order: logit descending, ties to the
 * lower expert index; ids[t,0] is the top-1.  Gate values: softmax restricted to the
 * selected experts (renorm != 0) or softmax over all E experts (renorm == 0); both are
 * non-negative, and the renormalised ones sum to 1.
 */
void ref_topk_weights(const float *logits, int T, int E, int k, int renorm, int32_t *ids, float *w) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    const float *l = logits + (size_t)t * E;
    int32_t *id = ids + (size_t)t * k;
    for (int j = 0; j < k; ++j) {
      int best = -1;
      for (int e = 0; e < E; ++e) {
        int taken = 0;
        for (int q = 0; q < j; ++q) taken |= (id[q] == e);
        if (taken) continue;
        if (best < 0 || l[e] > l[best]) best = e; /* strict > keeps the lower index on ties */
      }
      id[j] = best;
    }
    double lmax = (double)l[id[0]];
    double den = 0.0;
    if (renorm) {
      for (int j = 0; j < k; ++j) den += exp((double)l[id[j]] - lmax);
    } else {
      for (int e = 0; e < E; ++e) den += exp((double)l[e] - lmax);
    }
    for (int j = 0; j < k; ++j) w[(size_t)t * k + j] = (float)(exp((double)l[id[j]] - lmax) / den);
  }
}

/*
 * Group the T*k (token, choice) assignments by expert (Section V-B).  Assignment
 * a = t*k + j.  Stable: within one expert the assignments keep ascending a.
 * perm[p] = a for sorted position p; inv_perm[a] = p; offsets = exclusive scan of counts.
 */
void ref_dispatch(const int32_t *ids, int T, int k, int E, int32_t *counts, int32_t *offsets,
                  int32_t *perm, int32_t *inv_perm) {
  int n = T * k;
  for (int e = 0; e < E; ++e) counts[e] = 0;
  for (int a = 0; a < n; ++a) counts[ids[a]]++;
  offsets[0] = 0;
  for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
  int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
  for (int e = 0; e < E; ++e) cursor[e] = offsets[e];
  for (int a = 0; a < n; ++a) {
    int p = cursor[ids[a]]++;
    perm[p] = a;
    inv_perm[a] = p;
  }
  free(cursor);
}

/*
 * One SwiGLU expert on one token: y = W_down * bf16( silu(W_gate x) * (W_up x) ).
 * blob = [W_gate (I x d); W_up (I x d); W_down (d x I)] row-major bf16.
 * The intermediate h is rounded to bf16 (it is a bf16 tensor in a bf16 model);
 * y stays fp64.  h_scratch holds I doubles.
 */
static void expert_ffn(const uint16_t *x, const uint16_t *blob, int d, int I, double *h_scratch,
                       double *y) {
  const uint16_t *wg = blob, *wu = blob + (size_t)I * d, *wd = blob + (size_t)2 * I * d;
  for (int n = 0; n < I; ++n) {
    double g = 0.0, u = 0.0;
    const uint16_t *gr = wg + (size_t)n * d, *ur = wu + (size_t)n * d;
    for (int i = 0; i < d; ++i) {
      double xi = (double)bf16_f32(x[i]);
      g += xi * (double)bf16_f32(gr[i]);
      u += xi * (double)bf16_f32(ur[i]);
    }
    double h = g / (1.0 + exp(-g)) * u;
    h_scratch[n] = (double)bf16_f32(bf16_from_f64(h));
  }
  for (int c = 0; c < d; ++c) {
    const uint16_t *dr = wd + (size_t)c * I;
    double s = 0.0;
    for (int n = 0; n < I; ++n) s += h_scratch[n] * (double)bf16_f32(dr[n]);
    y[c] = s;
  }
}

void ref_expert_ffn(const uint16_t *x, const uint16_t *blob, int d, int I, double *y) {
  double *h = (double *)malloc(sizeof(double) * (size_t)I);
  expert_ffn(x, blob, d, I, h, y);
  free(h);
}

/*
 * Layer output for the selected tokens sel[0..n_sel):
 *   out[t] = sum_{j=0..k-1} w[t,j] * expert_{ids[t,j]}(x[t])  (+ shared(x[t]) with weight 1),
 * j ascending, shared last (Section II-A: weighted sum; Fig. 1: shared experts are fused
 * into the final output).  blobs[e] points at expert e's blob; shared_blob (I_shared wide)
 * may be NULL.  out_bf16 [n_sel,d] is the bf16 result, out_f64 [n_sel,d] (may be NULL) the
 * value before that last rounding.
 */
void ref_moe_tokens(const uint16_t *x, int d, int I, int k, const uint16_t *const *blobs,
                    const uint16_t *shared_blob, int I_shared, const int32_t *ids, const float *w,
                    const int32_t *sel, int n_sel, uint16_t *out_bf16, double *out_f64) {
  int units = k + (shared_blob ? 1 : 0);
  double *ybuf = (double *)malloc(sizeof(double) * (size_t)n_sel * units * d);
#pragma omp parallel
  {
    int Imax = I > I_shared ? I : I_shared;
    double *h = (double *)malloc(sizeof(double) * (size_t)Imax);
#pragma omp for schedule(dynamic, 1)
    for (int q = 0; q < n_sel * units; ++q) {
      int s = q / units, j = q % units;
      int t = sel[s];
      const uint16_t *xr = x + (size_t)t * d;
      double *y = ybuf + (size_t)q * d;
      if (j < k)
        expert_ffn(xr, blobs[ids[(size_t)t * k + j]], d, I, h, y);
      else
        expert_ffn(xr, shared_blob, d, I_shared, h, y);
    }
    free(h);
  }
  for (int s = 0; s < n_sel; ++s) {
    int t = sel[s];
    for (int c = 0; c < d; ++c) {
      double acc = 0.0;
      for (int j = 0; j < k; ++j)
        acc += (double)w[(size_t)t * k + j] * ybuf[((size_t)s * units + j) * d + c];
      if (shared_blob) acc += ybuf[((size_t)s * units + k) * d + c];
      if (out_f64) out_f64[(size_t)s * d + c] = acc;
      out_bf16[(size_t)s * d + c] = bf16_from_f64(acc);
    }
  }
  free(ybuf);
}

/*
 * Stand-in predictor: a seeded linear scorer replaces the paper's ExpertMLP
 * (Section IV-B); score[e] = sum_t (x[t] . Wp[e]) with each dot product in the fixed
 * fp32 order and the tokens added in ascending t; the m best (score descending, lower
 * index on ties) are the experts to prefetch for the next layer (Section V-C).
 */
void ref_predictor_score(const uint16_t *x, const uint16_t *wp, int B, int d, int E, int m,
                         float *scores, int32_t *top) {
  for (int e = 0; e < E; ++e) {
    float s = 0.0f;
    for (int t = 0; t < B; ++t) s = s + dot_fixed_order(x + (size_t)t * d, wp + (size_t)e * d, d);
    scores[e] = s;
  }
  for (int j = 0; j < m; ++j) {
    int best = -1;
    for (int e = 0; e < E; ++e) {
      int taken = 0;
      for (int q = 0; q < j; ++q) taken |= (top[q] == e);
      if (taken) continue;
      if (best < 0 || scores[e] > scores[best]) best = e;
    }
    top[j] = best;
  }
}

/*
 * ExpertMLP forward pass (Section IV-B): n_fc fully connected layers; every layer but the last is
 * followed by batch normalisation (inference form: an affine map per neuron, scale and shift) and
 * ReLU (dropout is the identity at inference); the last one yields one logit per expert, whose
 * sigmoid is the predicted activation probability.  Weights W[l] are bf16 [dims[l+1], dims[l]],
 * bias / scale / shift fp32.
 *   logits64 (may be NULL): the definition in fp64.
 *   logits32 (may be NULL): fp32 in a fixed order, which decides the top-m: element i of a dot
 *   product belongs to bin i mod 64, each bin adds its products in ascending i with one fused
 *   multiply-add per element, the 64 bins are summed by the butterfly (bit 5 first), then
 *   z = acc + bias and, for a hidden layer, z = max(0, fma(z, scale, shift)).
 */
void ref_mlp_forward(const float *s, const int32_t *dims, int n_fc, const uint16_t *const *W,
                     const float *const *bias, const float *const *scale, const float *const *shift,
                     float *logits32, double *logits64) {
  int maxd = 0;
  for (int l = 0; l <= n_fc; ++l)
    if (dims[l] > maxd) maxd = dims[l];
  if (logits64) {
    double *a = (double *)malloc(sizeof(double) * (size_t)maxd), *b = (double *)malloc(sizeof(double) * (size_t)maxd);
    for (int i = 0; i < dims[0]; ++i) a[i] = (double)s[i];
    for (int l = 0; l < n_fc; ++l) {
      const int in = dims[l], out = dims[l + 1];
      for (int n = 0; n < out; ++n) {
        double acc = 0.0;
        for (int i = 0; i < in; ++i) acc += a[i] * (double)bf16_f32(W[l][(size_t)n * in + i]);
        acc += (double)bias[l][n];
        if (l + 1 < n_fc) {
          acc = acc * (double)scale[l][n] + (double)shift[l][n];
          if (acc < 0.0) acc = 0.0;
        }
        b[n] = acc;
      }
      double *t = a; a = b; b = t;
    }
    for (int n = 0; n < dims[n_fc]; ++n) logits64[n] = a[n];
    free(a); free(b);
  }
  if (logits32) {
    float *a = (float *)malloc(sizeof(float) * (size_t)maxd), *b = (float *)malloc(sizeof(float) * (size_t)maxd);
    for (int i = 0; i < dims[0]; ++i) a[i] = s[i];
    for (int l = 0; l < n_fc; ++l) {
      const int in = dims[l], out = dims[l + 1];
      for (int n = 0; n < out; ++n) {
        float bin[64];
        for (int q = 0; q < 64; ++q) bin[q] = 0.0f;
        for (int i = 0; i < in; ++i) bin[i & 63] = fmaf(a[i], bf16_f32(W[l][(size_t)n * in + i]), bin[i & 63]);
        for (int m = 32; m >= 1; m >>= 1)
          for (int q = 0; q < 64; ++q)
            if ((q & m) == 0) bin[q] = bin[q] + bin[q | m];
        float z = bin[0] + bias[l][n];
        if (l + 1 < n_fc) {
          z = fmaf(z, scale[l][n], shift[l][n]);
          if (!(z > 0.0f)) z = 0.0f;
        }
        b[n] = z;
      }
      float *t = a; a = b; b = t;
    }
    for (int n = 0; n < dims[n_fc]; ++n) logits32[n] = a[n];
    free(a); free(b);
  }
}

/*
 * Expert weights that travel over the host link as 8-bit floats (the paper evaluates quantised
 * models, Section VI; the format here is this build's reading: OCP e4m3 codes with one fp32 scale
 * per output row).  A weight is  bf16_rne( fp32( value(code) * scale ) ):  the code's value is exact
 * in fp32, the product is rounded once to fp32 and once more to bf16, in that order.
 *   value(code): sign s, exponent field e (4 bits, bias 7), mantissa field m (3 bits):
 *     e > 0: (-1)^s * 2^(e-7) * (1 + m/8);   e = 0: (-1)^s * 2^-6 * (m/8);   e = 15, m = 7: NaN.
 */
float ref_e4m3_value(int code) {
  int s = (code >> 7) & 1, e = (code >> 3) & 15, m = code & 7;
  double v;
  if (e == 15 && m == 7) return NAN;
  if (e == 0) v = ldexp((double)m / 8.0, -6);
  else v = ldexp(1.0 + (double)m / 8.0, e - 7);
  return (float)(s ? -v : v);
}

void ref_dequant_e4m3_rows(const uint8_t *q, const float *scales, int64_t rows, int64_t cols, uint16_t *out_bf16) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      float prod = ref_e4m3_value(q[r * cols + c]) * scales[r];
      out_bf16[r * cols + c] = bf16_from_f64((double)prod);
    }
}

/*
 * 4-bit expert weights on the host link (Section VI serves quantised models; the format is this
 * build's reading: unsigned 4-bit integers, groups of 128 along a row, one fp32 scale and one zero
 * point per group).  A weight is  bf16_rne( fp32( (code - zero) * scale ) ):  the integer difference
 * (-15..15) is exact in fp32, the product is rounded once to fp32 and once more to bf16.
 * codes: two per byte, the even column in the low nibble.  cols % 128 == 0.
 */
void ref_dequant_int4_g128_rows(const uint8_t *codes, const float *scales, const uint8_t *zeros, int64_t rows,
                                int64_t cols, uint16_t *out_bf16) {
  const int64_t groups = cols / 128;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      const uint8_t byte = codes[(r * cols + c) / 2];
      const int code = (c & 1) ? (byte >> 4) : (byte & 15);
      const int64_t g = r * groups + c / 128;
      const float prod = (float)(code - (int)zeros[g]) * scales[g];
      out_bf16[r * cols + c] = bf16_from_f64((double)prod);
    }
}

/*
 * MXFP4 expert weights (OCP microscaling formats: 32 consecutive values of a row share the scale
 * 2^(s - 127), s one byte; each value is an e2m1 code: bit 3 sign, bits 2..1 exponent e, bit 0
 * mantissa m; e = 0: m / 2;  e > 0: 2^(e - 1) * (1 + m / 2)  ->  0, 0.5, 1, 1.5, 2, 3, 4, 6).
 * A weight is value(code) * 2^(s - 127): one mantissa bit times a power of two, exact in bf16, so
 * the expansion involves no rounding (1 <= s <= 254 here).  Two codes per byte, even column low.
 */
double ref_e2m1_value(int code) {
  int s = (code >> 3) & 1, e = (code >> 1) & 3, m = code & 1;
  double v = e == 0 ? 0.5 * m : ldexp(1.0 + 0.5 * m, e - 1);
  return s ? -v : v;
}

void ref_dequant_mxfp4_rows(const uint8_t *codes, const uint8_t *scales, int64_t rows, int64_t cols,
                            uint16_t *out_bf16) {
  const int64_t blocks = cols / 32;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      const uint8_t byte = codes[(r * cols + c) / 2];
      const int code = (c & 1) ? (byte >> 4) : (byte & 15);
      const int s = scales[r * blocks + c / 32];
      out_bf16[r * cols + c] = bf16_from_f64(ldexp(ref_e2m1_value(code), s - 127));
    }
}
