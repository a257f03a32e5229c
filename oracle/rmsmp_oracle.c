/*
 * RMSMP CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the RMSMP inference
 * hot path computes (row-wise mixed-scheme / multi-precision quantized GEMM,
 * ICCV'21 "RMSMP", arXiv 2111.00153).  It exists so that the HIP library can be
 * checked against something that was written from the paper alone.  It shares
 * no source, header, table or helper with the HIP library, and nothing on the
 * product path may call it: only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg do.
 *
 * Conventions
 *   W      M x K weight matrix, one row per filter (Section 3.1, Fig. 1).
 *   scheme one code per row: 0 = Fixed-4, 1 = PoT-4, 2 = Fixed-8
 *          (the three candidates of Section 3.2 / Fig. 2).
 *   alpha  one scaling factor per row (Eq. 1, Eq. 3).
 *   wint   the integer the level is written as: level = rowscale * wint.
 *   xq     activation codes, logically K x N, stored [N][K] (K contiguous),
 *          real value s_x * (code - z).
 *
 * Every loop is the textbook loop; there is no blocking, no SIMD, no
 * reordering.  OpenMP only distributes independent output rows.
 *
 * Parity pins (tests/test_oracle_*.py) cover every function in this file;
 * nothing here is "parity unpinned".
 *
 * Build: gcc -O2 -fno-fast-math -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define SCHEME_FIXED4 0
#define SCHEME_POT4 1
#define SCHEME_FIXED8 2

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* ------------------------------------------------------------------ */
/* Quantizers (Section 3.1.1, 3.1.2)                                   */
/* ------------------------------------------------------------------ */

/* Clip of Section 3.1.1 (the unnumbered equation after Eq. 2): w/alpha
 * limited to [-1, +1].  One fp32 divide. */
static float clip_unit(float w, float alpha) {
  if (w < -alpha) return -1.0f;
  if (w > alpha) return 1.0f;
  return w / alpha;
}

/* Number of positive levels of the m-bit Fixed set of Eq. 1:
 * {0, 1/(2^(m-1)-1), ..., 1} has 2^(m-1)-1 steps. */
static int fixed_steps(int m) { return (1 << (m - 1)) - 1; }

/* Fixed-point quantizer: projection of w onto Eq. 1's level set.
 * Eq. 1 is the authority for the set; Eq. 2's recipe (shift to [0,1], round on
 * a uniform grid, shift back) is followed with the grid that actually produces
 * Eq. 1's set, i.e. round(Q * clip(w/alpha)) with Q = 2^(m-1)-1.
 * round = round-half-to-even.  Returns the integer q in [-Q, Q]. */
int oracle_fixed_code(float w, float alpha, int m) {
  const int Q = fixed_steps(m);
  float x = clip_unit(w, alpha);
  float t = x * (float)Q;
  return (int)rintf(t);
}

/* PoT quantizer: projection onto Eq. 3's set {0, +-alpha*2^-k, k=0..2^(m-1)-2}
 * for m = 4 (k = 0..6).  Eq. 4's recipe -- round the base-2 logarithm -- is
 * applied to the magnitude of the clipped weight; magnitudes at or below half
 * of the smallest level (2^-7) go to zero, larger ones are clamped into the
 * exponent range.  Returns the signed integer sign * 2^(6-k) (so the level is
 * alpha * 2^-6 * wint), and 0 for the zero level. */
int oracle_pot4_int(float w, float alpha) {
  float x = clip_unit(w, alpha);
  float a = fabsf(x);
  if (!(a > 0.0078125f)) return 0; /* a <= 2^-7 */
  int ex;
  float f = frexpf(a, &ex); /* a = f * 2^ex, f in [0.5, 1) */
  int e = ex - 1;           /* a = (2f) * 2^e, 2f in [1, 2) */
  double g = 2.0 * (double)f;
  /* round(log2 a) = e + 1 iff log2(2f) > 1/2 iff (2f)^2 > 2; exact in double */
  if (g * g > 2.0) e += 1;
  if (e > 0) e = 0;
  if (e < -6) e = -6;
  int mag = 1 << (6 + e);
  return (x < 0.0f) ? -mag : mag;
}

/* max_k |w[k]|, the per-row scaling factor used when none is supplied. */
float oracle_row_alpha(const float* w, int64_t K) {
  float a = 0.0f;
  for (int64_t k = 0; k < K; ++k) {
    float v = fabsf(w[k]);
    if (v > a) a = v;
  }
  return a;
}

/* Vector forms of the two scalar quantizers, for dense sweeps in the tests. */
void oracle_fixed_codes(const float* w, int64_t n, float alpha, int m, int32_t* q) {
  for (int64_t i = 0; i < n; ++i) q[i] = oracle_fixed_code(w[i], alpha, m);
}
void oracle_pot4_ints(const float* w, int64_t n, float alpha, int32_t* q) {
  for (int64_t i = 0; i < n; ++i) q[i] = oracle_pot4_int(w[i], alpha);
}

/* Quantize every row of W with its own scheme and its own alpha.
 *   alpha_in  NULL -> alpha_r = max|w_r| (an all-zero row gets alpha 1).
 *   wint      M*K integers, level = rowscale[r] * wint
 *   rowscale  fp32: alpha/7 (Fixed-4), alpha/127 (Fixed-8), alpha*2^-6 (PoT-4)
 *   alpha_out the alpha actually used
 *   what      (nullable) M*K doubles, the quantized weights themselves:
 *             alpha*q/Q for Fixed rows, alpha*2^-k for PoT rows (Eq. 1, 3).
 * Returns 0, or -1 for an unknown scheme code / non-positive alpha. */
int oracle_quantize_rows(const float* W, int64_t M, int64_t K, const uint8_t* scheme,
                         const float* alpha_in, int32_t* wint, float* rowscale,
                         float* alpha_out, double* what) {
  for (int64_t r = 0; r < M; ++r) {
    const float* w = W + r * K;
    float alpha = alpha_in ? alpha_in[r] : oracle_row_alpha(w, K);
    if (!alpha_in && alpha == 0.0f) alpha = 1.0f;
    if (!(alpha > 0.0f)) return -1;
    alpha_out[r] = alpha;
    switch (scheme[r]) {
      case SCHEME_FIXED4:
      case SCHEME_FIXED8: {
        int m = scheme[r] == SCHEME_FIXED4 ? 4 : 8;
        int Q = fixed_steps(m);
        rowscale[r] = alpha / (float)Q;
        for (int64_t k = 0; k < K; ++k) {
          int q = oracle_fixed_code(w[k], alpha, m);
          wint[r * K + k] = q;
          if (what) what[r * K + k] = (double)alpha * (double)q / (double)Q;
        }
        break;
      }
      case SCHEME_POT4: {
        rowscale[r] = alpha * 0.015625f; /* alpha * 2^-6, exact */
        for (int64_t k = 0; k < K; ++k) {
          int q = oracle_pot4_int(w[k], alpha);
          wint[r * K + k] = q;
          if (what) what[r * K + k] = (double)alpha * (double)q / 64.0;
        }
        break;
      }
      default:
        return -1;
    }
  }
  return 0;
}

/* ------------------------------------------------------------------ */
/* Integer contraction (Alg. 1, forward line: out = proj(input).proj(W)) */
/* ------------------------------------------------------------------ */

/* acc[r][n] = sum_k wint[r][k] * xq[n][k].  Returns 0, or -2 if a partial
 * sum leaves the int32 range (the accumulator is checked in int64). */
int oracle_gemm_acc(const int32_t* wint, const int32_t* xq, int64_t M, int64_t K, int64_t N,
                    int32_t* acc) {
  int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
  for (int64_t r = 0; r < M; ++r) {
    for (int64_t n = 0; n < N; ++n) {
      int64_t s = 0;
      for (int64_t k = 0; k < K; ++k) {
        s += (int64_t)wint[r * K + k] * (int64_t)xq[n * K + k];
        if (s > INT32_MAX || s < INT32_MIN) bad = 1;
      }
      acc[r * N + n] = (int32_t)s;
    }
  }
  return bad ? -2 : 0;
}

/* The same sum for a PoT row written with shifts only: a weight +-2^(6-k)
 * times an activation code is the code shifted left by (6-k) bits, added or
 * subtracted (Section 2.1.2: the multiplication becomes a bit shift).
 * `scheme` selects the rows; other rows are left untouched in acc.
 * Negative activation codes are not accepted here (returns -3). */
int oracle_gemm_acc_pot_shift(const int32_t* wint, const uint8_t* scheme, const int32_t* xq,
                              int64_t M, int64_t K, int64_t N, int32_t* acc) {
  for (int64_t i = 0; i < N * K; ++i)
    if (xq[i] < 0) return -3;
  for (int64_t r = 0; r < M; ++r) {
    if (scheme[r] != SCHEME_POT4) continue;
    for (int64_t n = 0; n < N; ++n) {
      int64_t s = 0;
      for (int64_t k = 0; k < K; ++k) {
        int32_t w = wint[r * K + k];
        if (w == 0) continue;
        uint32_t mag = (uint32_t)(w < 0 ? -w : w);
        int sh = 0;
        while ((1u << sh) != mag) {
          ++sh;
          if (sh > 6) return -4; /* not a PoT integer */
        }
        int64_t term = (int64_t)((uint32_t)xq[n * K + k] << sh);
        s += (w < 0) ? -term : term;
      }
      acc[r * N + n] = (int32_t)s;
    }
  }
  return 0;
}

/* Row sums of the integer weights, needed when the activation code has a
 * zero point: sum_k w*(x - z) = sum_k w*x - z*sum_k w. */
void oracle_rowsum(const int32_t* wint, int64_t M, int64_t K, int32_t* rowsum) {
  for (int64_t r = 0; r < M; ++r) {
    int64_t s = 0;
    for (int64_t k = 0; k < K; ++k) s += wint[r * K + k];
    rowsum[r] = (int32_t)s;
  }
}

/* ------------------------------------------------------------------ */
/* Convolution, directly on the un-lowered tensors (Fig. 1: a filter of the
 * weight tensor is a row of the weight matrix).                        */
/* ------------------------------------------------------------------ */

typedef struct {
  int32_t B, C, H, W, KH, KW, stride, pad;
} oracle_conv_desc;

static int64_t conv_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad) {
  return (in + 2 * pad - k) / stride + 1;
}

int64_t oracle_conv_out_h(const oracle_conv_desc* d) { return conv_out_dim(d->H, d->KH, d->stride, d->pad); }
int64_t oracle_conv_out_w(const oracle_conv_desc* d) { return conv_out_dim(d->W, d->KW, d->stride, d->pad); }

/* One output value of the convolution: filter m at (b, oh, ow).
 *   wint [M][C][KH][KW]   x [B][H][W][C] codes   zpad = code written in the border
 * (a border pixel holds real value 0, i.e. code z). */
static int64_t conv_point(const int32_t* wint, const int32_t* x, const oracle_conv_desc* d,
                          int32_t zpad, int64_t m, int64_t b, int64_t oh, int64_t ow) {
  int64_t s = 0;
  for (int64_t c = 0; c < d->C; ++c)
    for (int64_t kh = 0; kh < d->KH; ++kh)
      for (int64_t kw = 0; kw < d->KW; ++kw) {
        int64_t ih = oh * d->stride - d->pad + kh;
        int64_t iw = ow * d->stride - d->pad + kw;
        int32_t xv = zpad;
        if (ih >= 0 && ih < d->H && iw >= 0 && iw < d->W)
          xv = x[((b * d->H + ih) * d->W + iw) * d->C + c];
        int32_t wv = wint[((m * d->C + c) * d->KH + kh) * d->KW + kw];
        s += (int64_t)wv * (int64_t)xv;
      }
  return s;
}

/* acc[m][(b*OH + oh)*OW + ow], every output. */
int oracle_conv_acc(const int32_t* wint, const int32_t* x, const oracle_conv_desc* d, int64_t M,
                    int32_t zpad, int32_t* acc) {
  const int64_t OH = oracle_conv_out_h(d), OW = oracle_conv_out_w(d);
  const int64_t N = (int64_t)d->B * OH * OW;
  int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t b = 0; b < d->B; ++b)
      for (int64_t oh = 0; oh < OH; ++oh)
        for (int64_t ow = 0; ow < OW; ++ow) {
          int64_t s = conv_point(wint, x, d, zpad, m, b, oh, ow);
          if (s > INT32_MAX || s < INT32_MIN) bad = 1;
          acc[m * N + (b * OH + oh) * OW + ow] = (int32_t)s;
        }
  return bad ? -2 : 0;
}

/* The same, at a list of (m, n) positions only (n = (b*OH+oh)*OW+ow): lets a
 * test sample a layer that is too large to compute in full. */
int oracle_conv_acc_at(const int32_t* wint, const int32_t* x, const oracle_conv_desc* d, int64_t M,
                       int32_t zpad, const int64_t* ms, const int64_t* ns, int64_t count,
                       int32_t* out) {
  const int64_t OH = oracle_conv_out_h(d), OW = oracle_conv_out_w(d);
  const int64_t N = (int64_t)d->B * OH * OW;
  int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
  for (int64_t i = 0; i < count; ++i) {
    int64_t m = ms[i], n = ns[i];
    if (m < 0 || m >= M || n < 0 || n >= N) {
      bad = 1;
      continue;
    }
    int64_t ow = n % OW, oh = (n / OW) % OH, b = n / (OW * OH);
    out[i] = (int32_t)conv_point(wint, x, d, zpad, m, b, oh, ow);
  }
  return bad ? -2 : 0;
}

/* GEMM at sampled positions, for the same purpose. */
int oracle_gemm_acc_at(const int32_t* wint, const int32_t* xq, int64_t M, int64_t K, int64_t N,
                       const int64_t* ms, const int64_t* ns, int64_t count, int32_t* out) {
  int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
  for (int64_t i = 0; i < count; ++i) {
    int64_t m = ms[i], n = ns[i];
    if (m < 0 || m >= M || n < 0 || n >= N) {
      bad = 1;
      continue;
    }
    int64_t s = 0;
    for (int64_t k = 0; k < K; ++k) s += (int64_t)wint[m * K + k] * (int64_t)xq[n * K + k];
    out[i] = (int32_t)s;
  }
  return bad ? -2 : 0;
}

/* ------------------------------------------------------------------ */
/* Epilogue: zero point, per-row scale, bias, ReLU, 4-bit re-quantization */
/* ------------------------------------------------------------------ */

/* For every (r, n), in fp32 with each operation rounded on its own:
 *   a  = acc - z * rowsum[r]                          (int32, exact)
 *   m  = rowscale[r] * s_x
 *   y  = (float)a * m ; y += bias[r] ; y = max(y, 0) when relu
 *   q  = clamp(rint(y * inv_s_out), 0, 15)            (round-half-to-even)
 * acc_corr, y, q are each optional (NULL to skip); q is one code per byte. */
void oracle_epilogue(const int32_t* acc, int64_t M, int64_t N, const int32_t* rowsum, int32_t z,
                     const float* rowscale, float s_x, const float* bias, int relu,
                     float inv_s_out, int32_t* acc_corr, float* y_out, uint8_t* q_out) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < M; ++r) {
    float m = rowscale[r] * s_x;
    for (int64_t n = 0; n < N; ++n) {
      int32_t a = acc[r * N + n] - z * rowsum[r];
      if (acc_corr) acc_corr[r * N + n] = a;
      float y = (float)a * m;
      if (bias) y = y + bias[r];
      if (relu) y = fmaxf(y, 0.0f);
      if (y_out) y_out[r * N + n] = y;
      if (q_out) {
        float t = y * inv_s_out;
        float c = rintf(t);
        c = fminf(fmaxf(c, 0.0f), 15.0f);
        q_out[r * N + n] = (uint8_t)c;
      }
    }
  }
}

/* GELU epilogue of the feed-forward up-projection of a transformer layer (the BERT-base
 * workload of Section 4.1 / Table 5; the paper names the model, not its activation quantizer):
 * the activation of BERT is GELU(y) = y * Phi(y), Phi the standard normal distribution
 * function, Phi(y) = (1 + erf(y / sqrt 2)) / 2 = erfc(-y / sqrt 2) / 2 (the second form keeps
 * its relative accuracy in the negative tail, where the first cancels), and its output -- signed, bounded below by about
 * -0.17 -- goes to the next layer as an unsigned 4-bit code with a zero point, the same
 * affine activation format the up-projection reads.
 *
 * oracle_gelu_f32: the definition, evaluated in float64 from the fp32 argument and rounded to
 * fp32 once. */
float oracle_gelu_f32(float y) {
  const double x = (double)y;
  return (float)(0.5 * x * erfc(-x / sqrt(2.0)));
}

/* For every (r, n), in fp32 with each operation rounded on its own:
 *   a = acc - z * rowsum[r] ; m = rowscale[r] * s_x ; y = (float)a * m ; y += bias[r]
 *   g = GELU(y)                                        (oracle_gelu_f32)
 *   q = clamp(rint(g * inv_s_out) + z_out, 0, 15)      (round-half-to-even)
 * g_out and q_out are each optional; q is one code per byte. */
void oracle_epilogue_gelu(const int32_t* acc, int64_t M, int64_t N, const int32_t* rowsum, int32_t z,
                          const float* rowscale, float s_x, const float* bias, float inv_s_out,
                          int32_t z_out, float* g_out, uint8_t* q_out) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < M; ++r) {
    float m = rowscale[r] * s_x;
    for (int64_t n = 0; n < N; ++n) {
      int32_t a = acc[r * N + n] - z * rowsum[r];
      float y = (float)a * m;
      if (bias) y = y + bias[r];
      float g = oracle_gelu_f32(y);
      if (g_out) g_out[r * N + n] = g;
      if (q_out) {
        float t = g * inv_s_out;
        float c = rintf(t) + (float)z_out;
        c = fminf(fmaxf(c, 0.0f), 15.0f);
        q_out[r * N + n] = (uint8_t)c;
      }
    }
  }
}

/* The same quantizer applied to a plain list of pre-activations y (no accumulator in front):
 * used to tabulate code(y) when thresholds are checked. */
void oracle_gelu_codes(const float* y, int64_t count, float inv_s_out, int32_t z_out, float* g_out,
                       uint8_t* q_out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    float g = oracle_gelu_f32(y[i]);
    if (g_out) g_out[i] = g;
    if (q_out) {
      float c = rintf(g * inv_s_out) + (float)z_out;
      c = fminf(fmaxf(c, 0.0f), 15.0f);
      q_out[i] = (uint8_t)c;
    }
  }
}

/* The plain definition in float64, with no integer factorisation at all:
 *   y64[r][n] = sum_k what[r][k] * ( s_x * (xq[n][k] - z) ) (+ bias, ReLU).
 * Used to check that the factorised fp32 epilogue stays within the stated
 * relative tolerance of the definition. */
void oracle_gemm_f64(const double* what, const int32_t* xq, int64_t M, int64_t K, int64_t N,
                     double s_x, int32_t z, const float* bias, int relu, double* y64) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < M; ++r)
    for (int64_t n = 0; n < N; ++n) {
      double s = 0.0;
      for (int64_t k = 0; k < K; ++k) s += what[r * K + k] * (s_x * (double)(xq[n * K + k] - z));
      if (bias) s += (double)bias[r];
      if (relu && s < 0.0) s = 0.0;
      y64[r * N + n] = s;
    }
}

/* ------------------------------------------------------------------ */
/* Row -> scheme assignment                                            */
/* ------------------------------------------------------------------ */

/* Row counts for a layer-uniform ratio PoT-4 : Fixed-4 : Fixed-8 = A : B : C
 * (A + B + C = 100, Section 4 / Alg. 1 input).  Fixed-8 takes round(M*C/100)
 * rows, at least one when C > 0; PoT-4 takes round(M*A/100); Fixed-4 the rest.
 * counts = {n_fixed4, n_pot4, n_fixed8}.  Returns -1 on a bad ratio. */
int oracle_ratio_counts(int64_t M, int pct_pot4, int pct_fixed4, int pct_fixed8, int64_t counts[3]) {
  if (pct_pot4 < 0 || pct_fixed4 < 0 || pct_fixed8 < 0 || pct_pot4 + pct_fixed4 + pct_fixed8 != 100 || M < 0)
    return -1;
  int64_t n8 = (int64_t)rint((double)M * pct_fixed8 / 100.0);
  if (pct_fixed8 > 0 && n8 < 1 && M > 0) n8 = 1;
  int64_t np = (int64_t)rint((double)M * pct_pot4 / 100.0);
  if (pct_fixed4 == 0) np = M - n8; /* nothing may be left over for an empty class */
  if (n8 + np > M) np = M - n8;
  counts[0] = M - n8 - np;
  counts[1] = np;
  counts[2] = n8;
  return 0;
}

/* Variance-based choice between PoT-4 and Fixed-4 (Alg. 1, the else-branch;
 * Section 3.1): rows already marked Fixed-8 in `scheme` keep it; the others are
 * ordered by the variance of their weights and the n_pot4 rows of lowest
 * variance become PoT-4, the rest Fixed-4.  Ties are broken by row index.
 * Variance is the population variance in float64. */
int oracle_assign_by_variance(const float* W, int64_t M, int64_t K, int64_t n_pot4, uint8_t* scheme) {
  double* var = (double*)malloc(sizeof(double) * (size_t)(M > 0 ? M : 1));
  int64_t* idx = (int64_t*)malloc(sizeof(int64_t) * (size_t)(M > 0 ? M : 1));
  if (!var || !idx) {
    free(var);
    free(idx);
    return -1;
  }
  int64_t cnt = 0;
  for (int64_t r = 0; r < M; ++r) {
    if (scheme[r] == SCHEME_FIXED8) continue;
    double mean = 0.0;
    for (int64_t k = 0; k < K; ++k) mean += W[r * K + k];
    mean /= (double)(K > 0 ? K : 1);
    double v = 0.0;
    for (int64_t k = 0; k < K; ++k) {
      double dlt = W[r * K + k] - mean;
      v += dlt * dlt;
    }
    var[r] = v / (double)(K > 0 ? K : 1);
    idx[cnt++] = r;
  }
  if (n_pot4 > cnt) n_pot4 = cnt;
  /* insertion sort by (variance, row index): small M, obviously correct */
  for (int64_t i = 1; i < cnt; ++i) {
    int64_t key = idx[i];
    int64_t j = i - 1;
    while (j >= 0 && (var[idx[j]] > var[key] || (var[idx[j]] == var[key] && idx[j] > key))) {
      idx[j + 1] = idx[j];
      --j;
    }
    idx[j + 1] = key;
  }
  for (int64_t i = 0; i < cnt; ++i) scheme[idx[i]] = (i < n_pot4) ? SCHEME_POT4 : SCHEME_FIXED4;
  free(var);
  free(idx);
  return 0;
}

/* ------------------------------------------------------------------ */
/* Quantization-aware training step (Alg. 1, loop body; Eq. 5, the STE) */
/* ------------------------------------------------------------------ */

/* Forward: proj_S(W) as fp32 -- every row projected onto the level set of its
 * own scheme with its own alpha (Eq. 1, Eq. 3), the level written as
 * rowscale * integer, one fp32 multiply, which is the value the inference path
 * works with.  alpha_in NULL -> alpha_r = max|w_r| (all-zero row: 1).
 * alpha_out (nullable) receives the alpha used.  Returns 0 / -1 as
 * oracle_quantize_rows does. */
int oracle_project_rows_f32(const float* W, int64_t M, int64_t K, const uint8_t* scheme,
                            const float* alpha_in, float* what, float* alpha_out) {
  for (int64_t r = 0; r < M; ++r) {
    const float* w = W + r * K;
    float alpha = alpha_in ? alpha_in[r] : oracle_row_alpha(w, K);
    if (!alpha_in && alpha == 0.0f) alpha = 1.0f;
    if (!(alpha > 0.0f)) return -1;
    if (alpha_out) alpha_out[r] = alpha;
    if (scheme[r] == SCHEME_POT4) {
      float rowscale = alpha * 0.015625f;
      for (int64_t k = 0; k < K; ++k) what[r * K + k] = rowscale * (float)oracle_pot4_int(w[k], alpha);
    } else if (scheme[r] == SCHEME_FIXED4 || scheme[r] == SCHEME_FIXED8) {
      int m = scheme[r] == SCHEME_FIXED4 ? 4 : 8;
      float rowscale = alpha / (float)fixed_steps(m);
      for (int64_t k = 0; k < K; ++k) what[r * K + k] = rowscale * (float)oracle_fixed_code(w[k], alpha, m);
    } else {
      return -1;
    }
  }
  return 0;
}

/* Backward (Eq. 5 and the back-propagation line of Alg. 1): the gradient with
 * respect to the projected weights is handed to the weights unchanged -- the
 * derivative of round() is taken as 1.  The clip in front of the rounding
 * (Section 3.1.1) is an ordinary function whose derivative is 0 outside
 * [-alpha, alpha], so a weight that was clipped receives no gradient; with
 * alpha = max|w_r| (alpha_in NULL) nothing is clipped and dW = dWhat. */
void oracle_ste_backward(const float* W, int64_t M, int64_t K, const float* alpha_in, const float* dwhat,
                         float* dw) {
  for (int64_t r = 0; r < M; ++r)
    for (int64_t k = 0; k < K; ++k) {
      float g = dwhat[r * K + k];
      if (alpha_in && fabsf(W[r * K + k]) > alpha_in[r]) g = 0.0f;
      dw[r * K + k] = g;
    }
}
