/*
 * halp_ref.c -- CPU oracle for the HALP epoch.  TEST INFRASTRUCTURE ONLY:
 * see halp_ref.h for what may use it, what it follows and how the open points
 * of the paper are read.  Plain C, one thread, fp64, exact 64-bit integers.
 */
#include "halp_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- Philox */

/* One Philox4x32 round (Salmon et al., SC'11, Sec. 3.3 / the "Philox-4x32"
 * row of their table of multipliers): two 32x32->64 products, the high halves
 * are xor-ed with the other counter words and the round key. */
static void philox_round(uint32_t c[4], uint32_t k0, uint32_t k1) {
  const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c[0];
  const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c[2];
  const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
  const uint32_t n1 = (uint32_t)p1;
  const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
  const uint32_t n3 = (uint32_t)p0;
  c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

void halp_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c[4] = {ctr[0], ctr[1], ctr[2], ctr[3]};
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { /* Weyl key schedule: golden ratio and sqrt(3)-1 */
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    philox_round(c, k0, k1);
  }
  memcpy(out, c, sizeof c);
}

uint32_t halp_ref_stream_word(uint64_t seed, uint32_t purpose, uint32_t epoch, uint64_t n) {
  const uint64_t block = n >> 2;
  const uint32_t ctr[4] = {(uint32_t)block, (uint32_t)(block >> 32), epoch, purpose};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  halp_ref_philox4x32_10(ctr, key, out);
  return out[n & 3];
}

/* Rounding bits of z.  A row of z is cut into strips 16 bits of rounding wide
 * (16/b coordinates: two at b = 8, one at b = 16).  One Philox block serves a
 * strip for the eight steps 8s .. 8s+7: counter = (strip, s, epoch, ZROUND);
 * step t uses the 16-bit field t mod 8 of the block (field f = half f%2 of
 * word f/2), and coordinate k of the strip the bits [k b, (k+1) b) of it. */
uint32_t halp_ref_zround_bits(uint64_t seed, uint32_t epoch, uint64_t t, int32_t d, int32_t b,
                              int32_t c, int32_t j) {
  if (b > 16) { /* wide models exist on the CPU only (the many-bits check against SVRG): one
                   word of the stream per step and coordinate, low b bits */
    const uint64_t n = t * (uint64_t)d * 64u + (uint64_t)c * (uint64_t)d + (uint64_t)j;
    return halp_ref_stream_word(seed, HALP_REF_PURPOSE_ZROUND, epoch, n) & ((1u << b) - 1u);
  }
  const int32_t cps = 16 / b;               /* coordinates per strip */
  const int32_t U = (d + cps - 1) / cps;    /* strips per class      */
  const uint32_t strip = (uint32_t)c * (uint32_t)U + (uint32_t)(j / cps);
  const uint32_t ctr[4] = {strip, (uint32_t)(t >> 3), epoch, HALP_REF_PURPOSE_ZROUND};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  halp_ref_philox4x32_10(ctr, key, out);
  const int f = (int)(t & 7);
  const uint32_t field = (out[f >> 1] >> (16 * (f & 1))) & 0xFFFFu;
  return (field >> ((j % cps) * b)) & ((1u << b) - 1u);
}

int64_t halp_ref_sample_index(uint64_t seed, uint32_t epoch, uint64_t t, int32_t B, int32_t m,
                              int64_t N) {
  const uint32_t r = halp_ref_stream_word(seed, HALP_REF_PURPOSE_IDX, epoch,
                                          t * (uint64_t)B + (uint64_t)m);
  return (int64_t)(((uint64_t)r * (uint64_t)N) >> 32);
}

int64_t halp_ref_option2_steps(uint64_t seed, uint32_t epoch, int64_t T) {
  if (T <= 0) return T;
  const uint32_t r = halp_ref_stream_word(seed, HALP_REF_PURPOSE_OPT2, epoch, 0);
  return (int64_t)(((uint64_t)r * (uint64_t)T) >> 32);
}

/* ------------------------------------------------------------ quantizers */

/* Sec. 3 "Quantization": inside the domain round down to the lattice point
 * below and up with probability equal to the fractional part; outside, the
 * nearest end of the domain.  floor(q + rho) with rho uniform on [0,1) is
 * exactly that rule. */
int64_t halp_ref_quantize_real(double x, double inv_delta, uint32_t r32, int64_t lo, int64_t hi,
                               int* clamped) {
  const double rho = (double)r32 * 0x1p-32;
  const double q = x * inv_delta;
  double f = floor(q + rho);
  int hit = 0;
  if (f < (double)lo) { f = (double)lo; hit = 1; }
  if (f > (double)hi) { f = (double)hi; hit = 1; }
  if (clamped) *clamped = hit;
  return (int64_t)f;
}

static int64_t floor_div_pow2(int64_t x, int b) {
  const int64_t m = (int64_t)1 << b;
  int64_t q = x / m;
  if (x % m != 0 && x < 0) q -= 1;
  return q;
}

/* Text after Algorithm 4: u lives in (delta_i, 2b), z enters it by a shift
 * left of b bits.  Q_(delta_m,b)(u) then only has to round v = u - (z << b):
 * with r uniform on {0..2^b-1}, floor((v + r)/2^b) rounds v/2^b up with
 * probability equal to its fractional part. */
int64_t halp_ref_round_shift(int64_t z, int64_t v, uint32_t r, int b, int* clamped) {
  const int64_t qmax = ((int64_t)1 << (b - 1)) - 1, qmin = -((int64_t)1 << (b - 1));
  int64_t out = z + floor_div_pow2(v + (int64_t)r, b);
  int hit = 0;
  if (out > qmax) { out = qmax; hit = 1; }
  if (out < qmin) { out = qmin; hit = 1; }
  if (clamped) *clamped = hit;
  return out;
}

static int64_t xq_at(const void* Xq, int b, int64_t k) {
  if (b == 8) return ((const int8_t*)Xq)[k];
  if (b == 16) return ((const int16_t*)Xq)[k];
  return ((const int32_t*)Xq)[k];
}

void halp_ref_quantize_data(const float* X, int64_t n, double delta_d, int b, void* Xq) {
  const double qmax = (double)(((int64_t)1 << (b - 1)) - 1);
  for (int64_t k = 0; k < n; ++k) {
    double q = nearbyint((double)X[k] / delta_d); /* default mode: ties to even */
    if (q > qmax) q = qmax;
    if (q < -qmax) q = -qmax;
    if (b == 8) ((int8_t*)Xq)[k] = (int8_t)q;
    else if (b == 16) ((int16_t*)Xq)[k] = (int16_t)q;
    else ((int32_t*)Xq)[k] = (int32_t)q;
  }
}

void halp_ref_quantize_data_scaled(const float* X, int64_t rows, int32_t d, double delta_d,
                                   const float* s, int b, void* Xq) {
  const double qmax = (double)(((int64_t)1 << (b - 1)) - 1);
  for (int64_t i = 0; i < rows; ++i)
    for (int32_t j = 0; j < d; ++j) {
      const int64_t k = i * d + j;
      double q = nearbyint((double)X[k] / (delta_d * (double)s[j]));
      if (q > qmax) q = qmax;
      if (q < -qmax) q = -qmax;
      if (b == 8) ((int8_t*)Xq)[k] = (int8_t)q;
      else if (b == 16) ((int16_t*)Xq)[k] = (int16_t)q;
      else ((int32_t*)Xq)[k] = (int32_t)q;
    }
}

/* ------------------------------------------------------- scalar losses l_i */

static double logistic_dl(double a, double y) { /* l'(a) for l = log(1+exp(-y a)) */
  return -y / (1.0 + exp(y * a));
}

static double logistic_l(double a, double y) {
  const double s = -y * a; /* log(1 + e^s) without overflow */
  return (s > 0 ? s : 0.0) + log1p(exp(-fabs(s)));
}

/* softmax probabilities of K logits (full-precision pass: the plain definition) */
static void softmax_p(const double* a, int K, double* prob) {
  double mx = a[0];
  for (int c = 1; c < K; ++c) if (a[c] > mx) mx = a[c];
  double s = 0.0;
  for (int c = 0; c < K; ++c) { prob[c] = exp(a[c] - mx); s += prob[c]; }
  for (int c = 0; c < K; ++c) prob[c] = prob[c] / s;
}

/* ---------------------------------------------- scalar path of the inner loop */

/* The inner loop turns l'(phi + x^T z) - l'(phi) into the integer gamma, so the last bit of
 * exp can decide an integer.  The paper does not say how exp is rounded; to make that decision
 * reproducible, the inner loop's exp is this fixed sequence of IEEE double operations (every
 * one of them correctly rounded, so any conforming machine gives the same bits):
 *   k = rint(x log2 e);  r = x - k ln2 (ln2 in two parts, two fused multiply-adds);
 *   e^r = 1 + (r + r^2 Q(r)), Q the Taylor polynomial sum_{n=2..13} r^(n-2)/n! evaluated
 *   pairwise (coefficients joined in pairs by r, pairs by r^2, then by r^4);
 *   result = e^r 2^k.
 * |r| <= ln2/2, where the omitted terms are below 1e-17; the result is within 1 ulp of exp. */
double halp_ref_exp(double x) {
  if (x != x) return x;
  if (x > 0x1.62e42fefa39efp+9) return INFINITY;  /* above log(DBL_MAX) */
  if (x < -0x1.74910d52d3052p+9) return 0.0;      /* below log of half the least subnormal */
  const double k = nearbyint(x * 0x1.71547652b82fep+0);
  double r = fma(-k, 0x1.62e42fefa39efp-1, x);
  r = fma(-k, 0x1.abc9e3b39803fp-56, r);
  const double r2 = r * r, r4 = r2 * r2;
  const double a0 = fma(0x1.5555555555555p-3, r, 0x1.0000000000000p-1);   /* 1/2!  + r/3!  */
  const double a1 = fma(0x1.1111111111111p-7, r, 0x1.5555555555555p-5);   /* 1/4!  + r/5!  */
  const double a2 = fma(0x1.a01a01a01a01ap-13, r, 0x1.6c16c16c16c17p-10); /* 1/6!  + r/7!  */
  const double a3 = fma(0x1.71de3a556c734p-19, r, 0x1.a01a01a01a01ap-16); /* 1/8!  + r/9!  */
  const double a4 = fma(0x1.ae64567f544e4p-26, r, 0x1.27e4fb7789f5cp-22); /* 1/10! + r/11! */
  const double a5 = fma(0x1.6124613a86d09p-33, r, 0x1.1eed8eff8d898p-29); /* 1/12! + r/13! */
  const double b0 = fma(a1, r2, a0), b1 = fma(a3, r2, a2), b2 = fma(a5, r2, a4);
  const double q = fma(fma(b2, r4, b1), r4, b0);
  const double e = fma(r2, q, r) + 1.0;
  return ldexp(e, (int)k);
}

void halp_ref_exp_array(const double* x, int64_t n, double* out) {
  for (int64_t k = 0; k < n; ++k) out[k] = halp_ref_exp(x[k]);
}

static double logistic_dl_inner(double a, double y) { /* l'(a), exp as above */
  return -y / (1.0 + halp_ref_exp(y * a));
}

/* Softmax probabilities of K logits for the inner loop.  The normaliser is summed pairwise
 * (classes 0+1, 2+3, ..., then those sums in adjacent pairs, and so on; missing classes count
 * as +0, which changes nothing): again a fixed order, chosen because it is a reduction tree. */
static void softmax_p_inner(const double* a, int K, double* prob) {
  double mx = a[0];
  for (int c = 1; c < K; ++c) if (a[c] > mx) mx = a[c];
  double v[64];
  int P = 1;
  while (P < K) P *= 2;
  for (int c = 0; c < P; ++c) {
    v[c] = 0.0;
    if (c < K) { prob[c] = halp_ref_exp(a[c] - mx); v[c] = prob[c]; }
  }
  for (; P > 1; P /= 2)
    for (int c = 0; c < P / 2; ++c) v[c] = v[2 * c] + v[2 * c + 1];
  for (int c = 0; c < K; ++c) prob[c] = prob[c] / v[0];
}

/* l'(a1) - l'(a0) per class, the bracket of Algorithm 4's beta line.  lin is the squared
 * loss's difference, formed by the caller without cancellation.  path selects the leg:
 * PLAIN is the definition (libm exp, normaliser summed left to right: the functions of the
 * full-precision pass), FIXED the reproducible reading above. */
static void scalar_difference(int loss, int path, int K, const double* a0, const double* a1,
                              double yi, double lin, double* out) {
  if (loss == HALP_REF_LOGISTIC) {
    out[0] = path == HALP_REF_SCALAR_PLAIN ? logistic_dl(a1[0], yi) - logistic_dl(a0[0], yi)
                                           : logistic_dl_inner(a1[0], yi) - logistic_dl_inner(a0[0], yi);
  } else if (loss == HALP_REF_SOFTMAX) {
    double q0[64], q1[64];
    if (path == HALP_REF_SCALAR_PLAIN) { softmax_p(a0, K, q0); softmax_p(a1, K, q1); }
    else { softmax_p_inner(a0, K, q0); softmax_p_inner(a1, K, q1); }
    for (int c = 0; c < K; ++c) out[c] = q1[c] - q0[c];
  } else {
    out[0] = lin;
  }
}

/* --------------------------------------------------- Algorithm 4, outer part */

int halp_ref_full_gradient(const halp_ref_problem* p, const float* X, int64_t ldx, const void* y,
                           const float* w, double* phi, double* g, double* loss) {
  const int64_t N = p->N; const int d = p->d, K = p->K;
  if (N <= 0 || d <= 0 || K <= 0 || K > 64) return -1;
  if (p->loss != HALP_REF_SOFTMAX && K != 1) return -1;
  double a[64], r[64];
  double total = 0.0;
  for (int64_t k = 0; k < (int64_t)K * d; ++k) g[k] = 0.0;
  for (int64_t i = 0; i < N; ++i) {
    const float* x = X + i * ldx;
    for (int c = 0; c < K; ++c) { /* phi_i = x_i^T w~ */
      double s = 0.0;
      for (int j = 0; j < d; ++j) s += (double)x[j] * (double)w[(int64_t)c * d + j];
      a[c] = s;
      phi[i * K + c] = s;
    }
    if (p->loss == HALP_REF_SQUARED) {
      const double yi = ((const float*)y)[i];
      r[0] = a[0] - yi;
      total += 0.5 * r[0] * r[0];
    } else if (p->loss == HALP_REF_LOGISTIC) {
      const double yi = ((const float*)y)[i];
      r[0] = logistic_dl(a[0], yi);
      total += logistic_l(a[0], yi);
    } else {
      const int yi = ((const int32_t*)y)[i];
      if (yi < 0 || yi >= K) return -2;
      softmax_p(a, K, r);
      /* -log p_y = log sum exp(a - max) + max - a_y */
      double mx = a[0];
      for (int c = 1; c < K; ++c) if (a[c] > mx) mx = a[c];
      double s = 0.0;
      for (int c = 0; c < K; ++c) s += exp(a[c] - mx);
      total += log(s) + mx - a[yi];
      r[yi] -= 1.0;
    }
    for (int c = 0; c < K; ++c) /* sum_i l'_i(phi_i) x_i */
      for (int j = 0; j < d; ++j) g[(int64_t)c * d + j] += r[c] * (double)x[j];
  }
  double w2 = 0.0;
  for (int64_t k = 0; k < (int64_t)K * d; ++k) {
    g[k] = g[k] / (double)N + p->lambda * (double)w[k];
    w2 += (double)w[k] * (double)w[k];
  }
  *loss = total / (double)N + 0.5 * p->lambda * w2;
  return 0;
}

int halp_ref_full_gradient_scaled(const halp_ref_problem* p, const float* X, int64_t ldx,
                                  const void* y, const float* v, const float* s, double* phi,
                                  double* g, double* loss) {
  const int64_t n = (int64_t)p->K * p->d;
  if (p->lambda != 0.0) return -1; /* lambda ||w||^2 is not lambda ||v||^2 */
  float* w = (float*)calloc((size_t)n + 1, sizeof(float));
  for (int64_t k = 0; k < n; ++k) w[k] = v[k] / s[k % p->d]; /* the model the data belong to */
  const int rc = halp_ref_full_gradient(p, X, ldx, y, w, phi, g, loss);
  free(w);
  if (rc != 0) return rc;
  for (int64_t k = 0; k < n; ++k) g[k] = g[k] / (double)s[k % p->d]; /* d f / d v_j */
  return 0;
}

int halp_ref_recenter(const halp_ref_problem* p, const float* g, uint32_t epoch, double scales[8],
                      int64_t* h, int32_t* z) {
  const int b = p->b;
  const int64_t n = (int64_t)p->K * p->d;
  if (b < 2 || b > 24 || !(p->mu > 0) || !(p->alpha > 0) || !(p->delta_d > 0)) return -1;
  const double qmax = (double)(((int64_t)1 << (b - 1)) - 1);
  double ss = 0.0;
  for (int64_t k = 0; k < n; ++k) ss += (double)g[k] * (double)g[k];
  const double nrm = sqrt(ss);
  for (int64_t k = 0; k < n; ++k) { h[k] = 0; z[k] = 0; } /* z_{k,0} = Q(0) = 0 */
  for (int k = 0; k < 8; ++k) scales[k] = 0.0;
  scales[3] = nrm;
  if (!isfinite(nrm)) { scales[7] = -1.0; return 0; }
  if (nrm == 0.0) { scales[7] = 1.0; return 0; }
  const double delta_m = nrm / (p->mu * qmax);          /* s~_k                  */
  const double delta_i = delta_m * ldexp(1.0, -b);      /* 2^-b delta_m          */
  const double delta_s = delta_i / p->delta_d;          /* 2^-b delta_m/delta_d  */
  const double inv_i = 1.0 / delta_i, inv_s = 1.0 / delta_s;
  if (!(delta_i > 0) || !isfinite(inv_i) || !isfinite(inv_s)) { scales[7] = -1.0; return 0; }
  scales[0] = delta_m; scales[1] = delta_i; scales[2] = delta_s;
  scales[4] = inv_i; scales[5] = inv_s;
  const int64_t hmax = ((int64_t)1 << (2 * b - 1)) - 1, hmin = -((int64_t)1 << (2 * b - 1));
  for (int64_t k = 0; k < n; ++k) { /* h~ = Q_(delta_i,2b)(alpha g~) */
    const uint32_t r = halp_ref_stream_word(p->seed, HALP_REF_PURPOSE_HROUND, epoch, (uint64_t)k);
    h[k] = halp_ref_quantize_real(p->alpha * (double)g[k], inv_i, r, hmin, hmax, 0);
  }
  return 0;
}

/* ------------------------------------------- Algorithm 2 in integers, epoch start */

int halp_ref_lp_begin(const halp_ref_problem* p, const float* g, const float* w, uint32_t epoch,
                      double scales[8], int64_t* h, int32_t* z) {
  const int b = p->b;
  const int64_t n = (int64_t)p->K * p->d;
  if (b < 2 || b > 24 || !(p->delta > 0) || !(p->alpha > 0) || !(p->delta_d > 0)) return -1;
  if (p->lambda != 0) return -1;
  const double qmax = (double)(((int64_t)1 << (b - 1)) - 1), qmin = -(double)((int64_t)1 << (b - 1));
  double ss = 0.0;
  for (int64_t k = 0; k < n; ++k) ss += (double)g[k] * (double)g[k];
  const double nrm = sqrt(ss);
  for (int64_t k = 0; k < n; ++k) { /* w_{k,0} = w~_k in (delta, b) */
    double q = nearbyint((double)w[k] / p->delta);
    if (!(q >= qmin)) q = qmin; /* also catches NaN */
    if (q > qmax) q = qmax;
    z[k] = (int32_t)q;
    h[k] = 0;
  }
  for (int k = 0; k < 8; ++k) scales[k] = 0.0;
  scales[3] = nrm;
  if (!isfinite(nrm)) { scales[7] = -1.0; return 0; }
  if (nrm == 0.0) { scales[7] = 1.0; return 0; }
  const double delta_m = p->delta;
  const double delta_i = delta_m * ldexp(1.0, -b);
  const double delta_s = delta_i / p->delta_d;
  const double inv_i = 1.0 / delta_i, inv_s = 1.0 / delta_s;
  if (!(delta_i > 0) || !isfinite(inv_i) || !isfinite(inv_s)) { scales[7] = -1.0; return 0; }
  scales[0] = delta_m; scales[1] = delta_i; scales[2] = delta_s;
  scales[4] = inv_i; scales[5] = inv_s;
  const int64_t hmax = ((int64_t)1 << (2 * b - 1)) - 1, hmin = -((int64_t)1 << (2 * b - 1));
  for (int64_t k = 0; k < n; ++k) {
    const uint32_t r = halp_ref_stream_word(p->seed, HALP_REF_PURPOSE_HROUND, epoch, (uint64_t)k);
    h[k] = halp_ref_quantize_real(p->alpha * (double)g[k], inv_i, r, hmin, hmax, 0);
  }
  return 0;
}

/* --------------------------------------------------- Algorithm 4, inner loop */

int halp_ref_inner_loop(const halp_ref_problem* p, const void* Xq, int64_t ldxq, const float* phi,
                        const void* y, const int64_t* h, const double scales[8], uint32_t epoch,
                        int64_t T, int32_t* z, const halp_ref_trace* trace, uint64_t counters[4]) {
  const int64_t N = p->N; const int d = p->d, K = p->K, B = p->B, b = p->b;
  if (counters) for (int k = 0; k < 4; ++k) counters[k] = 0;
  if (scales[7] != 0.0) return 0; /* converged or unusable gradient: z stays 0 */
  if (N <= 0 || d <= 0 || K <= 0 || K > 64 || B <= 0 || T < 0) return -1;
  const int64_t qmax = ((int64_t)1 << (b - 1)) - 1, qmin = -((int64_t)1 << (b - 1));
  const double delta_m = scales[0], inv_s = scales[5];
  const double dscale = p->delta_d * delta_m;  /* scale of the integer product x^T z */
  const double aB = p->alpha / (double)B;
  const int lp = p->algorithm == HALP_REF_ALG_LPSVRG;
  if (lp && p->lambda != 0) return -1;
  int64_t* idx = (int64_t*)malloc(sizeof(int64_t) * (size_t)B);
  int64_t* gam = (int64_t*)malloc(sizeof(int64_t) * (size_t)B * (size_t)K);
  int64_t* znew = (int64_t*)malloc(sizeof(int64_t) * (size_t)K * (size_t)d);
  double a0[64], a1[64], p0[64], p1[64], p2[64];
  for (int64_t t = 0; t < T; ++t) {
    const int rec = trace && t < trace->M;
    /* sample i uniformly */
    for (int m = 0; m < B; ++m) {
      idx[m] = halp_ref_sample_index(p->seed, epoch, (uint64_t)t, B, m, N);
      if (rec && trace->idx) trace->idx[t * B + m] = idx[m];
    }
    /* beta = alpha (l'(phi_i + x_i^T z) - l'(phi_i)), gamma = Q_(delta_s,b)(beta) */
    for (int m = 0; m < B; ++m) {
      const int64_t i = idx[m];
      for (int c = 0; c < K; ++c) {
        int64_t D = 0; /* low-precision dot product, scale delta_d * delta_m */
        for (int j = 0; j < d; ++j) D += xq_at(Xq, b, i * ldxq + j) * (int64_t)z[(int64_t)c * d + j];
        a0[c] = (double)phi[i * K + c];
        /* Algorithm 4: the margin moves by x^T z; Algorithm 2: x^T w is the whole margin */
        a1[c] = lp ? dscale * (double)D : a0[c] + dscale * (double)D;
        if (rec && trace->D) trace->D[(t * B + m) * K + c] = D;
        p0[c] = dscale * (double)D; /* kept for the squared loss */
      }
      const double yi = p->loss == HALP_REF_LOGISTIC ? (double)((const float*)y)[i] : 0.0;
      const double lin = lp ? p0[0] - a0[0] : p0[0];
      scalar_difference(p->loss, p->scalar_path, K, a0, a1, yi, lin, p1);
      const int other = rec && (trace->beta_other || trace->gamma_other);
      if (other) scalar_difference(p->loss, !p->scalar_path, K, a0, a1, yi, lin, p2);
      for (int c = 0; c < K; ++c) {
        const double beta = aB * p1[c];
        const uint64_t n = ((uint64_t)t * (uint64_t)B + (uint64_t)m) * (uint64_t)K + (uint64_t)c;
        const uint32_t r = halp_ref_stream_word(p->seed, HALP_REF_PURPOSE_GAMMA, epoch, n);
        int hit = 0;
        const int64_t gq = halp_ref_quantize_real(beta, inv_s, r, qmin, qmax, &hit);
        gam[m * K + c] = gq;
        if (counters) counters[1] += (uint64_t)hit;
        if (rec && trace->beta) trace->beta[(t * B + m) * K + c] = beta;
        if (rec && trace->gamma) trace->gamma[(t * B + m) * K + c] = (int32_t)gq;
        if (other) { /* the other leg, same state and same draw */
          const double beta2 = aB * p2[c];
          const int64_t gq2 = halp_ref_quantize_real(beta2, inv_s, r, qmin, qmax, 0);
          if (trace->beta_other) trace->beta_other[(t * B + m) * K + c] = beta2;
          if (trace->gamma_other) trace->gamma_other[(t * B + m) * K + c] = (int32_t)gq2;
        }
      }
    }
    /* L2: the variance-reduced difference contributes lambda z */
    int64_t c_lambda = 0;
    if (p->lambda > 0) {
      const uint32_t r = halp_ref_stream_word(p->seed, HALP_REF_PURPOSE_REG, epoch, (uint64_t)t);
      c_lambda = halp_ref_quantize_real(p->alpha * p->lambda, ldexp(1.0, b), r, 0, qmax, 0);
      if (counters && c_lambda != 0) counters[2] += 1;
    }
    /* u = z - gamma x_i - h~, then z = Q_(delta_m,b)(u) */
    for (int c = 0; c < K; ++c) {
      for (int j = 0; j < d; ++j) {
        const int64_t k = (int64_t)c * d + j;
        int64_t v = -h[k] - c_lambda * (int64_t)z[k];
        for (int m = 0; m < B; ++m) v -= gam[m * K + c] * xq_at(Xq, b, idx[m] * ldxq + j);
        const uint32_t r = halp_ref_zround_bits(p->seed, epoch, (uint64_t)t, d, b, c, j);
        int hit = 0;
        znew[k] = halp_ref_round_shift((int64_t)z[k], v, r, b, &hit);
        if (counters) counters[0] += (uint64_t)hit;
      }
    }
    for (int64_t k = 0; k < (int64_t)K * d; ++k) z[k] = (int32_t)znew[k];
    if (rec && trace->ztraj)
      memcpy(trace->ztraj + t * (int64_t)K * d, z, sizeof(int32_t) * (size_t)K * (size_t)d);
  }
  (void)qmin;
  free(idx); free(gam); free(znew);
  return 0;
}

/* ------------------------------------------------------ Algorithm 1, inner loop */

int halp_ref_svrg_inner(const halp_ref_problem* p, const float* X, int64_t ldx, const void* y,
                        const float* phi, const float* g, uint32_t epoch, int64_t T, double* w) {
  const int64_t N = p->N; const int d = p->d, B = p->B;
  if (N <= 0 || d <= 0 || p->K != 1 || B <= 0 || T < 0) return -1;
  if (p->loss != HALP_REF_SQUARED && p->loss != HALP_REF_LOGISTIC) return -1;
  double* wt = (double*)malloc(sizeof(double) * (size_t)d);
  double* step = (double*)malloc(sizeof(double) * (size_t)d);
  for (int j = 0; j < d; ++j) wt[j] = w[j];
  for (int64_t t = 0; t < T; ++t) {
    for (int j = 0; j < d; ++j) step[j] = p->lambda * (w[j] - wt[j]) + (double)g[j];
    for (int m = 0; m < B; ++m) {
      const int64_t i = halp_ref_sample_index(p->seed, epoch, (uint64_t)t, B, m, N);
      const float* x = X + i * ldx;
      double a1 = 0.0;
      for (int j = 0; j < d; ++j) a1 += (double)x[j] * w[j];
      const double a0 = (double)phi[i];
      double diff;
      if (p->loss == HALP_REF_LOGISTIC) {
        const double yi = ((const float*)y)[i];
        diff = logistic_dl(a1, yi) - logistic_dl(a0, yi);
      } else {
        diff = a1 - a0; /* (a1 - y) - (a0 - y) */
      }
      for (int j = 0; j < d; ++j) step[j] += diff / (double)B * (double)x[j];
    }
    for (int j = 0; j < d; ++j) w[j] -= p->alpha * step[j];
  }
  free(wt); free(step);
  return 0;
}

void halp_ref_apply_offset(const halp_ref_problem* p, const double scales[8], const int32_t* z,
                           float* w) {
  if (scales[7] != 0.0) return;
  const double delta_m = scales[0];
  for (int64_t k = 0; k < (int64_t)p->K * p->d; ++k) {
    const double step = delta_m * (double)z[k];
    if (p->algorithm == HALP_REF_ALG_LPSVRG) w[k] = (float)step; /* w~ = delta w (option I) */
    else w[k] = (float)((double)w[k] + step);
  }
}

int halp_ref_epoch(const halp_ref_problem* p, const float* X, int64_t ldx, const void* Xq,
                   int64_t ldxq, const void* y, float* w, uint32_t epoch, int64_t T, float* phi32,
                   float* g32, double scales[8], int64_t* h, int32_t* z, uint64_t counters[4]) {
  const int64_t nphi = p->N * p->K, nw = (int64_t)p->K * p->d;
  double* phi = (double*)malloc(sizeof(double) * (size_t)nphi);
  double* g = (double*)malloc(sizeof(double) * (size_t)nw);
  double loss = 0.0;
  int rc = halp_ref_full_gradient(p, X, ldx, y, w, phi, g, &loss);
  if (rc == 0) {
    /* the full-precision pass hands fp32 margins and an fp32 gradient on */
    for (int64_t k = 0; k < nphi; ++k) phi32[k] = (float)phi[k];
    for (int64_t k = 0; k < nw; ++k) g32[k] = (float)g[k];
    rc = p->algorithm == HALP_REF_ALG_LPSVRG ? halp_ref_lp_begin(p, g32, w, epoch, scales, h, z)
                                             : halp_ref_recenter(p, g32, epoch, scales, h, z);
    scales[6] = loss;
  }
  free(phi); free(g);
  if (rc != 0) return rc;
  rc = halp_ref_inner_loop(p, Xq, ldxq, phi32, y, h, scales, epoch, T, z, 0, counters);
  if (rc != 0) return rc;
  halp_ref_apply_offset(p, scales, z, w);
  return 0;
}
