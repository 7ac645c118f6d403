/* Driver that runs every entry point of the CPU oracle once on small ragged inputs, meant to
 * be built together with halp_ref.c under -fsanitize=address,undefined (oracle/build.py,
 * build_sanitized).  Test infrastructure only: it checks memory safety and defined behaviour
 * of the oracle's C, not its values (the pins in tests/ do that).  Prints "ok" and returns 0
 * when every call returned 0; any sanitizer report aborts the run.                           */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "halp_ref.h"

static uint64_t lcg_state = 0x9E3779B97F4A7C15ull;
static double unif(void) { /* (-1, 1) */
  lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
  return ((double)(lcg_state >> 11) / 9007199254740992.0) * 2.0 - 1.0;
}

#define CHECK(call)                                              \
  do {                                                           \
    int rc_ = (call);                                            \
    if (rc_ != 0) {                                              \
      fprintf(stderr, "%s returned %d\n", #call, rc_);           \
      return 1;                                                  \
    }                                                            \
  } while (0)

static halp_ref_problem problem(int64_t N, int d, int K, int loss, int b, int B, double lambda,
                                double delta_d) {
  halp_ref_problem p;
  memset(&p, 0, sizeof p);
  p.N = N; p.d = d; p.K = K; p.loss = loss; p.b = b; p.B = B;
  p.algorithm = HALP_REF_ALG_HALP;
  p.alpha = 0.05; p.mu = 0.5; p.lambda = lambda; p.delta_d = delta_d; p.seed = 1234;
  p.delta = 0.0; p.scalar_path = HALP_REF_SCALAR_FIXED;
  return p;
}

/* one epoch of every phase with a trace of the first steps, for one configuration */
static int run_config(int loss, int K, int b, int B, double lambda, int algorithm, int scalar_path) {
  const int64_t N = 53;
  const int d = 37;
  const int64_t T = 41, M = 9;
  const int64_t ldx = d + 3, ldxq = d + 1; /* strided rows on purpose */
  float* X = (float*)malloc(sizeof(float) * (size_t)(N * ldx));
  void* y = malloc(4 * (size_t)N);
  float* w = (float*)malloc(sizeof(float) * (size_t)(K * d));
  for (int64_t i = 0; i < N * ldx; ++i) X[i] = (float)unif();
  for (int64_t i = 0; i < N; ++i) {
    if (loss == HALP_REF_SOFTMAX) ((int32_t*)y)[i] = (int32_t)((unif() + 1.0) * 0.5 * K) % K;
    else if (loss == HALP_REF_LOGISTIC) ((float*)y)[i] = unif() < 0 ? -1.f : 1.f;
    else ((float*)y)[i] = (float)unif();
  }
  for (int i = 0; i < K * d; ++i) w[i] = (float)(0.1 * unif());
  const int qmax = (1 << (b - 1)) - 1;
  halp_ref_problem p = problem(N, d, K, loss, b, B, lambda, 1.0 / qmax);
  p.algorithm = algorithm;
  p.scalar_path = scalar_path;
  if (algorithm == HALP_REF_ALG_LPSVRG) p.delta = b == 8 ? 1.0 / 64 : 1.0 / 8192;

  const size_t esz = b == 8 ? 1 : (b == 16 ? 2 : 4);
  unsigned char* Xq = (unsigned char*)malloc(esz * (size_t)(N * ldxq));
  memset(Xq, 0, esz * (size_t)(N * ldxq));
  for (int64_t i = 0; i < N; ++i) /* row by row: the quantizer takes a dense run of values */
    halp_ref_quantize_data(X + i * ldx, d, p.delta_d, b, Xq + esz * (size_t)(i * ldxq));

  double* phi = (double*)malloc(sizeof(double) * (size_t)(N * K));
  double* g = (double*)malloc(sizeof(double) * (size_t)(K * d));
  float* phi32 = (float*)malloc(sizeof(float) * (size_t)(N * K));
  float* g32 = (float*)malloc(sizeof(float) * (size_t)(K * d));
  int64_t* h = (int64_t*)malloc(sizeof(int64_t) * (size_t)(K * d));
  int32_t* z = (int32_t*)malloc(sizeof(int32_t) * (size_t)(K * d));
  double scales[8], loss_value = 0.0;
  uint64_t counters[4];
  CHECK(halp_ref_full_gradient(&p, X, ldx, y, w, phi, g, &loss_value));
  for (int64_t k = 0; k < N * K; ++k) phi32[k] = (float)phi[k];
  for (int k = 0; k < K * d; ++k) g32[k] = (float)g[k];
  if (algorithm == HALP_REF_ALG_LPSVRG) CHECK(halp_ref_lp_begin(&p, g32, w, 2, scales, h, z));
  else CHECK(halp_ref_recenter(&p, g32, 2, scales, h, z));

  halp_ref_trace tr;
  tr.M = M;
  tr.idx = (int64_t*)malloc(sizeof(int64_t) * (size_t)(M * B));
  tr.D = (int64_t*)malloc(sizeof(int64_t) * (size_t)(M * B * K));
  tr.beta = (double*)malloc(sizeof(double) * (size_t)(M * B * K));
  tr.gamma = (int32_t*)malloc(sizeof(int32_t) * (size_t)(M * B * K));
  tr.ztraj = (int32_t*)malloc(sizeof(int32_t) * (size_t)(M * K * d));
  tr.beta_other = (double*)malloc(sizeof(double) * (size_t)(M * B * K));
  tr.gamma_other = (int32_t*)malloc(sizeof(int32_t) * (size_t)(M * B * K));
  CHECK(halp_ref_inner_loop(&p, Xq, ldxq, phi32, y, h, scales, 2, T, z, &tr, counters));
  halp_ref_apply_offset(&p, scales, z, w);
  /* and the same again through the epoch driver, without a trace */
  CHECK(halp_ref_epoch(&p, X, ldx, Xq, ldxq, y, w, 3, T, phi32, g32, scales, h, z, counters));
  if (loss != HALP_REF_SOFTMAX && algorithm == HALP_REF_ALG_HALP) {
    double* wd = (double*)malloc(sizeof(double) * (size_t)d);
    for (int k = 0; k < d; ++k) wd[k] = w[k];
    CHECK(halp_ref_svrg_inner(&p, X, ldx, y, phi32, g32, 4, T, wd));
    free(wd);
  }
  free(tr.idx); free(tr.D); free(tr.beta); free(tr.gamma); free(tr.ztraj);
  free(tr.beta_other); free(tr.gamma_other);
  free(X); free(y); free(w); free(Xq); free(phi); free(g); free(phi32); free(g32); free(h); free(z);
  return 0;
}

static int run_primitives(void) {
  const uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6};
  uint32_t out[4];
  halp_ref_philox4x32_10(ctr, key, out);
  uint64_t acc = out[0];
  for (uint64_t n = 0; n < 40; ++n) acc += halp_ref_stream_word(77, (uint32_t)(n % 6), 3, n * 0x100000001ull);
  acc += (uint64_t)halp_ref_option2_steps(77, 1, 1000);
  for (int t = 0; t < 20; ++t)
    for (int j = 0; j < 37; ++j) {
      acc += halp_ref_zround_bits(9, 2, (uint64_t)t, 37, 8, 1, j);
      acc += halp_ref_zround_bits(9, 2, (uint64_t)t, 37, 16, 0, j);
    }
  for (int t = 0; t < 20; ++t) acc += (uint64_t)halp_ref_sample_index(9, 2, (uint64_t)t, 4, t % 4, 53);
  int clamped = 0;
  const double xs[] = {0.0, 1e-300, -1e-300, 3.7, -3.7, 1e30, -1e30};
  for (unsigned k = 0; k < sizeof xs / sizeof xs[0]; ++k) {
    acc += (uint64_t)halp_ref_quantize_real(xs[k], 128.0, 0x80000000u, -128, 127, &clamped);
    acc += (uint64_t)halp_ref_quantize_real(xs[k], 128.0, 0xFFFFFFFFu, 0, 32767, 0);
  }
  for (int b = 8; b <= 24; b += 8) {
    const int64_t hi = (1 << (b - 1)) - 1, lo = -hi - 1;
    const int64_t zs[] = {lo, -1, 0, 1, hi};
    const int64_t vs[] = {-(hi << b), -1, 0, 1, hi << b};
    for (int i = 0; i < 5; ++i)
      for (int j = 0; j < 5; ++j)
        acc += (uint64_t)halp_ref_round_shift(zs[i], vs[j], (uint32_t)((1u << b) - 1u), b, &clamped);
  }
  const double es[] = {-800.0, -40.0, -1.0, 0.0, 1.0, 40.0, 709.0, 800.0};
  double eo[8];
  halp_ref_exp_array(es, 8, eo);
  for (int k = 0; k < 8; ++k) acc += (uint64_t)(halp_ref_exp(es[k]) == eo[k]);
  /* per-feature scales */
  enum { R = 11, D = 7 };
  float X[R * D], s[D], v[D], yv[R];
  int8_t q8[R * D];
  int16_t q16[R * D];
  for (int i = 0; i < R * D; ++i) X[i] = (float)unif();
  for (int j = 0; j < D; ++j) { s[j] = (float)(0.5 + 0.1 * j); v[j] = (float)(0.1 * unif()); }
  for (int i = 0; i < R; ++i) yv[i] = (float)unif();
  halp_ref_quantize_data_scaled(X, R, D, 1.0 / 127, s, 8, q8);
  halp_ref_quantize_data_scaled(X, R, D, 1.0 / 32767, s, 16, q16);
  halp_ref_problem p = problem(R, D, 1, HALP_REF_SQUARED, 8, 1, 0.0, 1.0 / 127);
  double phi[R], g[D], loss = 0.0;
  CHECK(halp_ref_full_gradient_scaled(&p, X, D, yv, v, s, phi, g, &loss));
  acc += (uint64_t)q8[0] + (uint64_t)q16[1];
  return acc == 1 ? 2 : 0; /* keeps the calls alive; the sum is never 1 in practice */
}

int main(void) {
  if (run_primitives() != 0) return 1;
  const int H = HALP_REF_ALG_HALP, L = HALP_REF_ALG_LPSVRG;
  /* loss, K, b, B, lambda, algorithm, scalar leg */
  if (run_config(HALP_REF_SQUARED, 1, 8, 1, 0.0, H, HALP_REF_SCALAR_FIXED)) return 1;
  if (run_config(HALP_REF_SQUARED, 1, 16, 4, 1e-2, H, HALP_REF_SCALAR_FIXED)) return 1;
  if (run_config(HALP_REF_LOGISTIC, 1, 8, 3, 1e-3, H, HALP_REF_SCALAR_PLAIN)) return 1;
  if (run_config(HALP_REF_LOGISTIC, 1, 24, 1, 0.0, H, HALP_REF_SCALAR_FIXED)) return 1;
  if (run_config(HALP_REF_SOFTMAX, 5, 8, 1, 1e-3, H, HALP_REF_SCALAR_FIXED)) return 1;  /* a softmax epoch */
  if (run_config(HALP_REF_SOFTMAX, 16, 16, 2, 0.0, H, HALP_REF_SCALAR_PLAIN)) return 1;
  if (run_config(HALP_REF_SQUARED, 1, 8, 1, 0.0, L, HALP_REF_SCALAR_FIXED)) return 1;   /* an LP-SVRG epoch */
  if (run_config(HALP_REF_LOGISTIC, 1, 16, 2, 0.0, L, HALP_REF_SCALAR_FIXED)) return 1;
  if (run_config(HALP_REF_SOFTMAX, 3, 8, 1, 0.0, L, HALP_REF_SCALAR_FIXED)) return 1;
  puts("ok");
  return 0;
}
