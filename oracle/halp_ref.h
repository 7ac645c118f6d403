/*
 * halp_ref.h -- CPU oracle for the HALP epoch (De Sa et al., "High-Accuracy
 * Low-Precision Training", arXiv 1803.03383).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded reference
 * written from the paper.  Only the test-suite, the smoke check and the
 * benchmark's "cpu_baseline" leg may load it.  It shares no code, header,
 * table or helper with the HIP library, and the HIP library never calls it.
 *
 * What it follows:
 *   - Sec. 3 "Representation" / "Quantization": dom(delta,b) and the unbiased
 *     quantizer Q_(delta,b); up/down probabilities as in the proof of Lemma 1.
 *   - Sec. 4 "Bit centering" and Algorithm 3 (HALP): delta = ||g~||/(mu(2^(b-1)-1)).
 *   - Sec. 4 "Efficient implementation" and Algorithm 4 (LM-HALP): the cached
 *     margins phi, the three compatible scales delta_m, delta_i, delta_s, the
 *     quantized scalar gamma and the integer update of the offset z.
 *
 * Floating point is fp64 throughout; integers are exact (int64 inside).
 * Build with contraction off (-ffp-contract=off) so every fp64 operation
 * below is rounded on its own.
 *
 * Readings of points the paper leaves open (each one is also listed in the
 * repository's design notes):
 *   - h~ is held in (delta_i, 2b) as the text after Algorithm 4 says (the
 *     listing's "b" for it is read as a slip).
 *   - the norm is the Euclidean / Frobenius norm.
 *   - real -> integer rounding is floor(x * (1/delta) + rho), rho = r32 * 2^-32
 *     with one 32-bit random word: P(up) equals the fractional part to 2^-32.
 *   - integer (delta_i,2b) -> (delta_m,b) rounding is floor((u + r) / 2^b) with
 *     exactly b random bits r: exactly unbiased.
 *   - random numbers: counter-based Philox4x32-10 (Salmon et al., SC'11);
 *     every draw is a pure function of (seed, purpose, epoch, step, position).
 *   - indices are drawn with replacement, i = floor(r32 * N / 2^32).
 *   - minibatch B > 1: all rows of a step see the same z, each row has its own
 *     gamma, beta carries alpha/B, z is quantized once per step.
 *   - L2 term lambda: outer gradient gets + lambda w~; inner update gets
 *     - c_lambda * z with c_lambda = Q_(2^-b, b)(alpha lambda), one draw per step.
 *   - multiclass: softmax cross-entropy, W stored [K][d], one gamma per class.
 *   - squared loss l(a) = (a-y)^2/2, so beta = (alpha/B) * (x^T z) exactly.
 *   - logistic labels are -1/+1, l(a) = log(1 + exp(-y a)).
 *   - in the inner loop, where the last bit of l' can decide the integer gamma,
 *     exp is a fixed sequence of correctly rounded double operations
 *     (halp_ref_exp, within 1 ulp of exp) and the softmax normaliser is summed
 *     pairwise over adjacent classes; the full-precision pass uses libm and
 *     plain loops.  The plain definition of the same scalar path (libm exp, the
 *     normaliser added from left to right) is the oracle's second leg,
 *     HALP_REF_SCALAR_PLAIN; the two legs are compared step by step in the tests.
 *
 *   - LP-SVRG (Algorithm 2) for linear models, which the paper says can be put in
 *     integers "using a similar technique" without printing it: the model w itself
 *     is the integer vector (scale delta given, b bits, box around 0); an epoch
 *     starts from w = round-to-nearest(w~ / delta), keeps the (delta_i, 2b) and
 *     (delta_s, b) bookkeeping of Algorithm 4 with delta_m = delta,
 *     beta = alpha (l'(x_i^T w) - l'(phi_i)) with x_i^T w the integer product and
 *     phi_i the margin of w~ from the full-precision pass, and ends with
 *     w~ = delta w (option I).  No L2 term in this mode.
 *
 * Parity pins: see tests/test_oracle_*.py.  Unpinned by the paper itself
 * ("parity unpinned" beyond unbiasedness against Algorithm 3 and reduction to
 * the written algorithm at K=1, B=1, lambda=0): the softmax, minibatch and L2
 * readings above.
 */
#ifndef HALP_REF_H
#define HALP_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { HALP_REF_SQUARED = 0, HALP_REF_LOGISTIC = 1, HALP_REF_SOFTMAX = 2 };
enum { HALP_REF_ALG_HALP = 0, HALP_REF_ALG_LPSVRG = 1, HALP_REF_ALG_SVRG = 2 };
/* Two legs of the inner loop's scalar path (Algorithm 4, the beta line).  PLAIN is the
 * definition written out: l' through the C library's exp, the softmax normaliser added class by
 * class from left to right -- the same code as the full-precision pass.  FIXED is the reading
 * that makes the integer gamma reproducible on any IEEE machine (halp_ref_exp, pairwise
 * normaliser); it is what parity with the GPU is held to.  The two differ by rounding only;
 * tests/test_oracle_scalar_legs.py measures how often that moves a gamma.                    */
enum { HALP_REF_SCALAR_FIXED = 0, HALP_REF_SCALAR_PLAIN = 1 };

/* purposes of the random streams (counter word 3) */
enum {
  HALP_REF_PURPOSE_IDX = 0,    /* sampled example indices            */
  HALP_REF_PURPOSE_GAMMA = 1,  /* rounding of the scalar beta         */
  HALP_REF_PURPOSE_ZROUND = 2, /* rounding of the offset vector z     */
  HALP_REF_PURPOSE_REG = 3,    /* rounding of alpha*lambda            */
  HALP_REF_PURPOSE_HROUND = 4, /* rounding of alpha*g~ into h~        */
  HALP_REF_PURPOSE_OPT2 = 5    /* option II: where an epoch ends      */
};

typedef struct {
  int64_t N;      /* examples                                         */
  int32_t d;      /* features                                         */
  int32_t K;      /* classes (1 unless softmax)                       */
  int32_t loss;   /* HALP_REF_*                                       */
  int32_t b;      /* bits of the low-precision model: 8 or 16 (up to 24 on the CPU only) */
  int32_t B;      /* inner minibatch                                  */
  int32_t algorithm; /* HALP_REF_ALG_HALP (Algorithm 4) or HALP_REF_ALG_LPSVRG (Algorithm 2) */
  double alpha;   /* step size                                        */
  double mu;      /* strong-convexity parameter used by bit centering */
  double lambda;  /* L2                                               */
  double delta_d; /* scale of the low-precision data (delta_d, b)     */
  uint64_t seed;  /* seed of this chain                               */
  double delta;   /* LP-SVRG only: the fixed scale of the model (delta, b) */
  int32_t scalar_path; /* how the inner loop evaluates l': HALP_REF_SCALAR_FIXED (0, the
                          reproducible reading) or HALP_REF_SCALAR_PLAIN (1, the definition) */
} halp_ref_problem;

/* optional per-step record of the first M steps; any pointer may be NULL */
typedef struct {
  int64_t M;
  int64_t* idx;    /* [M][B]        sampled indices                   */
  int64_t* D;      /* [M][B][K]     integer dot products x^T z         */
  double* beta;    /* [M][B][K]                                        */
  int32_t* gamma;  /* [M][B][K]                                        */
  int32_t* ztraj;  /* [M][K][d]     z after the step                   */
  /* what the other leg of the scalar path (see HALP_REF_SCALAR_*) gives at the same state z,
   * the same sampled row and the same rounding draw; the trajectory follows p->scalar_path  */
  double* beta_other;   /* [M][B][K] */
  int32_t* gamma_other; /* [M][B][K] */
} halp_ref_trace;

/* scales[8]: 0 delta_m, 1 delta_i, 2 delta_s, 3 ||g~||, 4 1/delta_i,
 * 5 1/delta_s, 6 f(w~) (filled by the epoch driver), 7 status
 * (0 ok, 1 gradient is exactly zero: converged, -1 non-finite).           */

/* Philox4x32-10, Salmon et al. SC'11 */
void halp_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* word n of a purpose's stream: Philox block n/4, word n%4,
 * counter = (lo32(n/4), hi32(n/4), epoch, purpose), key = (lo32 seed, hi32 seed) */
uint32_t halp_ref_stream_word(uint64_t seed, uint32_t purpose, uint32_t epoch, uint64_t n);

/* Option II of Algorithms 1-3: t uniform on {0, .., T-1}; the epoch ends at the iterate after
 * t steps (t = 0: the outer iterate does not move).  Word 0 of the purpose's stream of that
 * epoch, mapped like the sample indices.  The caller runs the inner loop for t steps.       */
int64_t halp_ref_option2_steps(uint64_t seed, uint32_t epoch, int64_t T);

/* the b rounding bits of coordinate (c,j) at 0-based step t */
uint32_t halp_ref_zround_bits(uint64_t seed, uint32_t epoch, uint64_t t, int32_t d, int32_t b,
                              int32_t c, int32_t j);

/* index of minibatch slot m at 0-based step t */
int64_t halp_ref_sample_index(uint64_t seed, uint32_t epoch, uint64_t t, int32_t B, int32_t m,
                              int64_t N);

/* Q for a real: clamp(floor(x * inv_delta + r32 * 2^-32), lo, hi); clamped!=NULL gets 1 if it hit a bound */
int64_t halp_ref_quantize_real(double x, double inv_delta, uint32_t r32, int64_t lo, int64_t hi,
                               int* clamped);

/* Q_(delta_m,b) of u = (z << b) + v held in (delta_i, 2b): clamp(z + floor((v + r) / 2^b)) */
int64_t halp_ref_round_shift(int64_t z, int64_t v, uint32_t r, int b, int* clamped);

/* exp as the inner loop evaluates it (see the readings above); n values at once */
double halp_ref_exp(double x);
void halp_ref_exp_array(const double* x, int64_t n, double* out);

/* X -> (delta_d, b): clamp(round-half-even(X / delta_d), -(2^(b-1)-1), 2^(b-1)-1);
 * Xq is int8 when b == 8, int16 when b == 16, int32 for 16 < b <= 24 (CPU only) */
void halp_ref_quantize_data(const float* X, int64_t n, double delta_d, int b, void* Xq);

/* Per-feature scales (diagonal preconditioning; the remark after Theorem 2 that low precision
 * should be combined with preconditioning).  The data are represented as x_ij = delta_d s_j q_ij
 * and the algorithm runs unchanged on q and the scaled model v_j = s_j w_j: the margins are the
 * same, x_i^T w = delta_d q_i^T v, and the gradient with respect to v is g_j / s_j.
 *   quantize:  q_ij = clamp(round-half-even(X_ij / (delta_d s_j)))          (rows x d, dense)
 *   gradient:  w_j = fp32(v_j / s_j), then the plain pass, then g_j / s_j;  lambda must be 0 */
void halp_ref_quantize_data_scaled(const float* X, int64_t rows, int32_t d, double delta_d,
                                   const float* s, int b, void* Xq);
int halp_ref_full_gradient_scaled(const halp_ref_problem* p, const float* X, int64_t ldx,
                                  const void* y, const float* v, const float* s, double* phi,
                                  double* g, double* loss);

/* Algorithm 2 in integers, start of an epoch: scales from the fixed p->delta
 * (delta_m = delta), h~ = Q_(delta_i,2b)(alpha g~), z = clamp(rne(w~ / delta)).
 * Same scales[] layout and status codes as halp_ref_recenter.               */
int halp_ref_lp_begin(const halp_ref_problem* p, const float* g, const float* w, uint32_t epoch,
                      double scales[8], int64_t* h, int32_t* z);

/* Algorithm 1 (SVRG), inner loop for a linear model in fp64, B rows per step averaged:
 *   w <- w - alpha ( (1/B) sum_m (l'(x_m^T w) - l'(phi_m)) x_m + lambda (w - w~) + g~ )
 * over T steps with the index stream of the other algorithms (squared or logistic loss, K = 1).
 * w (double, [d]) enters as w~ and leaves as w_T; phi are the margins of w~, g is g~.     */
int halp_ref_svrg_inner(const halp_ref_problem* p, const float* X, int64_t ldx, const void* y,
                        const float* phi, const float* g, uint32_t epoch, int64_t T, double* w);

/* Algorithm 4, the two outer lines: margins phi_i = x_i^T w~ and
 * g~ = (1/N) sum l'_i(phi_i) x_i (+ lambda w~); loss = f(w~).
 * y: float* for squared / logistic (+-1), int32* for softmax.           */
int halp_ref_full_gradient(const halp_ref_problem* p, const float* X, int64_t ldx, const void* y,
                           const float* w, double* phi, double* g, double* loss);

/* Algorithm 4, the re-scale lines, h~ = Q(alpha g~) and z = Q(0) */
int halp_ref_recenter(const halp_ref_problem* p, const float* g, uint32_t epoch, double scales[8],
                      int64_t* h, int32_t* z);

/* Algorithm 4, the inner loop: T steps on z (in/out) */
int halp_ref_inner_loop(const halp_ref_problem* p, const void* Xq, int64_t ldxq, const float* phi,
                        const void* y, const int64_t* h, const double scales[8], uint32_t epoch,
                        int64_t T, int32_t* z, const halp_ref_trace* trace, uint64_t counters[4]);

/* Algorithm 4, last outer line (option I): w~ <- w~ + delta_m z */
void halp_ref_apply_offset(const halp_ref_problem* p, const double scales[8], const int32_t* z,
                           float* w);

/* one whole epoch: the four calls above in order; phi32 / g32 receive the
 * fp32-rounded margins and gradient that the inner loop consumed           */
int halp_ref_epoch(const halp_ref_problem* p, const float* X, int64_t ldx, const void* Xq,
                   int64_t ldxq, const void* y, float* w, uint32_t epoch, int64_t T, float* phi32,
                   float* g32, double scales[8], int64_t* h, int32_t* z, uint64_t counters[4]);

#ifdef __cplusplus
}
#endif
#endif
