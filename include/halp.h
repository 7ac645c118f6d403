/*
 * halp.h -- C ABI of the MI355X (gfx950) HALP epoch library.
 *
 * The library runs the epoch of HALP for linear models (De Sa et al.,
 * "High-Accuracy Low-Precision Training", arXiv 1803.03383, Algorithm 4,
 * "LM-HALP") on one GPU for R independent chains at once:
 *
 *   1. full-precision pass   phi_i = x_i^T w~,  g~ = (1/N) sum_i l_i'(phi_i) x_i
 *   2. bit centering         delta_m = ||g~|| / (mu (2^(b-1) - 1)), the two
 *                            derived scales, h~ = Q(alpha g~), z = 0
 *   3. T low-precision inner steps on the integer offset z
 *   4. w~ <- w~ + delta_m z  (option I)
 *
 * The problem is the finite sum of the paper's eq. (1) with linear-model terms
 * f_i(w) = l_i(x_i^T w) (+ lambda/2 ||w||^2) (Sec. 4, "Efficient implementation").
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library
 *     never frees or reallocates caller memory.  Strides are in elements.
 *   - Every call that takes a stream is asynchronous on that hipStream_t
 *     (passed as void*; NULL is the default stream).  halp_create,
 *     halp_destroy, halp_bind, halp_set_option and halp_get_stats are host
 *     calls; halp_get_stats synchronizes the stream it is given.
 *   - Return value: 0 on success, a negative HALP_ERR_* otherwise.  Nothing is
 *     launched when an error is returned.  Conditions only the device can see
 *     (a zero or non-finite gradient) are reported through scales[7] and
 *     halp_get_stats, and turn the rest of that epoch into a no-op.
 *   - A handle is not thread-safe; distinct handles are independent.  There is
 *     no global state.
 *   - All randomness is counter-based (Philox4x32-10): each draw is a pure
 *     function of (seed + chain, epoch, step, purpose, position), so a run can
 *     be resumed from (w~, epoch, seed) alone and replayed on a CPU.
 */
#ifndef HALP_H
#define HALP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HALP_OK 0
#define HALP_ERR_NULL (-1)        /* a required pointer is NULL                         */
#define HALP_ERR_INVALID (-2)     /* a parameter is out of range                        */
#define HALP_ERR_UNSUPPORTED (-3) /* valid, but no kernel covers this shape             */
#define HALP_ERR_NOT_BOUND (-4)   /* halp_bind has not been called / lacks a buffer     */
#define HALP_ERR_HIP (-5)         /* a HIP runtime call failed                          */
#define HALP_ERR_ALIGN (-6)       /* pointer or stride alignment requirement not met    */
#define HALP_ERR_TOO_LARGE (-7)   /* beyond the fixed scratch of halp_full_gradient_static */
#define HALP_ERR_EXCHANGE_TIMEOUT (-8) /* halp_get_stats: a cross-workgroup wait of the split
                                     minibatch inner loop ran out; that chain's w~ was left as
                                     it was before the loop (status -2)                    */

/* scalar loss l_i of the linear model (Sec. 4); labels y as noted */
#define HALP_LOSS_SQUARED 0  /* l(a) = (a - y)^2 / 2,        y: float               */
#define HALP_LOSS_LOGISTIC 1 /* l(a) = log(1 + exp(-y a)),   y: float in {-1,+1}    */
#define HALP_LOSS_SOFTMAX 2  /* l(a) = -log softmax(a)_y,    y: int32 in [0,K)      */

/* Which of the paper's algorithms an epoch runs.  HALP_ALG_LPSVRG is Algorithm 2 for linear
 * models in the integer form the paper mentions after Algorithm 4: the model itself is the
 * integer vector z (scale delta, b bits, box around 0); halp_recenter then takes the scales
 * from delta instead of ||g~|| and sets z = round(w~ / delta); the inner loop uses
 * beta = alpha (l'(x_i^T z delta_d delta) - l'(phi_i)); an epoch ends with w~ = delta z.
 * lambda must be 0 in that mode; mu is ignored.                                          */
#define HALP_ALG_HALP 0
#define HALP_ALG_LPSVRG 1
/* HALP_ALG_SVRG is Algorithm 1, full-precision SVRG, for squared and logistic loss with one
 * row per step: the comparator of the paper's Table 3.  An epoch is halp_full_gradient and
 * then T steps  w <- w - alpha ((l'(x_i^T w) - l'(phi_i)) x_i + lambda (w - w~) + g~)  on the
 * fp32 data X with the same index stream as the other two; w~ <- w_T.  It needs X, y, w,
 * phi, g only; halp_recenter is not part of it (HALP_ERR_INVALID); b, mu, delta_d are unused. */
#define HALP_ALG_SVRG 2

typedef struct halp_handle halp_handle; /* opaque, library-owned */

/* The "given" lists of Algorithm 4 plus the problem sizes of eq. (1). */
typedef struct {
  int64_t N;          /* examples per chain, 1 <= N < 2^31                             */
  int32_t d;          /* features, >= 1 (gradient pass: <= 16384 for one-class losses)      */
  int32_t K;          /* classes: 1 for squared / logistic, 2..16 for softmax          */
  int32_t R;          /* independent chains (seeds / problem instances), >= 1          */
  int32_t loss;       /* HALP_LOSS_*                                                   */
  int32_t b;          /* bits of z, gamma and the data: 8 or 16                        */
  int32_t B;          /* inner minibatch (rows per step), >= 1                         */
  int32_t share_data; /* 0: each chain has its own X, Xq, y; 1: all chains share one   */
  int32_t algorithm;  /* HALP_ALG_HALP (Algorithm 4) or HALP_ALG_LPSVRG (Algorithm 2)  */
  int64_t T;          /* inner steps per epoch, 0 <= T < 2^32                          */
  double alpha;       /* step size, > 0                                                */
  double mu;          /* strong-convexity parameter of bit centering, > 0              */
  double lambda;      /* L2 coefficient, >= 0                                          */
  double delta_d;     /* scale of the low-precision data representation (delta_d, b)   */
  uint64_t seed;      /* chain r draws with seed + r                                   */
  double delta;       /* HALP_ALG_LPSVRG: the fixed scale of the model (delta, b), > 0 */
} halp_params;

/* Device buffers.  Rd = 1 if share_data else R.  "in" = read by the library,
 * "out" = written, both relative to a whole halp_epoch.                              */
typedef struct {
  const float* X;     /* in   [Rd][N][ldx] fp32 examples, ldx >= d, ldx % 4 == 0, 16-byte aligned */
  int64_t ldx;
  void* Xq;           /* in (out of halp_quantize_data) [Rd][N][ldxq] int8 (b=8) / int16 (b=16);
                         row stride a multiple of 8 bytes, base 8-byte aligned          */
  int64_t ldxq;
  const void* y;      /* in   [Rd][N] float or int32, see HALP_LOSS_*; may be NULL for squared loss
                         if halp_full_gradient is never called                          */
  float* w;           /* in/out [R][K][d] the full-precision model w~                   */
  float* phi;         /* out  [R][N][K] margins x_i^T w~ of the last full-gradient pass */
  float* g;           /* out  [R][K][d] full gradient g~                                */
  void* z;            /* out  [R][K][d] int8 / int16 offset in (delta_m, b)             */
  void* h;            /* out  [R][K][d] int16 / int32 h~ in (delta_i, 2b)               */
  double* scales;     /* out  [R][8]: delta_m, delta_i, delta_s, ||g~||, 1/delta_i, 1/delta_s,
                         f(w~), status (0 ok, 1 gradient exactly zero, -1 not finite, -2 a wait
                         between the workgroups of the split minibatch loop ran out: w~ was not
                         updated)                                                       */
  uint64_t* counters; /* out  [R][4]: coordinates of z clamped by the last inner loop, gammas
                         clamped, steps with a non-zero L2 draw, 1 if a cross-workgroup wait
                         of the split minibatch loop ran out (z is then invalid, w~ is left
                         unchanged and the status becomes -2)                              */
} halp_buffers;

typedef struct {
  double delta_m, delta_i, delta_s, grad_norm, loss;
  int32_t status;         /* 0 ok, 1 converged (gradient exactly zero), -1 gradient not finite,
                             -2 exchange wait ran out (w~ unchanged)                        */
  int32_t inner_variant;  /* kernel that ran the last inner loop: 1 generic, 2 register-resident */
  uint64_t n_clamped_z, n_clamped_gamma, n_reg_draws;
  float ms_full_gradient, ms_recenter, ms_inner_loop; /* mean per halp_epoch over timed_epochs */
  int32_t timed_epochs;   /* halp_epoch calls averaged (the last 32 at most since timing was set) */
  uint64_t n_exchange_timeouts; /* 1 if a cross-workgroup wait of the last split minibatch loop
                             ran out (counters[3]); halp_get_stats then returns
                             HALP_ERR_EXCHANGE_TIMEOUT with every field filled in           */
} halp_stats;

#define HALP_OPT_INNER_VARIANT 1 /* 0 auto (default), 1 general, 2 register-resident.
                                    Register-resident kernels exist for B = 1 with K = 1 (squared,
                                    logistic; d up to 8 strips of 16 rounding bits per lane and
                                    16 waves), for K = 1 with 2 <= B <= 64 (same limit on d), and
                                    for softmax with B = 1 (a class's row of z within 8
                                    strips per lane of one wave at 8 bits, 16 at 16 bits -- 8
                                    at either width for 16 classes, which share waves in
                                    pairs -- and the staged rows within the LDS of a CU), and
                                    for softmax with 2 <= B <= 512 (a class's
                                    row of z within 8 strips per lane at 8 bits, 16 at 16
                                    bits, 64 rows of a step within 128 KB of LDS; the same kernel
                                    takes K = 1 with 64 < B <= 512 on such rows); auto takes
                                    them when the shape fits, 2 fails with HALP_ERR_UNSUPPORTED
                                    when it does not.  HALP_ALG_SVRG has one fp32 kernel and
                                    ignores this option                                      */
#define HALP_OPT_TIMING 2        /* 1: halp_epoch brackets its phases with events on its stream;
                                    setting it restarts the averages of halp_get_stats     */
#define HALP_OPT_FULLGRAD_BLOCKS 4 /* workgroups per chain of the gradient pass, 0 = auto  */
#define HALP_OPT_INNER_WAVES 5   /* waves per chain of the register-resident inner loop: 1, 2, 4,
                                    8, 16, or 0 = auto (several when chains are few, one when
                                    they are many); results do not depend on it             */
#define HALP_OPT_OPTION_II 6     /* 0 (default): option I of Algorithms 1-3, an epoch ends at the
                                    last iterate.  1: option II, the form the theorems are stated
                                    for: chain r draws t uniformly from {0, .., T-1} (word 0 of
                                    stream purpose 5 of that epoch) and the epoch ends at the
                                    iterate after t steps: w~ <- w~ + delta_m z_t                */
#define HALP_OPT_INNER_PARTS 7   /* workgroups per chain of the minibatch (B > 1) register inner
                                    loop.  0 (default): the library's choice, the full-step form
                                    (the row cut across up to 16 workgroups, rows of a step held in
                                    registers) where it applies; 1, 2, 4, 8: the chunked form with
                                    that many workgroups.  The workgroups of a chain meet once per
                                    step in device memory and wait for each other (bounded; a wait
                                    that runs out is reported in counters[3]), so more than one
                                    is only taken when R times the count is at most the number of
                                    CUs, and launches of two handles in that mode should not
                                    overlap.  Results do not depend on it                       */
#define HALP_OPT_EXCHANGE_SPIN_LIMIT 8 /* polls after which a workgroup of the split minibatch
                                    loop stops waiting for the others for good (default 2^20,
                                    about a second); -1: never wait.  The launch then ends
                                    normally with counters[3] = 1, status -2 and w~ unchanged:
                                    for tests of that path                                */

#define HALP_OPT_INNER_PACKED 9  /* register-resident inner loop at 8 bits with one wave per chain:
                                    the form that updates the two coordinates of a strip as packed
                                    16-bit halves.  0 (default): taken when every SIMD holds two
                                    chains or more; 1: wherever that shape is launched; 2: never.
                                    Results do not depend on it                                */
#define HALP_OPT_INNER_HELPERS 10 /* register-resident inner loop with two or four waves per
                                    chain and at most two strips per lane: a helper wave beside
                                    every chain wave draws the rounding bits, fetches the sampled
                                    rows and refills the step-indexed draws, so that the chain
                                    waves issue the step's dependent chain and little else.
                                    0 (default): taken while a CU holds at most five chains
                                    (four chain waves up to two chains per CU, two beyond);
                                    1: wherever that shape is launched; 2: never; 3: the 8-bit
                                    form with ONE chain wave that holds all of z (two
                                    coordinates per register, packed 16-bit arithmetic) and
                                    helper waves on the other SIMDs of the CU, for rows up to
                                    1024 coordinates (HALP_ERR_UNSUPPORTED elsewhere); 0 takes
                                    it for rows of 129 .. 512 coordinates at up to two chains
                                    per CU and for wider rows at up to one.  Results do not
                                    depend on it                                              */

#define HALP_OPT_EXCHANGE_POLL_DELAY 11 /* split minibatch loop: sleeps of 256 cycles between a
                                    workgroup publishing its sums of a step and its first poll
                                    for the others' (0 .. 64, default 3).  A word needs about
                                    17 such units to cross device memory, but delays of 4 and
                                    more were measured to lengthen the step, so the default
                                    only skips the polls that cannot succeed for free.
                                    Results do not depend on it                                 */
#define HALP_OPT_GRADIENT_FP32 12 /* softmax gradient pass on rows of up to 800 coordinates, a
                                    multiple of 4: 0 (default): both matrix products take every
                                    fp32 operand as the sum of two halves (22 of its 24 bits)
                                    and accumulate in fp32, on the 16-bit path of the matrix
                                    cores; 1: fp32 products.  Both stay within the pass's
                                    1e-5; the first is the faster one                          */

/* Validates p (HALP_ERR_INVALID / HALP_ERR_UNSUPPORTED) and allocates the
 * library's own device workspace on the current device.                               */
int halp_create(halp_handle** out, const halp_params* p);
int halp_destroy(halp_handle* h);

/* Records the caller's buffers (the struct is copied).  Checks alignment and
 * strides.  Any pointer may be NULL if no later call needs it; calls that do
 * return HALP_ERR_NOT_BOUND.  The training set X is taken to stay as it is while bound:
 * bind again after changing it (the softmax gradient pass takes the largest |X| once per
 * bind, on its first call, and later calls reuse it).                                  */
int halp_bind(halp_handle* h, const halp_buffers* buf);

int halp_set_option(halp_handle* h, int32_t option, int64_t value);

/* Per-feature data scales: diagonal preconditioning (the remark after Theorem 2 that low
 * precision should be combined with preconditioning).  s is a DEVICE array of d positive
 * floats owned by the caller (NULL switches it off).  The low-precision data are then
 * x_ij = delta_d s_j q_ij -- halp_quantize_data writes q_ij = round(X_ij / (delta_d s_j)) --
 * and every algorithm runs unchanged on q and the scaled model v_j = s_j w_j: the buffer w
 * holds v (the caller divides by s to read the model); halp_full_gradient forms
 * w_j = v_j / s_j for the margins and hands on d f / d v_j = g_j / s_j in g.  lambda must be
 * 0 (HALP_ERR_UNSUPPORTED otherwise, and for HALP_ALG_SVRG).                          */
int halp_set_feature_scale(halp_handle* h, const float* s);

/* Step size and mu per chain, for grids of hyper-parameters run as independent chains (the
 * paper's conditioning study, Appendix "Conditioning Evaluation", searches both).  alpha and
 * mu are HOST arrays of R entries, copied synchronously into the library's device workspace;
 * a NULL array means the value of halp_params for every chain.  Chain r then runs Algorithm
 * 4 (or 2, or 1) with alpha[r] and mu[r] in place of the two parameters, everything else
 * as before.  Not to be called while work of this handle is in flight.                   */
int halp_set_chain_hyper(halp_handle* h, const double* alpha, const double* mu);

/* Data in the low-precision representation (delta_d, b) that Algorithm 4 is
 * given: Xq = clamp(round-half-even(X / delta_d), -(2^(b-1)-1), 2^(b-1)-1).
 * Needs X, Xq.                                                                        */
int halp_quantize_data(halp_handle* h, void* stream);

/* Algorithm 4, outer lines: phi_i = x_i^T w~ for every example and
 * g~ = (1/N) sum_i l_i'(phi_i) x_i + lambda w~, in fp32 with X read once;
 * also f(w~) into scales[6].  Needs X, y, w, phi, g, scales.  Softmax on rows of up to 800
 * coordinates: see HALP_OPT_GRADIENT_FP32; the first call after a halp_bind also makes one
 * more pass over X on the stream, for its largest magnitude.                            */
int halp_full_gradient(halp_handle* h, void* stream);

/* halp_full_gradient for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  No handle (halp_create
 * allocates): the parameters and the caller's buffers are passed directly, with the meaning,
 * layout and alignment rules of halp_params / halp_buffers (needs X, ldx, y, w, phi, g, scales;
 * T, B, b, mu, delta_d, seed are not used).  The per-workgroup partial sums that
 * halp_full_gradient keeps in workspace from halp_create live here in a fixed device array of
 * HALP_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends;
 * its address is looked up on the first call on a device.  The call itself allocates and frees
 * nothing.  Fewer workgroups per chain are launched when their partials would not fit
 * (results agree to rounding; bandwidth drops); when R (4 K d + 8) bytes, one workgroup per
 * chain, exceed the array the call fails with HALP_ERR_TOO_LARGE.  No per-feature scales.
 * All calls on one GPU share the array: calls that overlap in time on one GPU (two streams,
 * two threads) race and give wrong sums -- order them.  Nothing needs clearing between calls:
 * every launch overwrites the part it reads.                                              */
#define HALP_STATIC_SCRATCH_BYTES (16u << 20)
int halp_full_gradient_static(const halp_params* p, const halp_buffers* buf, void* stream);

/* Algorithm 4, the re-scale lines (bit centering, Sec. 4): from g~ computes
 * delta_m = ||g~||_2 / (mu (2^(b-1)-1)), delta_i = 2^-b delta_m,
 * delta_s = delta_i / delta_d, h~ = Q_(delta_i,2b)(alpha g~) and z = 0.
 * epoch < 2^32 selects the random stream.  Needs g, h, z, scales.                     */
int halp_recenter(halp_handle* h, int64_t epoch, void* stream);

/* Algorithm 4, inner loop: T steps of  sample i; beta = alpha (l_i'(phi_i +
 * x_i^T z) - l_i'(phi_i)); gamma = Q_(delta_s,b)(beta); u = z - gamma x_i - h~;
 * z = Q_(delta_m,b)(u)  in integer arithmetic, then w~ <- w~ + delta_m z.
 * Needs Xq, phi (not for squared loss), y (logistic only), h, z, scales, w, counters. */
int halp_inner_loop(halp_handle* h, int64_t epoch, void* stream);

/* The three calls above in order: one outer iteration of Algorithm 4.                 */
int halp_epoch(halp_handle* h, int64_t epoch, void* stream);

/* Debug form of halp_inner_loop (generic kernel): additionally records the
 * first M steps of every chain.  Any trace pointer may be NULL.
 *   idx   int64  [R][M][B]      sampled example indices
 *   D     int64  [R][M][B][K]   integer dot products x_i^T z
 *   beta  double [R][M][B][K]
 *   gamma int32  [R][M][B][K]
 *   ztraj int32  [R][M][K][d]   z after each step                                      */
int halp_inner_loop_trace(halp_handle* h, int64_t epoch, int64_t M, int64_t* idx, int64_t* D,
                          double* beta, int32_t* gamma, int32_t* ztraj, void* stream);

/* Synchronizes stream, then reads chain r's scales and counters.  Returns
 * HALP_ERR_EXCHANGE_TIMEOUT (out is still filled in) when that chain's last inner loop gave up
 * a wait between its workgroups.                                                       */
int halp_get_stats(halp_handle* h, int32_t chain, void* stream, halp_stats* out);

/* Debug: words n0 .. n0+count-1 of a purpose's random stream (purposes: 0 index,
 * 1 gamma, 3 L2, 4 h~, 5 option II), and the b rounding bits of every coordinate [K][d] of z at
 * step t (purpose 2), written as uint32 to device memory.                             */
int halp_debug_stream_words(uint64_t seed, uint32_t purpose, uint32_t epoch, uint64_t n0,
                            int64_t count, uint32_t* out, void* stream);
int halp_debug_zround_bits(uint64_t seed, uint32_t epoch, uint64_t t, int32_t d, int32_t b,
                           int32_t K, uint32_t* out, void* stream);

/* Measurement aid, not part of the method: one kernel that reads `bytes` (a multiple of 16,
 * 16-byte aligned DEVICE memory) exactly once with the load pattern of the gradient pass and
 * writes 2048 uint32 partial checksums to out (DEVICE).  Timed over the example matrix it is
 * the read-only bandwidth this GPU reaches, the yardstick beside the published HBM peak.  */
int halp_debug_read_bandwidth(const void* p, int64_t bytes, uint32_t* out, void* stream);

/* Measurement aid, not part of the method: the dependent chain of one 8-bit inner-loop step
 * (Algorithm 4, inner `for t`, one sampled row, two coordinates per lane) with nothing beside
 * it: multiply-adds, DPP fold, one LDS word per wave and a barrier, the fp64 path of gamma, the
 * update.  `blocks` workgroups (1 .. 65535) of `waves` waves (2 or 4) run `steps` steps (a
 * multiple of 8, >= 8) on lane constants; out (DEVICE) receives blocks * waves * 64 uint32.
 * Its time per step is the latency floor of the several-wave register kernels when a CU holds
 * one chain.  `waves` = 1: the chain of the form with one chain wave instead (a row of 512
 * coordinates, four strips per lane on packed 16-bit halves: packed dots, DPP fold, fp64 path,
 * packed update, one LDS store of the unclamped strips; records read from an LDS ring, one
 * barrier per 8 steps): the floor of that form.                                           */
int halp_debug_step_latency(int32_t waves, int64_t steps, int32_t blocks, uint32_t* out,
                            void* stream);

const char* halp_strerror(int code);
/* Text of the last HIP runtime failure seen by this thread inside the library
 * (which call, and HIP's message); empty if there was none.                            */
const char* halp_last_error_detail(void);
const char* halp_version(void);

#ifdef __cplusplus
}
#endif
#endif
