// Kernel arguments shared by the inner-loop kernels (Algorithm 4, inner `for t`).
#pragma once

#include <stdint.h>

#include "halp_internal.hpp"

namespace halp {

struct InArgs {
  const void* Xq;       // [Rd][N][ldxq] int8 / int16
  const float* phi;     // [R][N][K]
  const void* y;        // [Rd][N] float (+-1) for logistic; unused otherwise
  const void* h;        // [R][K][d] int16 / int32
  void* z;              // [R][K][d] int8 / int16
  float* w;             // [R][K][d]
  const double* scales; // [R][8]
  const double* hyper;  // [R][2] step size and mu of each chain
  uint64_t* counters;   // [R][4]
  int32_t* zh_work;     // general kernel: z and h~ of models too large for LDS, [R][2][K d] int32, or null
  int64_t N, ldxq, T;
  int64_t xq_chain_stride, y_chain_stride;  // elements; 0 when chains share the data
  int d, K, B, loss;
  int option2;  // 1: the epoch ends at a uniformly drawn earlier iterate (option II)
  int lp;  // 1: LP-SVRG (Algorithm 2): z is the model itself, the margin is x^T z alone
  double lambda, delta_d;
  uint64_t seed;
  uint32_t epoch;
  TraceBufs tr;
};

inline InArgs make_inner_args(const halp_handle& h, uint32_t epoch) {
  const halp_params& p = h.p;
  InArgs a;
  a.Xq = h.buf.Xq; a.phi = h.buf.phi; a.y = h.buf.y; a.h = h.buf.h; a.z = h.buf.z; a.w = h.buf.w;
  a.scales = h.buf.scales; a.counters = h.buf.counters; a.hyper = h.hyper;
  a.zh_work = nullptr;
  a.N = p.N; a.ldxq = h.buf.ldxq; a.T = p.T;
  a.xq_chain_stride = p.share_data ? 0 : p.N * h.buf.ldxq;
  a.y_chain_stride = p.share_data ? 0 : p.N;
  a.d = p.d; a.K = p.K; a.B = p.B; a.loss = p.loss;
  a.lp = p.algorithm == HALP_ALG_LPSVRG;
  a.option2 = h.option2 ? 1 : 0;
  a.lambda = p.lambda; a.delta_d = p.delta_d;
  a.seed = p.seed; a.epoch = epoch;
  return a;
}

}  // namespace halp
