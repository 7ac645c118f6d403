// Kernel arguments of the full-precision pass (Algorithm 4, outer lines).
#pragma once

#include <stdint.h>

#include "halp_internal.hpp"

namespace halp {

struct FgArgs {
  const float* X;
  const void* y;
  const float* w;
  const float* fscale;  // [d] per-feature data scales s_j, or null: w then holds v_j = s_j w_j
  float* phi;
  float* partial_g;
  double* partial_loss;
  int64_t N, ldx;
  int64_t x_chain_stride, y_chain_stride;  // 0 when chains share the data
  int d, K, parts;
};

// softmax: margins and gradient as two matrix products on the matrix cores
int fullgrad_softmax_supported(const halp_params& p);
int launch_fullgrad_softmax(const FgArgs& a, int R, hipStream_t s);
// true where the pipelined form runs: one workgroup per CU instead of two
bool fullgrad_softmax_pipelined(int d);

}  // namespace halp
