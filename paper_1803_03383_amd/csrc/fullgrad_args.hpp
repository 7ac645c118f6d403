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
  float* resid;         // softmax on wide rows: residuals [R][N][16] between its two passes, or null
  int64_t N, ldx;
  int64_t x_chain_stride, y_chain_stride;  // 0 when chains share the data
  int d, K, parts;
  int loss_parts;       // workgroups that write a partial loss (parts, except where noted)
  // softmax: bits of the largest |X| over the data (one word, device), or null if not known:
  // with it both products of the pass take their operands as pairs of halves
  const uint32_t* xabsmax = nullptr;
};

// softmax: margins and gradient as two matrix products on the matrix cores
int fullgrad_softmax_supported(const halp_params& p);
int launch_fullgrad_softmax(const FgArgs& a, int R, hipStream_t s);
// true where the pipelined form runs: one workgroup per CU instead of two
bool fullgrad_softmax_pipelined(int d);
// *out = bits of the largest |X[r][c]| over rows < rows, columns < d (rows ldx apart); one word, device
int launch_absmax(const float* X, int64_t rows, int d, int64_t ldx, uint32_t* out, hipStream_t s);
// true where the softmax pass keeps a tile of rows on chip (d <= 1024); wider rows take two passes
bool fullgrad_softmax_one_pass(int d);

// rows too wide for a wave (K = 1) or for a tile on chip (softmax)
int fullgrad_k1_wide_max_d();
int fullgrad_k1_wide_rows_per_batch();
int launch_fullgrad_k1_wide(const FgArgs& a, int loss, int R, hipStream_t s);
int launch_fullgrad_softmax_wide(const FgArgs& a, int R, hipStream_t s);
constexpr int kSoftmaxWideBlock = 512;  // columns per workgroup of the second pass

}  // namespace halp
