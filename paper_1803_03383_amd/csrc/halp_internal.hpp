// Host-side context of a handle and the launchers each kernel file exports.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/halp.h"

struct halp_handle {
  halp_params p;
  halp_buffers buf;
  bool bound = false;
  int device = 0;
  int num_cus = 256;
  // options
  int inner_variant = 0;
  bool timing = false;
  int fullgrad_blocks = 0;
  bool option2 = false; // option II of Algorithms 1-3 for the end of an epoch
  int inner_waves = 0;  // waves per chain of the register-resident inner loop, 0 = auto
  int inner_helpers = 0;  // helper waves beside the chain waves of that loop: 0 auto, 1 wherever built, 2 never
  int inner_packed = 0;  // packed 8-bit form of that loop: 0 auto, 1 wherever it exists, 2 never
  // library-owned workspace of the gradient pass: per-workgroup partial sums
  float* partial_g = nullptr;    // [R][parts][K*d]
  double* partial_loss = nullptr;  // [R][parts]
  int parts = 0;                 // workgroups per chain the workspace was sized for
  int loss_parts = 0;            // partial losses per chain (rows of partial_loss are max(parts, loss_parts) long)
  float* resid = nullptr;        // [R][N][16] residuals of the two-pass softmax gradient form, or null
  size_t partial_g_bytes = 0;
  // softmax gradient pass with operands in halves: the largest |X| of the bound data
  uint32_t* xabsmax = nullptr;   // one word (device), where that form exists for the shape
  bool xabsmax_fresh = false;    // taken since the last halp_bind
  bool gradient_fp32 = false;    // HALP_OPT_GRADIENT_FP32
  const float* fscale = nullptr; // caller's per-feature data scales [d] (device), or null
  // minibatch inner loop split over several workgroups per chain: partial dots and tags
  long long* batch_xbuf = nullptr;   // [R][2][kBatchSlots][64] tagged partial dots, margins and labels
  int inner_parts = 0;               // workgroups per chain of that kernel, 0 = auto
  int poll_delay = 3;                // 256-cycle sleeps between publishing a step's sums and the first poll
  int spin_limit = 1 << 20;          // polls before a workgroup stops waiting for the others
  double* hyper = nullptr;       // [R][2] step size and mu of each chain (device)
  int32_t* zh_work = nullptr;    // general inner kernel: z and h~ of models too large for LDS
  int last_inner_variant = 0;
  // timing: a ring of event quadruples, one per halp_epoch call since timing was switched on
  static constexpr int kTimedEpochs = 32;
  hipEvent_t ev[kTimedEpochs][4] = {};
  int64_t timed = 0;
};

namespace halp {

constexpr int kBatchMaxParts = 16;
constexpr int kBatchSlots = kBatchMaxParts + 2;  // exchange words per row, step parity and chain: the parts' sums, margin, label  // workgroups per chain of the minibatch inner loop at most

struct TraceBufs {
  int64_t M = 0;
  int64_t* idx = nullptr;
  int64_t* D = nullptr;
  double* beta = nullptr;
  int32_t* gamma = nullptr;
  int32_t* ztraj = nullptr;
};

// each returns HALP_OK or a HALP_ERR_* and launches nothing on error
int launch_quantize_data(const halp_handle& h, hipStream_t s);
int fullgrad_supported(const halp_params& p);
int fullgrad_parts(const halp_handle& h);  // workgroups per chain for this shape
int fullgrad_loss_parts(const halp_handle& h);
bool fullgrad_needs_resid(const halp_params& p);
// true where the softmax pass can take its operands in halves, given the largest |X| of the data
bool fullgrad_softmax_wants_absmax(int d);
int launch_full_gradient(const halp_handle& h, hipStream_t s);
// what the pass needs once per bound data set (the largest |X| for the softmax form in halves)
int prepare_full_gradient(halp_handle& h, hipStream_t s);
// the same pass with its workspace in the library's fixed device array: no allocation
int launch_full_gradient_static(const halp_params& p, const halp_buffers& buf, hipStream_t s);
int launch_recenter(const halp_handle& h, uint32_t epoch, hipStream_t s);
int inner_reg_supported(const halp_params& p);
int launch_inner_reg(const halp_handle& h, uint32_t epoch, hipStream_t s);
int inner_softmax_supported(const halp_handle& h);
int launch_inner_softmax(const halp_handle& h, uint32_t epoch, hipStream_t s);
int inner_softmax_batch_supported(const halp_handle& h);  // softmax with a minibatch
int launch_inner_softmax_batch(const halp_handle& h, uint32_t epoch, hipStream_t s);
int inner_generic_supported(const halp_params& p);
bool inner_generic_needs_workspace(const halp_params& p);
size_t inner_generic_workspace_bytes(const halp_params& p);
int launch_inner_generic(const halp_handle& h, uint32_t epoch, const TraceBufs& tr, hipStream_t s);
int inner_batch_supported(const halp_handle& h);
int launch_inner_batch(const halp_handle& h, uint32_t epoch, hipStream_t s);
int inner_svrg_supported(const halp_handle& h);
int launch_inner_svrg(const halp_handle& h, uint32_t epoch, hipStream_t s);
int launch_debug_stream_words(uint64_t seed, uint32_t purpose, uint32_t epoch, uint64_t n0,
                              int64_t count, uint32_t* out, hipStream_t s);
constexpr int kDebugReadBlocks = 2048;  // workgroups (and partial sums) of the read yardstick
int launch_debug_read(const void* p, int64_t bytes, uint32_t* out, hipStream_t s);
int launch_debug_step_latency(int waves, int64_t steps, int blocks, uint32_t* out, hipStream_t s);
int launch_debug_zround_bits(uint64_t seed, uint32_t epoch, uint64_t t, int32_t d, int32_t b,
                             int32_t K, uint32_t* out, hipStream_t s);

inline int hip_ok(hipError_t e) { return e == hipSuccess ? HALP_OK : HALP_ERR_HIP; }

}  // namespace halp
