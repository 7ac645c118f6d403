// C ABI of the library: argument checking, workspace, kernel selection and the
// order of the three phases of an epoch (Algorithm 4).  No arithmetic of the
// method happens on the host.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "halp_internal.hpp"

using namespace halp;

namespace {

// text of the last failed HIP runtime call on this thread, for halp_last_error_detail
thread_local char g_detail[256] = "";

bool hip_fail(hipError_t e, const char* what) {
  if (e == hipSuccess) return false;
  std::snprintf(g_detail, sizeof g_detail, "%s: %s", what, hipGetErrorString(e));
  (void)hipGetLastError();
  return true;
}

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

int check_params(const halp_params& p) {
  if (p.N < 1 || p.N >= (int64_t(1) << 31)) return HALP_ERR_INVALID;
  if (p.d < 1 || p.R < 1 || p.B < 1) return HALP_ERR_INVALID;
  if (p.b != 8 && p.b != 16) return HALP_ERR_UNSUPPORTED;
  if (p.T < 0 || p.T >= (int64_t(1) << 32)) return HALP_ERR_INVALID;
  if (p.loss < HALP_LOSS_SQUARED || p.loss > HALP_LOSS_SOFTMAX) return HALP_ERR_INVALID;
  if (p.loss == HALP_LOSS_SOFTMAX) {
    if (p.K < 2) return HALP_ERR_INVALID;
    if (p.K > 16) return HALP_ERR_UNSUPPORTED;
  } else if (p.K != 1) {
    return HALP_ERR_INVALID;
  }
  if (!(p.alpha > 0) || !std::isfinite(p.alpha)) return HALP_ERR_INVALID;
  if (p.algorithm == HALP_ALG_HALP && (!(p.mu > 0) || !std::isfinite(p.mu))) return HALP_ERR_INVALID;
  if (!(p.lambda >= 0) || !std::isfinite(p.lambda)) return HALP_ERR_INVALID;
  if (!(p.delta_d > 0) || !std::isfinite(p.delta_d)) return HALP_ERR_INVALID;
  if (p.share_data != 0 && p.share_data != 1) return HALP_ERR_INVALID;
  if (p.algorithm < HALP_ALG_HALP || p.algorithm > HALP_ALG_SVRG) return HALP_ERR_INVALID;
  if (p.algorithm == HALP_ALG_SVRG && (p.loss == HALP_LOSS_SOFTMAX || p.B != 1))
    return HALP_ERR_UNSUPPORTED;
  if (p.algorithm == HALP_ALG_LPSVRG) {
    if (!(p.delta > 0) || !std::isfinite(p.delta)) return HALP_ERR_INVALID;
    if (p.lambda != 0) return HALP_ERR_INVALID;  // no L2 term in the integer form of Algorithm 2
  }
  if ((int64_t)p.K * p.d >= (int64_t(1) << 24)) return HALP_ERR_UNSUPPORTED;
  return HALP_OK;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int need(const void* p) { return p ? HALP_OK : HALP_ERR_NOT_BOUND; }

int launch_inner(const halp_handle& h, int variant, uint32_t epoch, hipStream_t s);

// the register-resident family: one kernel for scalar margins, one for softmax
int reg_supported(const halp_handle& h) {
  if (h.p.loss != HALP_LOSS_SOFTMAX && h.p.B > 64) return inner_softmax_batch_supported(h);
  if (h.p.loss != HALP_LOSS_SOFTMAX && h.p.B > 1) return inner_batch_supported(h);
  if (h.p.loss == HALP_LOSS_SOFTMAX && h.p.B > 1) return inner_softmax_batch_supported(h);
  return h.p.loss == HALP_LOSS_SOFTMAX ? inner_softmax_supported(h) : inner_reg_supported(h.p);
}

int launch_reg(const halp_handle& h, uint32_t epoch, hipStream_t s) {
  if (h.p.loss != HALP_LOSS_SOFTMAX && h.p.B > 64) return launch_inner_softmax_batch(h, epoch, s);
  if (h.p.loss != HALP_LOSS_SOFTMAX && h.p.B > 1) return launch_inner_batch(h, epoch, s);
  if (h.p.loss == HALP_LOSS_SOFTMAX && h.p.B > 1) return launch_inner_softmax_batch(h, epoch, s);
  return h.p.loss == HALP_LOSS_SOFTMAX ? launch_inner_softmax(h, epoch, s)
                                       : launch_inner_reg(h, epoch, s);
}

int launch_inner(const halp_handle& h, int variant, uint32_t epoch, hipStream_t s) {
  if (variant == 3) return launch_inner_svrg(h, epoch, s);
  return variant == 2 ? launch_reg(h, epoch, s) : launch_inner_generic(h, epoch, TraceBufs{}, s);
}

int pick_inner_variant(const halp_handle& h) {
  if (h.p.algorithm == HALP_ALG_SVRG) return 3;  // the fp32 SVRG kernel
  if (h.inner_variant == 1) return 1;
  if (h.inner_variant == 2) return 2;
  return reg_supported(h) == HALP_OK ? 2 : 1;
}

int check_epoch(int64_t epoch) {
  return (epoch < 0 || epoch >= (int64_t(1) << 32)) ? HALP_ERR_INVALID : HALP_OK;
}

int need_full_gradient(const halp_handle& h) {
  if (!h.bound) return HALP_ERR_NOT_BOUND;
  if (!h.buf.X || !h.buf.y || !h.buf.w || !h.buf.phi || !h.buf.g || !h.buf.scales)
    return HALP_ERR_NOT_BOUND;
  return fullgrad_supported(h.p);
}

int need_recenter(const halp_handle& h) {
  if (!h.bound) return HALP_ERR_NOT_BOUND;
  if (!h.buf.g || !h.buf.h || !h.buf.z || !h.buf.scales) return HALP_ERR_NOT_BOUND;
  if (h.p.algorithm == HALP_ALG_LPSVRG && !h.buf.w) return HALP_ERR_NOT_BOUND;
  return HALP_OK;
}

int need_inner(const halp_handle& h, int variant) {
  if (!h.bound) return HALP_ERR_NOT_BOUND;
  if (h.p.algorithm == HALP_ALG_SVRG) {
    if (!h.buf.X || !h.buf.y || !h.buf.w || !h.buf.phi || !h.buf.g) return HALP_ERR_NOT_BOUND;
    return inner_svrg_supported(h);
  }
  if (!h.buf.Xq || !h.buf.h || !h.buf.z || !h.buf.scales || !h.buf.w || !h.buf.counters)
    return HALP_ERR_NOT_BOUND;
  if ((h.p.loss != HALP_LOSS_SQUARED || h.p.algorithm == HALP_ALG_LPSVRG) && !h.buf.phi)
    return HALP_ERR_NOT_BOUND;
  if (h.p.loss == HALP_LOSS_LOGISTIC && !h.buf.y) return HALP_ERR_NOT_BOUND;
  if (variant == 2) return reg_supported(h);
  return inner_generic_supported(h.p);  // so that halp_epoch refuses before its first launch
}

}  // namespace

extern "C" {

int halp_create(halp_handle** out, const halp_params* p) {
  if (!out || !p) return HALP_ERR_NULL;
  *out = nullptr;
  int rc = check_params(*p);
  if (rc != HALP_OK) return rc;
  halp_handle* h = new (std::nothrow) halp_handle();
  if (!h) return HALP_ERR_HIP;
  h->p = *p;
  std::memset(&h->buf, 0, sizeof h->buf);
  if (hip_fail(hipGetDevice(&h->device), "hipGetDevice")) { delete h; return HALP_ERR_HIP; }
  int cus = 0;
  if (hip_fail(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device),
               "hipDeviceGetAttribute")) { delete h; return HALP_ERR_HIP; }
  h->num_cus = cus > 0 ? cus : 256;
  // workspace of the gradient pass, if a kernel covers this shape
  if (fullgrad_supported(h->p) == HALP_OK) {
    h->parts = fullgrad_parts(*h);
    h->loss_parts = fullgrad_loss_parts(*h);
    const size_t loss_row = h->parts > h->loss_parts ? h->parts : h->loss_parts;
    h->partial_g_bytes = sizeof(float) * (size_t)p->R * h->parts * (size_t)p->K * p->d;
    if (hip_fail(hipMalloc(reinterpret_cast<void**>(&h->partial_g), h->partial_g_bytes),
                 "hipMalloc(partial_g)") ||
        hip_fail(hipMalloc(reinterpret_cast<void**>(&h->partial_loss),
                           sizeof(double) * (size_t)p->R * loss_row), "hipMalloc(partial_loss)")) {
      halp_destroy(h);
      return HALP_ERR_HIP;
    }
    if (p->loss == HALP_LOSS_SOFTMAX && fullgrad_softmax_wants_absmax(p->d) &&
        hip_fail(hipMalloc(reinterpret_cast<void**>(&h->xabsmax), 256), "hipMalloc(xabsmax)")) {
      halp_destroy(h);
      return HALP_ERR_HIP;
    }
    if (fullgrad_needs_resid(h->p) &&
        hip_fail(hipMalloc(reinterpret_cast<void**>(&h->resid), sizeof(float) * (size_t)p->R * p->N * 16),
                 "hipMalloc(resid)")) {
      halp_destroy(h);
      return HALP_ERR_HIP;
    }
  }
  // exchange buffers of the split minibatch inner loop, where it can apply
  if (p->K == 1 && p->B > 1 && (int64_t)p->R * 2 <= h->num_cus) {
    const size_t slots = (size_t)p->R * 2 * kBatchSlots;
    if (hip_fail(hipMalloc(reinterpret_cast<void**>(&h->batch_xbuf), slots * 64 * sizeof(long long)),
                 "hipMalloc(batch_xbuf)")) { halp_destroy(h); return HALP_ERR_HIP; }
  }
  if (p->algorithm != HALP_ALG_SVRG && inner_generic_supported(*p) == HALP_OK &&
      inner_generic_needs_workspace(*p) &&
      hip_fail(hipMalloc(reinterpret_cast<void**>(&h->zh_work), inner_generic_workspace_bytes(*p)),
               "hipMalloc(zh_work)")) { halp_destroy(h); return HALP_ERR_HIP; }
  // every chain starts with the step size and mu of the parameters
  if (hip_fail(hipMalloc(reinterpret_cast<void**>(&h->hyper), sizeof(double) * 2 * (size_t)p->R),
               "hipMalloc(hyper)")) { halp_destroy(h); return HALP_ERR_HIP; }
  rc = halp_set_chain_hyper(h, nullptr, nullptr);
  if (rc != HALP_OK) { halp_destroy(h); return rc; }
  for (auto& quad : h->ev)
    for (auto& e : quad)
      if (hip_fail(hipEventCreate(&e), "hipEventCreate")) { halp_destroy(h); return HALP_ERR_HIP; }
  *out = h;
  return HALP_OK;
}

int halp_destroy(halp_handle* h) {
  if (!h) return HALP_ERR_NULL;
  if (h->partial_g) (void)hipFree(h->partial_g);
  if (h->partial_loss) (void)hipFree(h->partial_loss);
  if (h->resid) (void)hipFree(h->resid);
  if (h->xabsmax) (void)hipFree(h->xabsmax);
  if (h->hyper) (void)hipFree(h->hyper);
  if (h->zh_work) (void)hipFree(h->zh_work);
  if (h->batch_xbuf) (void)hipFree(h->batch_xbuf);
  for (auto& quad : h->ev)
    for (auto& e : quad)
      if (e) (void)hipEventDestroy(e);
  delete h;
  return HALP_OK;
}

int halp_set_chain_hyper(halp_handle* h, const double* alpha, const double* mu) {
  if (!h) return HALP_ERR_NULL;
  const halp_params& p = h->p;
  std::vector<double> host(2 * (size_t)p.R);
  for (int r = 0; r < p.R; ++r) {
    const double av = alpha ? alpha[r] : p.alpha;
    const double mv = mu ? mu[r] : p.mu;
    if (!(av > 0) || !std::isfinite(av)) return HALP_ERR_INVALID;
    if (p.algorithm == HALP_ALG_HALP && (!(mv > 0) || !std::isfinite(mv))) return HALP_ERR_INVALID;
    host[2 * (size_t)r] = av;
    host[2 * (size_t)r + 1] = mv;
  }
  if (hip_fail(hipMemcpy(h->hyper, host.data(), sizeof(double) * host.size(), hipMemcpyHostToDevice),
               "hipMemcpy(hyper)"))
    return HALP_ERR_HIP;
  return HALP_OK;
}

int halp_set_feature_scale(halp_handle* h, const float* s) {
  if (!h) return HALP_ERR_NULL;
  if (s) {
    // lambda ||w||^2 is not uniform in the scaled model; Algorithm 1 here works on X and w directly
    if (h->p.lambda != 0 || h->p.algorithm == HALP_ALG_SVRG) return HALP_ERR_UNSUPPORTED;
    if (!aligned(s, 4)) return HALP_ERR_ALIGN;
  }
  h->fscale = s;
  return HALP_OK;
}

int halp_bind(halp_handle* h, const halp_buffers* b) {
  if (!h || !b) return HALP_ERR_NULL;
  const halp_params& p = h->p;
  if (b->X) {
    if (b->ldx < p.d) return HALP_ERR_INVALID;
    if (b->ldx % 4 != 0 || !aligned(b->X, 16)) return HALP_ERR_ALIGN;
  }
  if (b->Xq) {
    if (b->ldxq < p.d) return HALP_ERR_INVALID;
    const int64_t row_bytes = b->ldxq * (p.b / 8);
    if (row_bytes % 8 != 0 || !aligned(b->Xq, 8)) return HALP_ERR_ALIGN;
    // the last 8-byte group of a row must lie inside the row
    const int cpg = 64 / p.b;
    if (((p.d + cpg - 1) / cpg) * 8 > row_bytes) return HALP_ERR_ALIGN;
  }
  if ((b->w && !aligned(b->w, 4)) || (b->phi && !aligned(b->phi, 4)) || (b->g && !aligned(b->g, 4)) ||
      (b->scales && !aligned(b->scales, 8)) || (b->counters && !aligned(b->counters, 8)) ||
      (b->h && !aligned(b->h, 4)) || (b->z && !aligned(b->z, 2)))
    return HALP_ERR_ALIGN;
  h->buf = *b;
  h->bound = true;
  h->xabsmax_fresh = false;
  return HALP_OK;
}

int halp_set_option(halp_handle* h, int32_t option, int64_t value) {
  if (!h) return HALP_ERR_NULL;
  switch (option) {
    case HALP_OPT_INNER_VARIANT:
      if (value < 0 || value > 2) return HALP_ERR_INVALID;
      h->inner_variant = (int)value;
      return HALP_OK;
    case HALP_OPT_TIMING:
      h->timing = value != 0;
      h->timed = 0;
      return HALP_OK;
    case HALP_OPT_INNER_PARTS:
      if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return HALP_ERR_INVALID;
      h->inner_parts = (int)value;
      return HALP_OK;
    case HALP_OPT_EXCHANGE_SPIN_LIMIT:
      if (value < -1 || value > (int64_t(1) << 30)) return HALP_ERR_INVALID;
      h->spin_limit = (int)value;
      return HALP_OK;
    case HALP_OPT_EXCHANGE_POLL_DELAY:
      if (value < 0 || value > 64) return HALP_ERR_INVALID;
      h->poll_delay = (int)value;
      return HALP_OK;
    case HALP_OPT_OPTION_II:
      if (value != 0 && value != 1) return HALP_ERR_INVALID;
      h->option2 = value != 0;
      return HALP_OK;
    case HALP_OPT_INNER_PACKED:
      if (value < 0 || value > 2) return HALP_ERR_INVALID;
      h->inner_packed = (int)value;
      return HALP_OK;
    case HALP_OPT_INNER_HELPERS:
      if (value < 0 || value > 3) return HALP_ERR_INVALID;
      h->inner_helpers = (int)value;
      return HALP_OK;
    case HALP_OPT_GRADIENT_FP32:
      if (value != 0 && value != 1) return HALP_ERR_INVALID;
      h->gradient_fp32 = value != 0;
      return HALP_OK;
    case HALP_OPT_INNER_WAVES:
      if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8 && value != 16)
        return HALP_ERR_INVALID;
      h->inner_waves = (int)value;
      return HALP_OK;
    case HALP_OPT_FULLGRAD_BLOCKS: {
      if (value < 0 || value > 65535) return HALP_ERR_INVALID;
      if (fullgrad_supported(h->p) != HALP_OK) return HALP_ERR_UNSUPPORTED;
      const int old = h->fullgrad_blocks;
      h->fullgrad_blocks = (int)value;
      const int parts = fullgrad_parts(*h), loss_parts = fullgrad_loss_parts(*h);
      if (parts != h->parts || loss_parts != h->loss_parts) {  // resize the workspace
        float* ng = nullptr;
        double* nl = nullptr;
        const size_t bytes = sizeof(float) * (size_t)h->p.R * parts * (size_t)h->p.K * h->p.d;
        const size_t loss_row = parts > loss_parts ? parts : loss_parts;
        if (hipMalloc(reinterpret_cast<void**>(&ng), bytes) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&nl), sizeof(double) * (size_t)h->p.R * loss_row) !=
                hipSuccess) {
          if (ng) (void)hipFree(ng);
          h->fullgrad_blocks = old;
          return HALP_ERR_HIP;
        }
        (void)hipDeviceSynchronize();
        (void)hipFree(h->partial_g);
        (void)hipFree(h->partial_loss);
        h->partial_g = ng;
        h->partial_loss = nl;
        h->partial_g_bytes = bytes;
        h->parts = parts;
        h->loss_parts = loss_parts;
      }
      return HALP_OK;
    }
    default:
      return HALP_ERR_INVALID;
  }
}

int halp_quantize_data(halp_handle* h, void* stream) {
  if (!h) return HALP_ERR_NULL;
  if (!h->bound || !h->buf.X || !h->buf.Xq) return HALP_ERR_NOT_BOUND;
  return launch_quantize_data(*h, as_stream(stream));
}

int halp_full_gradient(halp_handle* h, void* stream) {
  if (!h) return HALP_ERR_NULL;
  int rc = need_full_gradient(*h);
  if (rc != HALP_OK) return rc;
  if ((rc = prepare_full_gradient(*h, as_stream(stream))) != HALP_OK) return rc;
  return launch_full_gradient(*h, as_stream(stream));
}

int halp_full_gradient_static(const halp_params* p, const halp_buffers* b, void* stream) {
  if (!p || !b) return HALP_ERR_NULL;
  int rc = check_params(*p);
  if (rc != HALP_OK) return rc;
  if (!b->X || !b->y || !b->w || !b->phi || !b->g || !b->scales) return HALP_ERR_NOT_BOUND;
  if (b->ldx < p->d) return HALP_ERR_INVALID;
  if (b->ldx % 4 != 0 || !aligned(b->X, 16) || !aligned(b->w, 4) || !aligned(b->phi, 4) ||
      !aligned(b->g, 4) || !aligned(b->y, 4) || !aligned(b->scales, 8))
    return HALP_ERR_ALIGN;
  return launch_full_gradient_static(*p, *b, as_stream(stream));
}

int halp_recenter(halp_handle* h, int64_t epoch, void* stream) {
  if (!h) return HALP_ERR_NULL;
  if (h->p.algorithm == HALP_ALG_SVRG) return HALP_ERR_INVALID;
  int rc = check_epoch(epoch);
  if (rc == HALP_OK) rc = need_recenter(*h);
  if (rc != HALP_OK) return rc;
  return launch_recenter(*h, (uint32_t)epoch, as_stream(stream));
}

int halp_inner_loop(halp_handle* h, int64_t epoch, void* stream) {
  if (!h) return HALP_ERR_NULL;
  int rc = check_epoch(epoch);
  if (rc != HALP_OK) return rc;
  const int variant = pick_inner_variant(*h);
  rc = need_inner(*h, variant);
  if (rc != HALP_OK) return rc;
  rc = launch_inner(*h, variant, (uint32_t)epoch, as_stream(stream));
  if (rc == HALP_OK) h->last_inner_variant = variant;
  return rc;
}

int halp_inner_loop_trace(halp_handle* h, int64_t epoch, int64_t M, int64_t* idx, int64_t* D,
                          double* beta, int32_t* gamma, int32_t* ztraj, void* stream) {
  if (!h) return HALP_ERR_NULL;
  int rc = check_epoch(epoch);
  if (rc != HALP_OK) return rc;
  if (M < 0 || h->p.algorithm == HALP_ALG_SVRG) return HALP_ERR_INVALID;
  rc = need_inner(*h, 1);
  if (rc != HALP_OK) return rc;
  TraceBufs tr;
  tr.M = M; tr.idx = idx; tr.D = D; tr.beta = beta; tr.gamma = gamma; tr.ztraj = ztraj;
  rc = launch_inner_generic(*h, (uint32_t)epoch, tr, as_stream(stream));
  if (rc == HALP_OK) h->last_inner_variant = 1;
  return rc;
}

int halp_epoch(halp_handle* h, int64_t epoch, void* stream) {
  if (!h) return HALP_ERR_NULL;
  int rc = check_epoch(epoch);
  if (rc != HALP_OK) return rc;
  // every requirement is checked before the first launch
  const int variant = pick_inner_variant(*h);
  if ((rc = need_full_gradient(*h)) != HALP_OK) return rc;
  const bool svrg = h->p.algorithm == HALP_ALG_SVRG;  // Algorithm 1 has no re-scaling step
  if (!svrg && (rc = need_recenter(*h)) != HALP_OK) return rc;
  if ((rc = need_inner(*h, variant)) != HALP_OK) return rc;
  hipStream_t s = as_stream(stream);
  if ((rc = prepare_full_gradient(*h, s)) != HALP_OK) return rc;
  hipEvent_t* ev = h->ev[h->timed % halp_handle::kTimedEpochs];
  if (h->timing && hipEventRecord(ev[0], s) != hipSuccess) return HALP_ERR_HIP;
  if ((rc = launch_full_gradient(*h, s)) != HALP_OK) return rc;
  if (h->timing && hipEventRecord(ev[1], s) != hipSuccess) return HALP_ERR_HIP;
  if (!svrg && (rc = launch_recenter(*h, (uint32_t)epoch, s)) != HALP_OK) return rc;
  if (h->timing && hipEventRecord(ev[2], s) != hipSuccess) return HALP_ERR_HIP;
  if ((rc = launch_inner(*h, variant, (uint32_t)epoch, s)) != HALP_OK) return rc;
  h->last_inner_variant = variant;
  if (h->timing) {
    if (hipEventRecord(ev[3], s) != hipSuccess) return HALP_ERR_HIP;
    h->timed += 1;
  }
  return HALP_OK;
}

int halp_get_stats(halp_handle* h, int32_t chain, void* stream, halp_stats* out) {
  if (!h || !out) return HALP_ERR_NULL;
  if (chain < 0 || chain >= h->p.R) return HALP_ERR_INVALID;
  if (!h->bound || !h->buf.scales) return HALP_ERR_NOT_BOUND;
  if (hipStreamSynchronize(as_stream(stream)) != hipSuccess) return HALP_ERR_HIP;
  std::memset(out, 0, sizeof *out);
  double sc[8];
  if (hipMemcpy(sc, h->buf.scales + (int64_t)chain * 8, sizeof sc, hipMemcpyDeviceToHost) !=
      hipSuccess)
    return HALP_ERR_HIP;
  out->delta_m = sc[0]; out->delta_i = sc[1]; out->delta_s = sc[2]; out->grad_norm = sc[3];
  out->loss = sc[6]; out->status = (int32_t)sc[7];
  out->inner_variant = h->last_inner_variant;
  if (h->buf.counters) {
    uint64_t c[4];
    if (hipMemcpy(c, h->buf.counters + (int64_t)chain * 4, sizeof c, hipMemcpyDeviceToHost) !=
        hipSuccess)
      return HALP_ERR_HIP;
    out->n_clamped_z = c[0]; out->n_clamped_gamma = c[1]; out->n_reg_draws = c[2];
    out->n_exchange_timeouts = c[3];
  }
  if (h->timing && h->timed > 0) {  // mean over the recorded epochs (the last 32 at most)
    const int64_t n = h->timed < halp_handle::kTimedEpochs ? h->timed : halp_handle::kTimedEpochs;
    double acc[3] = {0, 0, 0};
    int64_t ok = 0;
    for (int64_t k = 0; k < n; ++k) {
      float a = 0.f, b = 0.f, c = 0.f;
      if (hipEventElapsedTime(&a, h->ev[k][0], h->ev[k][1]) == hipSuccess &&
          hipEventElapsedTime(&b, h->ev[k][1], h->ev[k][2]) == hipSuccess &&
          hipEventElapsedTime(&c, h->ev[k][2], h->ev[k][3]) == hipSuccess) {
        acc[0] += a; acc[1] += b; acc[2] += c;
        ok += 1;
      }
    }
    (void)hipGetLastError();
    if (ok > 0) {
      out->ms_full_gradient = (float)(acc[0] / ok);
      out->ms_recenter = (float)(acc[1] / ok);
      out->ms_inner_loop = (float)(acc[2] / ok);
    }
    out->timed_epochs = (int32_t)ok;
  }
  return out->n_exchange_timeouts ? HALP_ERR_EXCHANGE_TIMEOUT : HALP_OK;
}

int halp_debug_stream_words(uint64_t seed, uint32_t purpose, uint32_t epoch, uint64_t n0,
                            int64_t count, uint32_t* out, void* stream) {
  if (!out) return HALP_ERR_NULL;
  if (count < 0 || count > (int64_t(1) << 30)) return HALP_ERR_INVALID;
  return launch_debug_stream_words(seed, purpose, epoch, n0, count, out, as_stream(stream));
}

int halp_debug_read_bandwidth(const void* p, int64_t bytes, uint32_t* out, void* stream) {
  if (!p || !out) return HALP_ERR_NULL;
  if (bytes < 0 || bytes % 16 != 0) return HALP_ERR_INVALID;
  if (!aligned(p, 16) || !aligned(out, 4)) return HALP_ERR_ALIGN;
  return launch_debug_read(p, bytes, out, as_stream(stream));
}

int halp_debug_step_latency(int32_t waves, int64_t steps, int32_t blocks, uint32_t* out,
                            void* stream) {
  if (!out || steps < 8 || steps % 8 != 0 || blocks < 1 || blocks > 65535) return HALP_ERR_INVALID;
  if (waves != 1 && waves != 2 && waves != 4) return HALP_ERR_INVALID;
  return launch_debug_step_latency(waves, steps, blocks, out, as_stream(stream));
}

int halp_debug_zround_bits(uint64_t seed, uint32_t epoch, uint64_t t, int32_t d, int32_t b,
                           int32_t K, uint32_t* out, void* stream) {
  if (!out) return HALP_ERR_NULL;
  if (d < 1 || K < 1 || (b != 8 && b != 16)) return HALP_ERR_INVALID;
  return launch_debug_zround_bits(seed, epoch, t, d, b, K, out, as_stream(stream));
}

const char* halp_strerror(int code) {
  switch (code) {
    case HALP_OK: return "ok";
    case HALP_ERR_NULL: return "a required pointer is NULL";
    case HALP_ERR_INVALID: return "a parameter is out of range";
    case HALP_ERR_UNSUPPORTED: return "no kernel covers this shape or bit width";
    case HALP_ERR_NOT_BOUND: return "a buffer this call needs has not been bound";
    case HALP_ERR_HIP: return "a HIP runtime call failed";
    case HALP_ERR_ALIGN: return "pointer or stride alignment requirement not met";
    case HALP_ERR_EXCHANGE_TIMEOUT:
      return "a wait between the workgroups of the split minibatch loop ran out; w~ was not updated";
    case HALP_ERR_TOO_LARGE:
      return "the problem does not fit the fixed scratch of the allocation-free entry point";
    default: return "unknown error code";
  }
}

const char* halp_last_error_detail(void) { return g_detail; }

const char* halp_version(void) { return "halp-gfx950 0.1"; }

}  // extern "C"
