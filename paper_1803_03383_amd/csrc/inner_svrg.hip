// Inner loop of full-precision SVRG (Algorithm 1) for linear models, one sampled row per
// step: the comparator the paper times HALP against (its Table 3), on the same index stream
// and with the same launch structure as the low-precision inner loop.
//
//   w <- w - alpha ( (l'(x_i^T w) - l'(phi_i)) x_i + lambda (w - w~) + g~ ),   phi_i = x_i^T w~
//
// One workgroup per chain.  A thread owns CPL consecutive coordinates of w (fp32 registers)
// together with alpha g~ and w~; rows of the fp32 data are gathered in windows of 8 steps, the
// next window's fragments being requested at the top of the current one.  Vector work is
// fp32 (fused multiply-adds), the scalar l' difference fp64, the wave sums DPP folds, the
// cross-wave sum one LDS word per wave added in wave order.  Sample indices (and the margins
// and labels of the sampled rows) are produced 256 steps at a time into LDS.
#include "halp_device.hpp"
#include "halp_internal.hpp"

namespace halp {
namespace {

constexpr int kBatch = 256;
constexpr int kWin = 8;

struct SvArgs {
  const float* X;    // [Rd][N][ldx]
  const float* y;    // [Rd][N]
  const float* phi;  // [R][N]
  const float* g;    // [R][d]
  float* w;          // [R][d] in: w~, out: w_T
  int64_t N, ldx, T;
  int64_t x_chain_stride, y_chain_stride;
  int d, loss;
  int option2;
  const double* hyper;  // [R][2] step size (and mu, unused here) of each chain
  double lambda;
  uint64_t seed;
  uint32_t epoch;
};

__device__ __forceinline__ double logistic_dl(double a, double y) {
  return __ddiv_rn(-y, __dadd_rn(1.0, halp_exp(__dmul_rn(y, a))));
}

template <int CPL, int NWT, int LOSS>
__global__ __launch_bounds__(64 * NWT) void inner_svrg_kernel(SvArgs a) {
  const int chain = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = NWT > 1 ? tid >> 6 : 0;
  const int d = a.d;
  const uint32_t N = (uint32_t)a.N;
  const int64_t T = epoch_steps(a.seed + (uint64_t)blockIdx.x, a.epoch, a.T, a.option2);
  const float* __restrict__ X = a.X + (int64_t)chain * a.x_chain_stride;
  const float* __restrict__ y = a.y + (int64_t)chain * a.y_chain_stride;
  const float* __restrict__ phi = a.phi + (int64_t)chain * a.N;
  const float* __restrict__ g = a.g + (int64_t)chain * d;
  float* __restrict__ wg = a.w + (int64_t)chain * d;
  const uint64_t seed = a.seed + (uint64_t)chain;
  constexpr bool logistic = LOSS == HALP_LOSS_LOGISTIC;
  constexpr int kMask = 2 * kBatch - 1;

  __shared__ __attribute__((aligned(16))) int s_idx[2 * kBatch];
  __shared__ __attribute__((aligned(16))) float s_phi[2 * kBatch];
  __shared__ __attribute__((aligned(16))) float s_y[2 * kBatch];
  __shared__ float s_part[2][16];
  __shared__ float s_dump[NWT > 1 ? 64 * NWT : 1];
  using LdsF = __attribute__((address_space(3))) float;
  LdsF* const slot0 = (LdsF*)((NWT > 1 && lane != 63) ? &s_dump[tid] : &s_part[0][wave]);
  LdsF* const slot1 = (LdsF*)((NWT > 1 && lane != 63) ? &s_dump[tid] : &s_part[1][wave]);

  // ---- per-thread state; coordinates past d hold zeros and never change
  const int j0 = tid * CPL;
  // Rows are padded to a multiple of 4 floats, so the fragment at j0 < d lies inside the row
  // even when it runs past d (the excess is masked); threads past the row re-read its start.
  const int jc = j0 < d ? j0 : 0;
  const double alpha = a.hyper[2 * chain];
  float w[CPL], wt[CPL], ag[CPL];
  bool keep[CPL];
#pragma unroll
  for (int k = 0; k < CPL; ++k) {
    const bool ok = j0 + k < d;
    const int j = min(j0 + k, d - 1);
    w[k] = wt[k] = ok ? wg[j] : 0.f;
    ag[k] = ok ? (float)__dmul_rn(alpha, (double)g[j]) : 0.f;
    keep[k] = ok;
  }
  const float al = (float)__dmul_rn(alpha, a.lambda);
  const bool use_reg = a.lambda > 0;

  auto fill_batch = [&](int64_t bb) {
    const int half = (int)(bb & 1) * kBatch;
    if (tid < 64) {
      const U4 ri = stream_block(seed, kIdx, a.epoch, (uint64_t)bb * 64 + (uint64_t)tid);
      int4 iv;
      iv.x = (int)__umulhi(ri.x, N); iv.y = (int)__umulhi(ri.y, N);
      iv.z = (int)__umulhi(ri.z, N); iv.w = (int)__umulhi(ri.w, N);
      *reinterpret_cast<int4*>(&s_idx[half + 4 * tid]) = iv;
      float4 pv;
      pv.x = phi[iv.x]; pv.y = phi[iv.y]; pv.z = phi[iv.z]; pv.w = phi[iv.w];
      *reinterpret_cast<float4*>(&s_phi[half + 4 * tid]) = pv;
      if (logistic) {
        float4 yv;
        yv.x = y[iv.x]; yv.y = y[iv.y]; yv.z = y[iv.z]; yv.w = y[iv.w];
        *reinterpret_cast<float4*>(&s_y[half + 4 * tid]) = yv;
      }
    }
  };
  fill_batch(0);
  fill_batch(1);
  __syncthreads();

  // ---- row fragments: two buffers of one window each.  Any step number names a valid row
  // (the index batches are whole), so every load is unconditional.
  float xa[kWin][CPL], xb[kWin][CPL];
  auto request = [&](float (&dst)[CPL], int i) {
    const float* rp = X + (int64_t)i * a.ldx + jc;
    if (CPL == 1) {
      dst[0] = rp[0];
    } else if (CPL == 2) {
      const float2 v = *reinterpret_cast<const float2*>(rp);
      dst[0] = v.x; dst[CPL > 1 ? 1 : 0] = v.y;
    } else {
      const float4 v = *reinterpret_cast<const float4*>(rp);
      dst[0] = v.x; dst[CPL > 1 ? 1 : 0] = v.y; dst[CPL > 2 ? 2 : 0] = v.z; dst[CPL > 3 ? 3 : 0] = v.w;
    }
  };
#pragma unroll
  for (int s = 0; s < kWin; ++s) request(xa[s], __builtin_amdgcn_readfirstlane(s_idx[s]));

  auto window = [&](int64_t t0, float (&xr)[kWin][CPL], float (&xnext)[kWin][CPL]) {
    const int base = (int)(t0 & kMask);
    float phi8[kWin], y8[kWin];
    int nidx[kWin];
    {
      const float4 p0 = *reinterpret_cast<const float4*>(&s_phi[base]);
      const float4 p1 = *reinterpret_cast<const float4*>(&s_phi[base + 4]);
      phi8[0] = p0.x; phi8[1] = p0.y; phi8[2] = p0.z; phi8[3] = p0.w;
      phi8[4] = p1.x; phi8[5] = p1.y; phi8[6] = p1.z; phi8[7] = p1.w;
#pragma unroll
      for (int s = 0; s < kWin; ++s) y8[s] = 0.f;
      if (logistic) {
        const float4 y0 = *reinterpret_cast<const float4*>(&s_y[base]);
        const float4 y1 = *reinterpret_cast<const float4*>(&s_y[base + 4]);
        y8[0] = y0.x; y8[1] = y0.y; y8[2] = y0.z; y8[3] = y0.w;
        y8[4] = y1.x; y8[5] = y1.y; y8[6] = y1.z; y8[7] = y1.w;
      }
      const int nb = (base + kWin) & kMask;
      const int4 i0 = *reinterpret_cast<const int4*>(&s_idx[nb]);
      const int4 i1 = *reinterpret_cast<const int4*>(&s_idx[nb + 4]);
      nidx[0] = i0.x; nidx[1] = i0.y; nidx[2] = i0.z; nidx[3] = i0.w;
      nidx[4] = i1.x; nidx[5] = i1.y; nidx[6] = i1.z; nidx[7] = i1.w;
    }
    // this window's fragments leave the load buffer (masked) before the next ones are requested
    float xw[kWin][CPL];
#pragma unroll
    for (int s = 0; s < kWin; ++s)
#pragma unroll
      for (int k = 0; k < CPL; ++k) xw[s][k] = keep[k] ? xr[s][k] : 0.f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < kWin; ++s) request(xnext[s], __builtin_amdgcn_readfirstlane(nidx[s]));

#pragma unroll
    for (int s = 0; s < kWin; ++s) {
      if (t0 + s < T) {
        float part = 0.f;
#pragma unroll
        for (int k = 0; k < CPL; ++k) part = __builtin_fmaf(xw[s][k], w[k], part);
        // several waves: lane 63, where the fold leaves the sum, stores it; the other lanes store
        // into a dump row, so that no lane mask is set up and no lane is read
        float dot = NWT > 1 ? wave_fold_f32(part) : wave_sum_f32(part);
        if (NWT > 1) {
          *((s & 1) ? slot1 : slot0) = dot;
          __syncthreads();
          float tot = 0.f;
#pragma unroll
          for (int w2 = 0; w2 < NWT; ++w2) tot += s_part[s & 1][w2];
          dot = tot;
        }
        // alpha (l'(x_i^T w) - l'(phi_i)): the scalar path in fp64
        const double a1 = (double)dot, a0 = (double)phi8[s];
        double diff;
        if (logistic) diff = __dadd_rn(logistic_dl(a1, (double)y8[s]), -logistic_dl(a0, (double)y8[s]));
        else diff = __dadd_rn(a1, -a0);  // (a1 - y) - (a0 - y)
        const float c = (float)__dmul_rn(alpha, diff);
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
          float u = __builtin_fmaf(-c, xw[s][k], w[k]) - ag[k];
          if (use_reg) u = __builtin_fmaf(-al, w[k] - wt[k], u);
          w[k] = u;
        }
      }
    }
  };

  int64_t t0 = 0;
  for (; t0 < T; t0 += 2 * kWin) {
    if ((t0 & (kBatch - 1)) == 0 && t0 > 0) {  // batch t0/256 - 1 is finished: refill its half
      __syncthreads();
      fill_batch(t0 / kBatch + 1);
      __syncthreads();
    }
    window(t0, xa, xb);
    if (t0 + kWin < T) window(t0 + kWin, xb, xa);
  }

  // ---- w~ <- w_T (option I)
#pragma unroll
  for (int k = 0; k < CPL; ++k)
    if (j0 + k < d) wg[j0 + k] = w[k];
}

template <int CPL, int NWT>
int launch_loss(const SvArgs& a, int R, hipStream_t s) {
  const dim3 grid(R), block(64 * NWT);
  if (a.loss == HALP_LOSS_LOGISTIC)
    hipLaunchKernelGGL((inner_svrg_kernel<CPL, NWT, HALP_LOSS_LOGISTIC>), grid, block, 0, s, a);
  else
    hipLaunchKernelGGL((inner_svrg_kernel<CPL, NWT, HALP_LOSS_SQUARED>), grid, block, 0, s, a);
  return hip_ok(hipGetLastError());
}

struct SvShape {
  int cpl, nw;
};

// coordinates per thread and waves per chain: as many waves (up to 4 when chains are few, else
// 1) as keep every thread busy, then wider fragments
SvShape pick_shape(const halp_handle& h) {
  const int d = h.p.d;
  int nw = 1;
  const int64_t simds = 4 * (int64_t)h.num_cus;
  if (h.inner_waves > 0) nw = h.inner_waves;
  else while (nw < 4 && (int64_t)h.p.R * nw * 2 <= simds && 64 * nw < d) nw *= 2;
  int cpl = 1;
  while (cpl < 4 && 64 * nw * cpl < d) cpl *= 2;
  while (64 * nw * cpl < d && nw < 16) nw *= 2;
  return SvShape{cpl, nw};
}

}  // namespace

// squared or logistic loss, one row per step, d <= 4096 (16 waves of 64 threads of 4 coordinates)
int inner_svrg_supported(const halp_handle& h) {
  const halp_params& p = h.p;
  if (p.K != 1 || p.B != 1) return HALP_ERR_UNSUPPORTED;
  if (p.loss != HALP_LOSS_SQUARED && p.loss != HALP_LOSS_LOGISTIC) return HALP_ERR_UNSUPPORTED;
  const SvShape sh = pick_shape(h);
  if (64 * sh.nw * sh.cpl < p.d) return HALP_ERR_UNSUPPORTED;
  const bool built = (sh.nw <= 4 && (sh.nw == 1 || sh.nw == 2 || sh.nw == 4)) ||
                     (sh.cpl == 4 && (sh.nw == 8 || sh.nw == 16));
  return built ? HALP_OK : HALP_ERR_UNSUPPORTED;
}

int launch_inner_svrg(const halp_handle& h, uint32_t epoch, hipStream_t s) {
  const halp_params& p = h.p;
  const int rc = inner_svrg_supported(h);
  if (rc != HALP_OK) return rc;
  SvArgs a;
  a.X = h.buf.X; a.y = reinterpret_cast<const float*>(h.buf.y); a.phi = h.buf.phi; a.g = h.buf.g;
  a.w = h.buf.w;
  a.N = p.N; a.ldx = h.buf.ldx; a.T = p.T;
  a.x_chain_stride = p.share_data ? 0 : p.N * h.buf.ldx;
  a.y_chain_stride = p.share_data ? 0 : p.N;
  a.d = p.d; a.loss = p.loss; a.hyper = h.hyper; a.lambda = p.lambda; a.option2 = h.option2 ? 1 : 0;
  a.seed = p.seed; a.epoch = epoch;
  const SvShape sh = pick_shape(h);
#define HALP_SV(C_, W_) \
  if (sh.cpl == C_ && sh.nw == W_) return launch_loss<C_, W_>(a, p.R, s);
  HALP_SV(1, 1) HALP_SV(2, 1) HALP_SV(4, 1)
  HALP_SV(1, 2) HALP_SV(2, 2) HALP_SV(4, 2)
  HALP_SV(1, 4) HALP_SV(2, 4) HALP_SV(4, 4)
  HALP_SV(4, 8) HALP_SV(4, 16)
#undef HALP_SV
  return HALP_ERR_UNSUPPORTED;
}

}  // namespace halp
