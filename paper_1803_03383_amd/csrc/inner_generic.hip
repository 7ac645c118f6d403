// Inner loop of Algorithm 4 (LM-HALP), general form: any loss, K classes,
// minibatch B, 8 or 16 bits, optional per-step trace.  One workgroup per chain;
// z and h~ live in LDS as 32-bit integers, all integer arithmetic is exact in
// 64 bits, the scalar path (beta, gamma) is fp64.  This kernel is the fallback
// for shapes the register-resident kernel does not take and the one the debug
// trace runs on; it favours simplicity over speed.
#include "halp_device.hpp"
#include "inner_args.hpp"

namespace halp {
namespace {

__device__ __forceinline__ double logistic_dl(double a, double y) {
  // l'(a) for l(a) = log(1 + exp(-y a))
  return __ddiv_rn(-y, __dadd_rn(1.0, halp_exp(__dmul_rn(y, a))));
}

template <int BITS>
__global__ __launch_bounds__(512) void inner_generic_kernel(InArgs a) {
  using XT = typename std::conditional<BITS == 8, int8_t, int16_t>::type;
  using HT = typename std::conditional<BITS == 8, int16_t, int32_t>::type;
  constexpr int CPS = 16 / BITS;  // coordinates per strip of 16 rounding bits
  constexpr int EPG = 64 / BITS;  // elements per 8-byte group of a data row
  const int chain = blockIdx.x;
  const int tid = threadIdx.x, NT = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, NW = NT >> 6;
  const int d = a.d, K = a.K, B = a.B;
  const int n = K * d;
  const int U = (d + CPS - 1) / CPS;
  const int ngroups = (d + EPG - 1) / EPG;
  const int64_t N = a.N, ldxq = a.ldxq;
  const XT* __restrict__ Xq = reinterpret_cast<const XT*>(a.Xq) + (int64_t)chain * a.xq_chain_stride;
  const float* __restrict__ phi = a.phi + (int64_t)chain * N * K;
  const float* __restrict__ y =
      reinterpret_cast<const float*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const HT* __restrict__ hg = reinterpret_cast<const HT*>(a.h) + (int64_t)chain * n;
  XT* __restrict__ zg = reinterpret_cast<XT*>(a.z) + (int64_t)chain * n;
  float* __restrict__ wg = a.w + (int64_t)chain * n;
  const double* sc = a.scales + (int64_t)chain * 8;
  uint64_t* cnt_out = a.counters + (int64_t)chain * 4;
  const uint64_t seed = a.seed + (uint64_t)chain;

  if (sc[7] != 0.0) {  // converged or unusable gradient: the epoch is a no-op
    if (tid < 4) cnt_out[tid] = 0;
    return;
  }

  // z and h~ as 32-bit integers: in LDS, or -- a model too large for it -- in this chain's part
  // of a device-memory workspace (the waves of a workgroup share the CU's cache, and every
  // hand-over between them below is a barrier)
  extern __shared__ unsigned char smem_raw[];
  const int nz = n + (n & 1);
  int32_t* zs = a.zh_work ? a.zh_work + (int64_t)chain * 2 * nz : reinterpret_cast<int32_t*>(smem_raw);
  int32_t* hs = zs + nz;
  long long* idxs = reinterpret_cast<long long*>(a.zh_work ? smem_raw : smem_raw + sizeof(int32_t) * 2 * nz);
  long long* Ds = idxs + B;
  double* es = reinterpret_cast<double*>(Ds + (int64_t)B * K);  // softmax: exp terms [B*K][2]
  double* rowst = es + 2 * (int64_t)B * K;                       // per row: max0, max1, sum0, sum1
  int32_t* gams = reinterpret_cast<int32_t*>(rowst + 4 * (int64_t)B);
  __shared__ unsigned long long s_cnt[3];
  __shared__ int s_clambda;

  for (int k = tid; k < n; k += NT) {
    zs[k] = (int32_t)zg[k];
    hs[k] = (int32_t)hg[k];
  }
  if (tid < 3) s_cnt[tid] = 0;
  if (tid == 0) s_clambda = 0;
  __syncthreads();

  const double delta_m = sc[0], inv_s = sc[5];
  const double dscale = __dmul_rn(a.delta_d, delta_m);
  const double alpha = a.hyper[2 * chain];
  const double aB = __ddiv_rn(alpha, (double)B);
  const bool lp = a.lp != 0;
  // the margin after the move: Algorithm 4 adds x^T z to phi, in Algorithm 2 x^T w is all of it
  auto after_margin = [&](double a0, long long D) {
    const double delta = __dmul_rn(dscale, (double)D);
    return lp ? delta : __dadd_rn(a0, delta);
  };
  const double qmaxd = (double)((1 << (BITS - 1)) - 1), qmind = -(double)(1 << (BITS - 1));
  const long long qmax = (1 << (BITS - 1)) - 1, qmin = -(1 << (BITS - 1));
  unsigned long long my_zclamp = 0, my_gclamp = 0;
  constexpr int kCached = 8;
  U4 zcache[kCached];
  const bool cache_blocks = K * U <= kCached * NT;

  const int64_t T = epoch_steps(seed, a.epoch, a.T, a.option2);
  for (int64_t t = 0; t < T; ++t) {
    const bool rec = t < a.tr.M;
    // sample i uniformly (with replacement)
    if (tid < B) {
      const uint64_t nn = (uint64_t)t * (uint64_t)B + (uint64_t)tid;
      const uint32_t r = pick(stream_block(seed, kIdx, a.epoch, nn >> 2), (uint32_t)(nn & 3));
      const long long i = (long long)(((uint64_t)r * (uint64_t)N) >> 32);
      idxs[tid] = i;
      if (rec && a.tr.idx) a.tr.idx[((int64_t)chain * a.tr.M + t) * B + tid] = i;
    }
    if (tid == 0 && a.lambda > 0) {  // c_lambda = Q_(2^-b, b)(alpha lambda)
      const uint32_t r = pick(stream_block(seed, kReg, a.epoch, (uint64_t)t >> 2), (uint32_t)(t & 3));
      const int cl = (int)quantize_real(__dmul_rn(alpha, a.lambda), (double)(1 << BITS), r, 0.0,
                                        qmaxd, nullptr);
      s_clambda = cl;
      if (cl != 0) s_cnt[2] += 1;
    }
    __syncthreads();
    // integer dot products x_i^T z, one (row, class) pair per wave at a time
    for (int pr = wave; pr < B * K; pr += NW) {
      const int m = pr / K, c = pr % K;
      // rows are 8-byte aligned and padded to whole 8-byte groups: one load per group
      const uint2* xr = reinterpret_cast<const uint2*>(Xq + idxs[m] * ldxq);
      long long acc = 0;
      for (int q0 = lane; q0 < ngroups; q0 += 64 * 8) {  // eight loads in flight per lane
        uint2 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = xr[min(q0 + 64 * i, ngroups - 1)];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int q = q0 + 64 * i;
          if (q < ngroups) {
#pragma unroll
            for (int e = 0; e < EPG; ++e) {
              const uint32_t wv = e < EPG / 2 ? v[i].x : v[i].y;
              const int sh = (e % (EPG / 2)) * BITS;
              const int xv = BITS == 8 ? (int)(int8_t)(wv >> sh) : (int)(int16_t)(wv >> sh);
              const int j = q * EPG + e;
              if (j < d) acc += (long long)(xv * zs[c * d + j]);  // |x z| < 2^30
            }
          }
        }
      }
      acc = wave_sum_i64(acc);
      if (lane == 0) {
        Ds[pr] = acc;
        if (rec && a.tr.D) a.tr.D[((int64_t)chain * a.tr.M + t) * B * K + pr] = acc;
      }
    }
    __syncthreads();
    // beta = (alpha/B)(l'(phi_i + x_i^T z) - l'(phi_i)); gamma = Q_(delta_s, b)(beta).
    // One thread per (row, class) pair; the softmax normalisers are formed per row, the
    // exponentials summed pairwise over adjacent classes.
    const bool softmax = a.loss == HALP_LOSS_SOFTMAX;
    if (softmax) {
      if (tid < B) {
        const long long i = idxs[tid];
        double mx0 = (double)phi[i * K];
        double mx1 = after_margin(mx0, Ds[tid * K]);
        for (int c = 1; c < K; ++c) {
          const double a0 = (double)phi[i * K + c];
          const double a1 = after_margin(a0, Ds[tid * K + c]);
          if (a0 > mx0) mx0 = a0;
          if (a1 > mx1) mx1 = a1;
        }
        rowst[4 * tid + 0] = mx0;
        rowst[4 * tid + 1] = mx1;
      }
      __syncthreads();
      for (int pr = tid; pr < B * K; pr += NT) {
        const int m = pr / K, c = pr % K;
        const double a0 = (double)phi[idxs[m] * K + c];
        const double a1 = after_margin(a0, Ds[pr]);
        es[2 * pr + 0] = halp_exp(__dadd_rn(a0, -rowst[4 * m + 0]));
        es[2 * pr + 1] = halp_exp(__dadd_rn(a1, -rowst[4 * m + 1]));
      }
      __syncthreads();
      if (tid < B) {
        // pairwise over adjacent classes (absent classes count as +0), K <= 16
        double v0[16], v1[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) {
          v0[c] = c < K ? es[2 * (tid * K + c) + 0] : 0.0;
          v1[c] = c < K ? es[2 * (tid * K + c) + 1] : 0.0;
        }
#pragma unroll
        for (int P = 16; P > 1; P /= 2) {
#pragma unroll
          for (int c = 0; c < P / 2; ++c) {
            v0[c] = __dadd_rn(v0[2 * c], v0[2 * c + 1]);
            v1[c] = __dadd_rn(v1[2 * c], v1[2 * c + 1]);
          }
        }
        const double s0 = v0[0], s1 = v1[0];
        rowst[4 * tid + 2] = s0;
        rowst[4 * tid + 3] = s1;
      }
      __syncthreads();
    }
    for (int pr = tid; pr < B * K; pr += NT) {
      const int m = pr / K, c = pr % K;
      const long long i = idxs[m];
      const double delta = __dmul_rn(dscale, (double)Ds[pr]);
      double diff;
      if (a.loss == HALP_LOSS_SQUARED) {
        // Algorithm 4: (phi + Delta - y) - (phi - y) = Delta; Algorithm 2: (x^T w - y) - (phi - y)
        diff = lp ? __dadd_rn(delta, -(double)phi[i]) : delta;
      } else if (a.loss == HALP_LOSS_LOGISTIC) {
        const double a0 = (double)phi[i];
        const double yi = (double)y[i];
        diff = __dadd_rn(logistic_dl(after_margin(a0, Ds[pr]), yi), -logistic_dl(a0, yi));
      } else {
        const double p0 = __ddiv_rn(es[2 * pr + 0], rowst[4 * m + 2]);
        const double p1 = __ddiv_rn(es[2 * pr + 1], rowst[4 * m + 3]);
        diff = __dadd_rn(p1, -p0);
      }
      const double beta = __dmul_rn(aB, diff);
      const uint64_t nn = ((uint64_t)t * (uint64_t)B + (uint64_t)m) * (uint64_t)K + (uint64_t)c;
      const uint32_t r = pick(stream_block(seed, kGamma, a.epoch, nn >> 2), (uint32_t)(nn & 3));
      bool hit = false;
      const int gq = (int)quantize_real(beta, inv_s, r, qmind, qmaxd, &hit);
      gams[pr] = gq;
      if (hit) my_gclamp += 1;
      if (rec) {
        const int64_t o = ((int64_t)chain * a.tr.M + t) * B * K + pr;
        if (a.tr.beta) a.tr.beta[o] = beta;
        if (a.tr.gamma) a.tr.gamma[o] = gq;
      }
    }
    __syncthreads();
    // u = z - gamma x_i - h~ (- c_lambda z) in (delta_i, 2b); z = Q_(delta_m, b)(u)
    const long long cl = s_clambda;
    // gsum = sum over the minibatch of gamma_m x_m for one strip
    auto finish_strip = [&](int u, const U4& r, const long long (&gsum)[CPS]) {
      const int c = u / U, strip = u % U;
      const uint32_t field = zround_field(r, (uint32_t)t);
      for (int e = 0; e < CPS; ++e) {
        const int j = strip * CPS + e;
        if (j >= d) break;
        const int k = c * d + j;
        const long long zk = zs[k];
        const long long v = -(long long)hs[k] - cl * zk - gsum[e];
        const long long rb = (long long)((field >> (e * BITS)) & ((1u << BITS) - 1u));
        long long zn = zk + ((v + rb) >> BITS);  // arithmetic shift: floor
        if (zn > qmax) { zn = qmax; my_zclamp += 1; }
        if (zn < qmin) { zn = qmin; my_zclamp += 1; }
        zs[k] = (int32_t)zn;
      }
    };
    if (cache_blocks) {
      // A thread's strips are the same every step: their Philox blocks are kept for 8 steps,
      // and the minibatch is summed row by row over all of them, so that the loads of a
      // row are independent of each other and in flight together.
      long long gsum[kCached][CPS];
      int sc[kCached], sj[kCached];  // class and first coordinate of each strip (-1: none)
#pragma unroll
      for (int s = 0; s < kCached; ++s) {
        const int u = tid + s * NT;
        sc[s] = u < K * U ? u / U : -1;
        sj[s] = u < K * U ? (u % U) * CPS : 0;
#pragma unroll
        for (int e = 0; e < CPS; ++e) gsum[s][e] = 0;
      }
#pragma unroll 4
      for (int m = 0; m < B; ++m) {
        const XT* xr = Xq + idxs[m] * ldxq;
#pragma unroll
        for (int s = 0; s < kCached; ++s) {
          if (sc[s] >= 0) {
            const long long g = gams[m * K + sc[s]];
#pragma unroll
            for (int e = 0; e < CPS; ++e)
              if (sj[s] + e < d) gsum[s][e] += g * (long long)xr[sj[s] + e];
          }
        }
      }
#pragma unroll
      for (int s = 0; s < kCached; ++s) {
        const int u = tid + s * NT;
        if (u < K * U) {
          if ((t & 7) == 0) zcache[s] = zround_block(seed, a.epoch, (uint32_t)u, (uint32_t)(t >> 3));
          finish_strip(u, zcache[s], gsum[s]);
        }
      }
    } else {
      for (int u = tid; u < K * U; u += NT) {
        const int c = u / U, j0 = (u % U) * CPS;
        long long gsum[CPS];
#pragma unroll
        for (int e = 0; e < CPS; ++e) gsum[e] = 0;
        for (int m = 0; m < B; ++m)
#pragma unroll
          for (int e = 0; e < CPS; ++e)
            if (j0 + e < d) gsum[e] += (long long)gams[m * K + c] * (long long)Xq[idxs[m] * ldxq + j0 + e];
        finish_strip(u, zround_block(seed, a.epoch, (uint32_t)u, (uint32_t)(t >> 3)), gsum);
      }
    }
    __syncthreads();
    if (rec && a.tr.ztraj) {
      int32_t* zt = a.tr.ztraj + ((int64_t)chain * a.tr.M + t) * n;
      for (int k = tid; k < n; k += NT) zt[k] = zs[k];
    }
  }

  // w~ <- w~ + delta_m z (option I), and hand z out
  for (int k = tid; k < n; k += NT) {
    const int32_t zk = zs[k];
    zg[k] = (XT)zk;
    const double step = __dmul_rn(delta_m, (double)zk);
    wg[k] = lp ? (float)step : (float)__dadd_rn((double)wg[k], step);  // Alg. 2: w~ = delta w
  }
  if (my_zclamp) atomicAdd(&s_cnt[0], my_zclamp);
  if (my_gclamp) atomicAdd(&s_cnt[1], my_gclamp);
  __syncthreads();
  if (tid < 4) cnt_out[tid] = tid < 3 ? s_cnt[tid] : 0ull;
}

}  // namespace

// LDS the kernel needs per row of a step (index, dots, scalars), and for z and h~ as int32
static size_t generic_step_smem(const halp_params& p) {
  return (size_t)p.B * 8 + (size_t)p.B * p.K * 8 + (size_t)p.B * p.K * 16 + (size_t)p.B * 32 +
         (size_t)p.B * p.K * 4;
}
static size_t generic_model_smem(const halp_params& p) {
  const int64_t n = (int64_t)p.K * p.d;
  return (size_t)(2 * (n + (n & 1))) * 4;
}
constexpr size_t kGenericSmemCap = 150 * 1024;

// a model that does not fit LDS beside a step's scalars lives in device memory
bool inner_generic_needs_workspace(const halp_params& p) {
  return generic_step_smem(p) + generic_model_smem(p) > kGenericSmemCap;
}
size_t inner_generic_workspace_bytes(const halp_params& p) { return (size_t)p.R * generic_model_smem(p); }

// at most 512 rows per step, and their scalars must fit the LDS of one CU
int inner_generic_supported(const halp_params& p) {
  return (generic_step_smem(p) > kGenericSmemCap || p.B > 512) ? HALP_ERR_UNSUPPORTED : HALP_OK;
}

int launch_inner_generic(const halp_handle& h, uint32_t epoch, const TraceBufs& tr, hipStream_t s) {
  const halp_params& p = h.p;
  InArgs a = make_inner_args(h, epoch);
  a.tr = tr;
  if (inner_generic_supported(p) != HALP_OK) return HALP_ERR_UNSUPPORTED;
  const bool outside = inner_generic_needs_workspace(p);
  if (outside && !h.zh_work) return HALP_ERR_UNSUPPORTED;
  a.zh_work = outside ? h.zh_work : nullptr;
  const size_t smem = generic_step_smem(p) + (outside ? 0 : generic_model_smem(p));
  const int threads = 512;
  hipError_t e;
  if (p.b == 8) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(inner_generic_kernel<8>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return HALP_ERR_HIP;
    hipLaunchKernelGGL(inner_generic_kernel<8>, dim3(p.R), dim3(threads), smem, s, a);
  } else {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(inner_generic_kernel<16>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return HALP_ERR_HIP;
    hipLaunchKernelGGL(inner_generic_kernel<16>, dim3(p.R), dim3(threads), smem, s, a);
  }
  return hip_ok(hipGetLastError());
}

}  // namespace halp
