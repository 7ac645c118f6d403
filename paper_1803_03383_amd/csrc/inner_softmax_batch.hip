// Inner loop of Algorithm 4 (LM-HALP) for softmax regression with a minibatch: K classes,
// B sampled rows per step, register-resident form.  Also takes the scalar margins (K = 1,
// squared or logistic loss) of minibatches wider than the kernel for that case holds.
//
// One workgroup per chain: K class waves and (up to 15 classes) one more wave that only takes
// part in the work that is dealt by thread.  Class wave c owns row c of z ([K][d]): lane l holds the UPL
// consecutive strips (16 rounding bits each: two coordinates at 8 bits, one at 16) starting at
// l * UPL, with h~ and the strips' Philox blocks of the current window of 8 steps, in
// registers for the whole epoch.
//
// One step:
//   threads < B       draw the sample indices (and thread 0 the L2 draw)                 | barrier
//   all threads       copy the B sampled rows of the quantized data into LDS             | barrier
//   class waves       x_m^T z_c for every row m: fragment from LDS, multiply-adds, fold  | barrier
//   all threads       softmax before and after the offset per row (maxima, exponentials,
//                     normalisers summed pairwise over adjacent classes),
//                     gamma_{m,c} = Q_(delta_s,b)(beta_{m,c}), one (row, class) per thread | barriers
//   class waves       sum_m gamma_{m,c} x_m from the rows in LDS, integer update of row c | barrier
// The arithmetic of every stage is that of the general kernel (inner_generic.hip): the same
// streams, the same order of the floating-point operations.
#include <algorithm>

#include "halp_device.hpp"
#include "inner_args.hpp"

namespace halp {
namespace {

constexpr int kMaxB = 64;     // rows of a step in LDS at a time (a step has up to 512)
constexpr int kMaxK = 16;     // classes: one wave each, and one wave more where 16 waves allow it
constexpr int kKPad = 16;     // classes are padded to 16 in the pairwise sums

__device__ __forceinline__ double logistic_dl(double a, double y) {
  // l'(a) for l(a) = log(1 + exp(-y a))
  return __ddiv_rn(-y, __dadd_rn(1.0, halp_exp(__dmul_rn(y, a))));
}

// WAVES: the most waves a launch of this instance has (K + 1 <= WAVES): fewer waves, more registers each
// MANY: more rows per step than LDS holds at a time (the loop over chunks then has one pass, and the
// sums of the update live only inside it)
template <int BITS, int UPL, int WAVES, bool MANY>
__global__ __launch_bounds__(64 * WAVES) void inner_softmax_batch_kernel(InArgs a, int slot_bytes) {
  using XT = typename std::conditional<BITS == 8, int8_t, int16_t>::type;
  using HT = typename std::conditional<BITS == 8, int16_t, int32_t>::type;
  using AccT = typename std::conditional<BITS == 8, int, long long>::type;
  constexpr int CT = 16 / BITS;    // coordinates per strip
  constexpr int CPL = UPL * CT;    // coordinates per lane
  constexpr int FQ = UPL / 8;      // 16-byte reads per fragment
  const int chain = blockIdx.x;
  const int tid = threadIdx.x, NT = blockDim.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int d = a.d, K = a.K, Bt = a.B;  // Bt rows per step, taken kMaxB at a time
  const int n = K * d;
  const int U = (d + CT - 1) / CT;
  const int64_t N = a.N, ldxq = a.ldxq;
  const int row_dw = (int)(ldxq * (BITS / 8) / 4);
  const int slot_dw = slot_bytes / 4;
  const int copy_dw = min(row_dw, slot_dw);     // at most 512: a slot holds 1024 strips of 2 bytes
  constexpr int kRowLoads = 8;                   // dwords per lane and row at most
  const int nq = (copy_dw + 63) / 64;
  const int NW = NT >> 6;
  const unsigned char* __restrict__ Xq = reinterpret_cast<const unsigned char*>(a.Xq) +
                                         (int64_t)chain * a.xq_chain_stride * (BITS / 8);
  const float* __restrict__ phi = a.phi + (int64_t)chain * N * K;
  const float* __restrict__ y = reinterpret_cast<const float*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const bool softmax = a.loss == HALP_LOSS_SOFTMAX;  // else K = 1: squared or logistic loss
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

  extern __shared__ __attribute__((aligned(16))) uint32_t s_rows[];  // [B][slot_dw]
  __shared__ long long s_idx[kMaxB];
  __shared__ long long s_D[kMaxB * kKPad];
  __shared__ double s_es[kMaxB * kKPad * 2];   // exponentials before / after
  __shared__ double s_rowst[kMaxB * 4];        // per row: max0, max1, sum0, sum1
  __shared__ int s_gam[kMaxB * kKPad];
  __shared__ __attribute__((aligned(4))) int8_t s_gamb[kKPad * kMaxB];  // 8 bits: gamma as bytes [class][row]
  __shared__ unsigned long long s_cnt[3];
  __shared__ int s_clambda;
  if (tid < 3) s_cnt[tid] = 0;
  if (tid == 0) s_clambda = 0;
  for (int e = tid; e < kKPad * kMaxB / 4; e += NT) reinterpret_cast<int*>(s_gamb)[e] = 0;  // rows past B stay 0

  const double delta_m = sc[0], inv_s = sc[5];
  const double dscale = __dmul_rn(a.delta_d, delta_m);
  const double alpha = a.hyper[2 * chain];
  const double aB = __ddiv_rn(alpha, (double)Bt);
  const bool lp = a.lp != 0;
  // the margin after the move: Algorithm 4 adds x^T z to phi, in Algorithm 2 x^T w is all of it
  auto after_margin = [&](double a0, long long D) {
    const double delta = __dmul_rn(dscale, (double)D);
    return lp ? delta : __dadd_rn(a0, delta);
  };
  constexpr int QMAX = (1 << (BITS - 1)) - 1, QMIN = -(1 << (BITS - 1));
  const double qmaxd = (double)QMAX, qmind = (double)QMIN;

  // ---- class wave state
  const bool class_wave = wave < K;
  const int cls = class_wave ? wave : 0;
  const int NACT = (U + UPL - 1) / UPL;        // lanes that hold part of the row
  const bool lane_ok = class_wave && lane < NACT;
  const int s0 = lane_ok ? lane * UPL : 0;     // first strip of this lane
  const int j0 = s0 * CT;
  const int nvalid = lane_ok ? min(CPL, d - j0) : 0;
  int z[CPL];
  int hv[CPL];
#pragma unroll
  for (int k = 0; k < CPL; ++k) {
    const bool ok = k < nvalid;
    z[k] = ok ? (int)zg[(int64_t)cls * d + j0 + k] : 0;
    hv[k] = ok ? (int)hg[(int64_t)cls * d + j0 + k] : 0;
  }
  U4 zblk[UPL];
  unsigned long long my_zclamp = 0, my_gclamp = 0;
  const uint4* frag = reinterpret_cast<const uint4*>(s_rows) + (s0 * 2) / 16;  // + m * slot_dw / 4
  auto x_of = [&](const uint4 (&f)[FQ], int k) {
    const uint4& q = f[(k * BITS) / 128];
    const int w = ((k * BITS) % 128) / 32;
    const uint32_t xv = w == 0 ? q.x : (w == 1 ? q.y : (w == 2 ? q.z : q.w));
    const int sh = (k * BITS) % 32;
    return BITS == 8 ? (int)(int8_t)(xv >> sh) : (int)(int16_t)(xv >> sh);
  };
  __syncthreads();

  const int64_t T = epoch_steps(seed, a.epoch, a.T, a.option2);
  for (int64_t t = 0; t < T; ++t) {
    // sum_m gamma_{m,c} x_m over the whole minibatch, and c_lambda: class waves, across the chunks
    AccT gsum[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) gsum[k] = 0;
    int cl = 0;
    for (int mb = 0; mb < (MANY ? Bt : 1); mb += kMaxB) {
    const int B = min(kMaxB, Bt - mb);  // rows of this chunk: mb .. mb + B - 1 of the step
    // sample i uniformly (with replacement)
    if (tid < B) {
      const uint64_t nn = (uint64_t)t * (uint64_t)Bt + (uint64_t)(mb + tid);
      const uint32_t r = pick(stream_block(seed, kIdx, a.epoch, nn >> 2), (uint32_t)(nn & 3));
      s_idx[tid] = (long long)(((uint64_t)r * (uint64_t)N) >> 32);
    }
    if (mb == 0 && tid == 0 && a.lambda > 0) {  // c_lambda = Q_(2^-b, b)(alpha lambda)
      const uint32_t r = pick(stream_block(seed, kReg, a.epoch, (uint64_t)t >> 2), (uint32_t)(t & 3));
      const int clq = (int)quantize_real(__dmul_rn(alpha, a.lambda), (double)(1 << BITS), r, 0.0,
                                         qmaxd, nullptr);
      s_clambda = clq;
      if (clq != 0) s_cnt[2] += 1;
    }
    __syncthreads();
    // the B rows into LDS: both the dot products and the update read them there
    // (a wave takes whole rows, 256 bytes per load, and has all loads of a row in flight at once)
#pragma unroll 2
    for (int m = wave; m < B; m += NW) {
      const uint32_t* src = reinterpret_cast<const uint32_t*>(Xq + s_idx[m] * ldxq * (BITS / 8));
      uint32_t v[kRowLoads];
#pragma unroll
      for (int i = 0; i < kRowLoads; ++i)
        if (i < nq) v[i] = src[min(lane + 64 * i, copy_dw - 1)];
#pragma unroll
      for (int i = 0; i < kRowLoads; ++i)
        if (i < nq && lane + 64 * i < copy_dw) s_rows[m * slot_dw + lane + 64 * i] = v[i];
    }
    __syncthreads();
    // integer dot products x_m^T z_c
    if (class_wave) {
      int zpk[BITS == 8 ? CPL / 4 : 1];  // 8 bits: z as bytes, four to a register
      if constexpr (BITS == 8) {
#pragma unroll
        for (int q = 0; q < CPL / 4; ++q)
          zpk[q] = (z[4 * q] & 0xff) | ((z[4 * q + 1] & 0xff) << 8) | ((z[4 * q + 2] & 0xff) << 16) |
                   (int)((uint32_t)z[4 * q + 3] << 24);
      }
#pragma unroll 4
      for (int m = 0; m < B; ++m) {  // four rows at a time: their reads and folds overlap
        uint4 f[FQ];
#pragma unroll
        for (int q = 0; q < FQ; ++q) f[q] = frag[m * (slot_dw / 4) + q];
        AccT acc = 0;
        if constexpr (BITS == 8) {  // four coordinates per instruction, z as packed bytes
          int a32 = 0;
#pragma unroll
          for (int q = 0; q < CPL / 4; ++q) {
            const uint4& fq = f[q / 4];
            const uint32_t xv = q % 4 == 0 ? fq.x : (q % 4 == 1 ? fq.y : (q % 4 == 2 ? fq.z : fq.w));
            a32 = __builtin_amdgcn_sdot4((int)xv, zpk[q], a32, false);
          }
          acc = a32;
        } else {
#pragma unroll
          for (int k = 0; k < CPL; ++k) acc += (AccT)(x_of(f, k) * z[k]);  // |x z| < 2^30; z = 0 past the row
        }
        long long tot;
        if (BITS == 8) tot = (long long)wave_sum_i32((int)acc);
        else tot = wave_sum_i64((long long)acc);
        if (lane == 0) s_D[m * K + cls] = tot;
      }
    }
    __syncthreads();
    // beta = (alpha/B)(p_c(phi_i + x_i^T z) - p_c(phi_i)); gamma = Q_(delta_s, b)(beta).
    // The normalisers are formed per row, the exponentials summed pairwise over adjacent classes.
    if (softmax) {
    if (tid < B) {
      const long long i = s_idx[tid];
      double mx0 = (double)phi[i * K];
      double mx1 = after_margin(mx0, s_D[tid * K]);
      for (int c = 1; c < K; ++c) {
        const double a0 = (double)phi[i * K + c];
        const double a1 = after_margin(a0, s_D[tid * K + c]);
        if (a0 > mx0) mx0 = a0;
        if (a1 > mx1) mx1 = a1;
      }
      s_rowst[4 * tid + 0] = mx0;
      s_rowst[4 * tid + 1] = mx1;
    }
    __syncthreads();
    for (int pr = tid; pr < B * K; pr += NT) {
      const int m = pr / K, c = pr - m * K;
      const double a0 = (double)phi[s_idx[m] * K + c];
      const double a1 = after_margin(a0, s_D[pr]);
      s_es[2 * pr + 0] = halp_exp(__dadd_rn(a0, -s_rowst[4 * m + 0]));
      s_es[2 * pr + 1] = halp_exp(__dadd_rn(a1, -s_rowst[4 * m + 1]));
    }
    __syncthreads();
    if (tid < B) {
      // pairwise over adjacent classes (absent classes count as +0), before, then after
#pragma unroll 1
      for (int side = 0; side < 2; ++side) {
        double v[kKPad / 2];
#pragma unroll
        for (int c = 0; c < kKPad / 2; ++c) {
          const double e0 = 2 * c < K ? s_es[2 * (tid * K + 2 * c) + side] : 0.0;
          const double e1 = 2 * c + 1 < K ? s_es[2 * (tid * K + 2 * c + 1) + side] : 0.0;
          v[c] = __dadd_rn(e0, e1);
        }
#pragma unroll
        for (int P = kKPad / 2; P > 1; P /= 2) {
#pragma unroll
          for (int c = 0; c < P / 2; ++c) v[c] = __dadd_rn(v[2 * c], v[2 * c + 1]);
        }
        s_rowst[4 * tid + 2 + side] = v[0];
      }
    }
    __syncthreads();
    }
    for (int pr = tid; pr < B * K; pr += NT) {
      const int m = pr / K, c = pr - m * K;
      double diff;
      if (softmax) {
        const double p0 = __ddiv_rn(s_es[2 * pr + 0], s_rowst[4 * m + 2]);
        const double p1 = __ddiv_rn(s_es[2 * pr + 1], s_rowst[4 * m + 3]);
        diff = __dadd_rn(p1, -p0);
      } else {
        const long long i = s_idx[m];
        const double delta = __dmul_rn(dscale, (double)s_D[pr]);
        if (a.loss == HALP_LOSS_SQUARED) {
          // Algorithm 4: (phi + Delta - y) - (phi - y) = Delta; Algorithm 2: (x^T w - y) - (phi - y)
          diff = lp ? __dadd_rn(delta, -(double)phi[i]) : delta;
        } else {
          const double a0 = (double)phi[i], yi = (double)y[i];
          diff = __dadd_rn(logistic_dl(after_margin(a0, s_D[pr]), yi), -logistic_dl(a0, yi));
        }
      }
      const double beta = __dmul_rn(aB, diff);
      const uint64_t nn = ((uint64_t)t * (uint64_t)Bt + (uint64_t)(mb + m)) * (uint64_t)K + (uint64_t)c;
      const uint32_t r = pick(stream_block(seed, kGamma, a.epoch, nn >> 2), (uint32_t)(nn & 3));
      bool hit = false;
      const int gq = (int)quantize_real(beta, inv_s, r, qmind, qmaxd, &hit);
      s_gam[pr] = gq;
      if constexpr (BITS == 8) s_gamb[c * kMaxB + m] = (int8_t)gq;
      if (hit) my_gclamp += 1;
    }
    if constexpr (BITS == 8) {  // the update takes rows in fours: no gamma for the rows past the chunk
      if (tid < 4 * K) {
        const int m = B + (tid & 3);
        if (m < ((B + 3) & ~3)) s_gamb[(tid >> 2) * kMaxB + m] = 0;
      }
    }
    __syncthreads();
    // u = z - sum_m gamma_m x_m - h~ (- c_lambda z) in (delta_i, 2b); z = Q_(delta_m, b)(u)
    if (class_wave) {
      cl = s_clambda;
      if constexpr (BITS == 8) {
        // four rows at a time: their bytes of a coordinate are brought into one register (a 4 x 4
        // byte transpose per dword of the fragments) and meet the rows' four gammas in one
        // 4-way dot product
        for (int m = 0; m < B; m += 4) {
          uint4 f[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) f[i] = frag[min(m + i, B - 1) * (slot_dw / 4)];  // gamma is 0 past B
          const int g4 = reinterpret_cast<const int*>(s_gamb)[(cls * kMaxB + m) >> 2];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            auto dw = [&](const uint4& v) { return q == 0 ? v.x : (q == 1 ? v.y : (q == 2 ? v.z : v.w)); };
            const uint32_t ra = dw(f[0]), rb = dw(f[1]), rc = dw(f[2]), rd = dw(f[3]);
            const uint32_t ab_lo = __builtin_amdgcn_perm(rb, ra, 0x05010400u), ab_hi = __builtin_amdgcn_perm(rb, ra, 0x07030602u);
            const uint32_t cd_lo = __builtin_amdgcn_perm(rd, rc, 0x05010400u), cd_hi = __builtin_amdgcn_perm(rd, rc, 0x07030602u);
            const uint32_t t0 = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x05040100u), t1 = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x07060302u);
            const uint32_t t2 = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x05040100u), t3 = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x07060302u);
            gsum[4 * q + 0] = __builtin_amdgcn_sdot4((int)t0, g4, (int)gsum[4 * q + 0], false);
            gsum[4 * q + 1] = __builtin_amdgcn_sdot4((int)t1, g4, (int)gsum[4 * q + 1], false);
            gsum[4 * q + 2] = __builtin_amdgcn_sdot4((int)t2, g4, (int)gsum[4 * q + 2], false);
            gsum[4 * q + 3] = __builtin_amdgcn_sdot4((int)t3, g4, (int)gsum[4 * q + 3], false);
          }
        }
      } else {
#pragma unroll 4
        for (int m = 0; m < B; ++m) {
          uint4 f[FQ];
#pragma unroll
          for (int q = 0; q < FQ; ++q) f[q] = frag[m * (slot_dw / 4) + q];
          const int g = s_gam[m * K + cls];
#pragma unroll
          for (int k = 0; k < CPL; ++k) gsum[k] += (AccT)g * (AccT)x_of(f, k);
        }
      }
    }
    __syncthreads();  // the rows, indices and gammas of this chunk are done with
    }
    if (class_wave) {
      if ((t & 7) == 0) {
#pragma unroll
        for (int u = 0; u < UPL; ++u)
          zblk[u] = zround_block(seed, a.epoch, (uint32_t)(cls * U + s0 + u), (uint32_t)(t >> 3));
      }
#pragma unroll
      for (int u = 0; u < UPL; ++u) {
        const uint32_t field = zround_field(zblk[u], (uint32_t)t);
#pragma unroll
        for (int e = 0; e < CT; ++e) {
          const int k = u * CT + e;
          if (k < nvalid) {
            const long long zk = z[k];
            const long long v = -(long long)hv[k] - (long long)cl * zk - (long long)gsum[k];
            const long long rb = (long long)((field >> (e * BITS)) & ((1u << BITS) - 1u));
            long long zn = zk + ((v + rb) >> BITS);  // arithmetic shift: floor
            if (zn > QMAX) { zn = QMAX; my_zclamp += 1; }
            if (zn < QMIN) { zn = QMIN; my_zclamp += 1; }
            z[k] = (int)zn;
          }
        }
      }
    }
  }

  // w~ <- w~ + delta_m z (option I), and hand z out
  if (class_wave) {
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
      if (k < nvalid) {
        const int64_t o = (int64_t)cls * d + j0 + k;
        zg[o] = (XT)z[k];
        const double step = __dmul_rn(delta_m, (double)z[k]);
        wg[o] = lp ? (float)step : (float)__dadd_rn((double)wg[o], step);  // Alg. 2: w~ = delta w
      }
    }
  }
  if (my_zclamp) atomicAdd(&s_cnt[0], my_zclamp);
  if (my_gclamp) atomicAdd(&s_cnt[1], my_gclamp);
  __syncthreads();
  if (tid < 4) cnt_out[tid] = tid < 3 ? s_cnt[tid] : 0ull;
}

// strips per lane: 8 up to 512 strips per row, 16 (16 bits only) up to 1024
int strips_per_lane(const halp_params& p) {
  const int ct = 16 / p.b;
  const int U = (p.d + ct - 1) / ct;
  if (U <= 512) return 8;
  return (p.b == 16 && U <= 1024) ? 16 : 0;
}

// bytes of a row's slot in LDS: whole fragments for every lane on the row
int slot_bytes_of(const halp_params& p, int upl) {
  const int ct = 16 / p.b;
  const int U = (p.d + ct - 1) / ct;
  return (U + upl - 1) / upl * upl * 2;
}

template <int BITS, int UPL, int WAVES>
int launch_waves(const InArgs& a, int R, int slot_bytes, hipStream_t s) {
  const size_t smem = (size_t)std::min(a.B, kMaxB) * slot_bytes;
  auto kern = a.B > kMaxB ? inner_softmax_batch_kernel<BITS, UPL, WAVES, true>
                          : inner_softmax_batch_kernel<BITS, UPL, WAVES, false>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)smem) != hipSuccess)
    return HALP_ERR_HIP;
  hipLaunchKernelGGL(kern, dim3(R), dim3(64 * std::min(a.K + 1, 16)), smem, s, a, slot_bytes);
  return hip_ok(hipGetLastError());
}

template <int BITS, int UPL>
int launch_one(const InArgs& a, int R, int slot_bytes, hipStream_t s) {
  if (a.K + 1 <= 8) return launch_waves<BITS, UPL, 8>(a, R, slot_bytes, s);
  if (a.K + 1 <= 12) return launch_waves<BITS, UPL, 12>(a, R, slot_bytes, s);
  return launch_waves<BITS, UPL, 16>(a, R, slot_bytes, s);
}

}  // namespace

int inner_softmax_batch_supported(const halp_handle& h) {
  const halp_params& p = h.p;
  if (p.B < 2 || p.B > 512 || p.K > kMaxK) return HALP_ERR_UNSUPPORTED;
  // softmax; or a scalar margin with more rows per step than the kernel for that case takes
  if (p.loss == HALP_LOSS_SOFTMAX ? p.K < 2 : (p.K != 1 || p.B <= 64)) return HALP_ERR_UNSUPPORTED;
  const int upl = strips_per_lane(p);
  if (upl == 0) return HALP_ERR_UNSUPPORTED;
  if (!h.bound || !h.buf.Xq) return HALP_ERR_NOT_BOUND;
  // 128 KB of rows beside the 31 KB of per-step scalars
  if ((size_t)std::min(p.B, kMaxB) * slot_bytes_of(p, upl) > 128 * 1024) return HALP_ERR_UNSUPPORTED;
  return HALP_OK;
}

int launch_inner_softmax_batch(const halp_handle& h, uint32_t epoch, hipStream_t s) {
  const halp_params& p = h.p;
  const int rc = inner_softmax_batch_supported(h);
  if (rc != HALP_OK) return rc;
  const InArgs a = make_inner_args(h, epoch);
  const int upl = strips_per_lane(p);
  const int slot = slot_bytes_of(p, upl);
  if (p.b == 8) return launch_one<8, 8>(a, p.R, slot, s);
  return upl == 8 ? launch_one<16, 8>(a, p.R, slot, s) : launch_one<16, 16>(a, p.R, slot, s);
}

}  // namespace halp
