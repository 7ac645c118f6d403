// Inner loop of Algorithm 4 (LM-HALP), register-resident form for one sampled
// row per step (B = 1) and one class (squared or logistic loss).  This header
// holds the kernel template; inner_reg_b8.hip / inner_reg_b16.hip instantiate it.
//
// One workgroup per chain, NW waves.  A row of z is cut into strips of 16
// rounding bits (two int8 or one int16 coordinate, i.e. 2 bytes of a data row);
// lane l of wave w owns the UPL consecutive strips starting at (64 w + l) UPL.
// z, -h~, the strips' Philox blocks and a ring of prefetched row fragments stay
// in registers for the whole epoch; inside the loop only the sampled rows are
// read from memory.  Per step:
//   dot      per-lane 24-bit multiply-adds, folded across the wave with DPP and,
//            when NW > 1, across waves through one LDS word per wave and a barrier
//   scalar   beta and gamma = Q_(delta_s,b)(beta) in fp64, wave-uniform
//   update   u = -gamma x - h~ (- c_lambda z) in (delta_i, 2b), stochastic
//            rounding with b Philox bits per coordinate, clamp to the box
// One wave per chain gives the best throughput when chains are many; several
// waves per chain cut the step latency (each wave carries a fraction of the
// Philox and update work) at the price of one barrier per step.
//
// Everything that depends on the step number only -- sample indices, the
// rounding draws of gamma and of the L2 term -- is produced 256 steps at a time
// into LDS and pulled into registers one window of 8 steps at a time; a window
// is also the span one Philox block per strip covers, and row fragments are
// requested one window ahead.  The steady-state loop over full windows has no
// data-dependent branches, so outstanding loads are waited for one at a time.
#pragma once

#include "halp_device.hpp"
#include "inner_args.hpp"

namespace halp {
namespace innerreg {

constexpr int kBatch = 256;  // steps per batch of precomputed draws
constexpr int kWin = 8;      // steps per window

__device__ __forceinline__ double logistic_dl(double a, double y) {
  return __ddiv_rn(-y, __dadd_rn(1.0, halp_exp(__dmul_rn(y, a))));
}

// a * b + c on the 24-bit multiplier; a and b must fit 24 bits (they are codes of at most
// 16 bits here).  Written as the instruction because the compiler cannot see the range of
// a value that comes out of a float conversion and would re-extend it first.
__device__ __forceinline__ int mad24(int a, int b, int c) {
  int r;
  asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

typedef short short2r __attribute__((ext_vector_type(2)));  // the two coordinates of an 8-bit strip

// squared loss whose step needs the margin phi_i of w~ (LP-SVRG); a value apart from HALP_LOSS_*
constexpr int kLossSquaredWithMargins = 3;

// PKF: the 8-bit strips are updated as packed 16-bit halves (one wave per chain only).
template <int BITS, int LOSS, int UPL, int NWT, bool PKF = false>
__global__ __launch_bounds__(64 * NWT) void inner_reg_kernel(InArgs a) {
  static_assert(!PKF || (BITS == 8 && NWT == 1), "the packed form is built for 8 bits, one wave per chain");
  constexpr bool COUNT = true;  // clamped coordinates are always counted
  using XT = typename std::conditional<BITS == 8, int8_t, int16_t>::type;
  using HT = typename std::conditional<BITS == 8, int16_t, int32_t>::type;
  using AccT = typename std::conditional<BITS == 8, int, long long>::type;
  constexpr int CT = 16 / BITS;          // coordinates per strip
  constexpr int CPL = UPL * CT;          // coordinates per lane
  constexpr int NDW = (UPL + 1) / 2;     // dwords of row data per lane and step
  constexpr int QMAX = (1 << (BITS - 1)) - 1, QMIN = -(1 << (BITS - 1));
  constexpr int kMask = 2 * kBatch - 1;
  const int chain = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = NWT > 1 ? __builtin_amdgcn_readfirstlane(tid >> 6) : 0;
  const int d = a.d;
  const int U = (d + CT - 1) / CT;  // strips in a row
  const uint32_t N = (uint32_t)a.N;
  const int64_t row_bytes = a.ldxq * (BITS / 8);
  const unsigned char* __restrict__ Xq = reinterpret_cast<const unsigned char*>(a.Xq) +
                                         (int64_t)chain * a.xq_chain_stride * (BITS / 8);
  const float* __restrict__ phi = a.phi + (int64_t)chain * a.N;
  const float* __restrict__ y =
      reinterpret_cast<const float*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const HT* __restrict__ hg = reinterpret_cast<const HT*>(a.h) + (int64_t)chain * d;
  XT* __restrict__ zg = reinterpret_cast<XT*>(a.z) + (int64_t)chain * d;
  float* __restrict__ wg = a.w + (int64_t)chain * d;
  const double* sc = a.scales + (int64_t)chain * 8;
  uint64_t* cnt_out = a.counters + (int64_t)chain * 4;
  const uint64_t seed = a.seed + (uint64_t)chain;
  const int64_t T = epoch_steps(seed, a.epoch, a.T, a.option2);

  if (sc[7] != 0.0) {  // converged or unusable gradient: the epoch is a no-op
    if (tid < 4) cnt_out[tid] = 0;
    return;
  }

  __shared__ __attribute__((aligned(16))) int s_idx[2 * kBatch];
  __shared__ __attribute__((aligned(16))) double s_rho[2 * kBatch];
  __shared__ __attribute__((aligned(16))) int s_creg[2 * kBatch];
  __shared__ __attribute__((aligned(16))) float s_phi[2 * kBatch];  // logistic: margins and labels
  __shared__ __attribute__((aligned(16))) float s_y[2 * kBatch];    // of the sampled rows
  // logistic loss: l'(phi_i) of the sampled rows, evaluated four per lane when a batch is drawn
  // instead of once per step by the whole wave
  __shared__ __attribute__((aligned(16))) double s_dl0[LOSS == HALP_LOSS_LOGISTIC ? 2 * kBatch : 2];
  __shared__ __attribute__((aligned(16))) AccT s_part[2][16];
  __shared__ unsigned long long s_cnt[3];
  __shared__ AccT s_dump[NWT > 1 ? 64 * NWT : 1];  // where lanes 0..62 of a wave put their partial folds
  using LdsAcc = __attribute__((address_space(3))) AccT;
  LdsAcc* const slot0 = (LdsAcc*)((NWT > 1 && lane != 63) ? &s_dump[tid] : &s_part[0][wave]);
  LdsAcc* const slot1 = (LdsAcc*)((NWT > 1 && lane != 63) ? &s_dump[tid] : &s_part[1][wave]);

  const double delta_m = sc[0], inv_s = sc[5];
  const double dscale = __dmul_rn(a.delta_d, delta_m);
  const double aB = a.hyper[2 * chain];  // B = 1: alpha / 1
  const bool use_reg = a.lambda > 0;
  constexpr bool logistic = LOSS == HALP_LOSS_LOGISTIC;
  constexpr bool need_phi = LOSS != HALP_LOSS_SQUARED;  // logistic, or squared loss of LP-SVRG
  const bool lp = a.lp != 0;
  const double al = __dmul_rn(aB, a.lambda);

  // ---- per-lane state
  const int s0 = (wave * 64 + lane) * UPL;  // first strip of the lane
  const int j0 = s0 * CT;                   // first coordinate
  const bool lane_ok = s0 < U;              // the lane owns at least one strip
  int z[CPL];
  int hv[CPL];  // -h~ when b = 8; h~ itself when b = 16 (its negation may not fit 32 bits)
  uint32_t xmask[NDW];  // bytes of a fragment that are coordinates < d
#pragma unroll
  for (int k = 0; k < NDW; ++k) xmask[k] = 0;
#pragma unroll
  for (int k = 0; k < CPL; ++k) {
    const int j = j0 + k;
    const bool ok = j < d;
    z[k] = ok ? (int)zg[j] : 0;
    hv[k] = ok ? (BITS == 8 ? -(int)hg[j] : (int)hg[j]) : 0;
    if (ok) xmask[(k * BITS) / 32] |= (BITS == 8 ? 0xFFu : 0xFFFFu) << ((k * BITS) % 32);
  }

  // Packed form: between windows z lives packed, the two coordinates of a strip as the 16-bit
  // halves of one register, next to -h~ = 256 hh + hl cut the same way (0 <= hl < 256).
  // Windows without an L2 draw run on these with packed 16-bit arithmetic.
  short2r zp[UPL], hlp[UPL], hhp[UPL];
#pragma unroll
  for (int u = 0; u < UPL; ++u) {
    const int k0 = BITS == 8 ? 2 * u : 0, k1 = BITS == 8 ? 2 * u + 1 : 0;
    zp[u] = short2r{(short)z[k0], (short)z[k1]};
    hlp[u] = short2r{(short)(hv[k0] & 0xFF), (short)(hv[k1] & 0xFF)};
    hhp[u] = short2r{(short)(hv[k0] >> 8), (short)(hv[k1] >> 8)};
  }
  auto unpack_z = [&]() {
    if (PKF) {
#pragma unroll
      for (int k = 0; k < CPL; ++k) z[k] = (int)zp[(k / 2) % UPL][k % 2];
    }
  };
  auto pack_z = [&]() {
    if (PKF) {
#pragma unroll
      for (int u = 0; u < UPL; ++u) zp[u] = short2r{(short)z[(2 * u) % CPL], (short)z[(2 * u + 1) % CPL]};
    }
  };

  // ---- draws that depend on the step number only, 256 steps per batch
  auto fill_batch = [&](int64_t bb) {
    const int half = (int)(bb & 1) * kBatch;
    if (tid < 64) {
      const uint64_t blk = (uint64_t)bb * 64 + (uint64_t)tid;
      const U4 ri = stream_block(seed, kIdx, a.epoch, blk);
      const U4 rg = stream_block(seed, kGamma, a.epoch, blk);
      int4 iv;
      iv.x = (int)__umulhi(ri.x, N); iv.y = (int)__umulhi(ri.y, N);
      iv.z = (int)__umulhi(ri.z, N); iv.w = (int)__umulhi(ri.w, N);
      *reinterpret_cast<int4*>(&s_idx[half + 4 * tid]) = iv;
      if (need_phi) {  // gather phi_i (and y_i) of the batch's rows here, off the step path
        float4 pv;
        pv.x = phi[iv.x]; pv.y = phi[iv.y]; pv.z = phi[iv.z]; pv.w = phi[iv.w];
        *reinterpret_cast<float4*>(&s_phi[half + 4 * tid]) = pv;
      }
      if (logistic) {
        float4 yv;
        yv.x = y[iv.x]; yv.y = y[iv.y]; yv.z = y[iv.z]; yv.w = y[iv.w];
        *reinterpret_cast<float4*>(&s_y[half + 4 * tid]) = yv;
        const float4 pw = *reinterpret_cast<const float4*>(&s_phi[half + 4 * tid]);
        s_dl0[half + 4 * tid + 0] = logistic_dl((double)pw.x, (double)yv.x);
        s_dl0[half + 4 * tid + 1] = logistic_dl((double)pw.y, (double)yv.y);
        s_dl0[half + 4 * tid + 2] = logistic_dl((double)pw.z, (double)yv.z);
        s_dl0[half + 4 * tid + 3] = logistic_dl((double)pw.w, (double)yv.w);
      }
      s_rho[half + 4 * tid + 0] = __dmul_rn((double)rg.x, 0x1p-32);
      s_rho[half + 4 * tid + 1] = __dmul_rn((double)rg.y, 0x1p-32);
      s_rho[half + 4 * tid + 2] = __dmul_rn((double)rg.z, 0x1p-32);
      s_rho[half + 4 * tid + 3] = __dmul_rn((double)rg.w, 0x1p-32);
      if (use_reg) {
        const U4 rr = stream_block(seed, kReg, a.epoch, blk);
        const double two_b = (double)(1 << BITS);
        int4 cv;
        cv.x = (int)quantize_real(al, two_b, rr.x, 0.0, (double)QMAX, nullptr);
        cv.y = (int)quantize_real(al, two_b, rr.y, 0.0, (double)QMAX, nullptr);
        cv.z = (int)quantize_real(al, two_b, rr.z, 0.0, (double)QMAX, nullptr);
        cv.w = (int)quantize_real(al, two_b, rr.w, 0.0, (double)QMAX, nullptr);
        *reinterpret_cast<int4*>(&s_creg[half + 4 * tid]) = cv;
      }
    }
  };
  if (tid < 3) s_cnt[tid] = 0;
  if (tid < 32) (&s_part[0][0])[tid] = 0;
  fill_batch(0);
  fill_batch(1);
  __syncthreads();

  // ---- prefetched row fragments: two buffers of one window (8 steps) each.  While a window
  // runs on one buffer, the fragments of the next window are in flight into the other; they
  // are all requested at the top of the window, a full window before they are used.
  // Every lane loads (lanes past the end of the row re-read its first bytes and mask them
  // away), so there are no divergent loads in the loop.
  uint32_t xa[kWin][NDW], xb[kWin][NDW];
  // byte offset of the lane's fragment inside a row; a 2-byte fragment is fetched as the
  // aligned dword around it (rows are 8-byte aligned) and shifted into place
  const int lane_off = lane_ok ? (UPL == 1 ? (s0 * 2) & ~3 : s0 * 2) : 0;
  const int half_sh = (UPL == 1 && lane_ok) ? ((s0 * 2) & 2) * 8 : 0;
#pragma unroll
  for (int s = 0; s < kWin; ++s) {
#pragma unroll
    for (int k = 0; k < NDW; ++k) xa[s][k] = xb[s][k] = 0;
  }
  auto request = [&](uint32_t (&dst)[NDW], int i) {
    const unsigned char* rp = Xq + (int64_t)i * row_bytes + lane_off;
    if (UPL <= 2) {
      dst[0] = *reinterpret_cast<const uint32_t*>(rp);
    } else if (UPL == 4) {
      const uint2 v = *reinterpret_cast<const uint2*>(rp);
      dst[0] = v.x;
      dst[NDW > 1 ? 1 : 0] = v.y;
    } else {
      const uint4 v = *reinterpret_cast<const uint4*>(rp);
      dst[0] = v.x;
      dst[NDW > 1 ? 1 : 0] = v.y;
      dst[NDW > 2 ? 2 : 0] = v.z;
      dst[NDW > 3 ? 3 : 0] = v.w;
    }
  };
#pragma unroll
  for (int s = 0; s < kWin; ++s) {
    if (s < T) request(xa[s], __builtin_amdgcn_readfirstlane(s_idx[s]));
  }

  unsigned int n_zclamp = 0, n_gclamp = 0, n_reg = 0;
  unsigned int n_zclamp_wave = 0;  // the same count kept for the whole wave (uniform)
  U4 zr[UPL];  // the strips' rounding blocks for the current window

  // One window of 8 steps starting at t0 (a multiple of 8).  FULL: all 8 steps
  // exist and so do the 8 steps after them, so nothing inside is conditional.
  auto window = [&](int64_t t0, auto full_tag, auto reg_tag, const int (&creg)[kWin],
                    uint32_t (&xr)[kWin][NDW], uint32_t (&xnext)[kWin][NDW]) {
    constexpr bool FULL = decltype(full_tag)::value;
    constexpr bool REGW = decltype(reg_tag)::value;  // some step of the window has c_lambda != 0
    // Packed arithmetic on zp: fewer instructions per strip but a longer dependent chain and a
    // branch per step, so it is for many chains per SIMD, where issue slots are what runs out;
    // chains that wait on their own dependent chain keep the scalar form.
    constexpr bool PK = PKF && !REGW;
    if (!PK) unpack_z();
    const int base = (int)(t0 & kMask);  // multiple of 8: the window is contiguous in LDS
    // draws of this window and the row indices of the next one, in a few wide LDS reads
    double rho[kWin];
    int nidx[kWin];
    float phi8[kWin], y8[kWin];
    double dl08[kWin];
#pragma unroll
    for (int s = 0; s < kWin; ++s) {
      phi8[s] = y8[s] = 0.f;
      dl08[s] = 0.0;
    }
    if (need_phi) {
      const float4 p0 = *reinterpret_cast<const float4*>(&s_phi[base]);
      const float4 p1 = *reinterpret_cast<const float4*>(&s_phi[base + 4]);
      phi8[0] = p0.x; phi8[1] = p0.y; phi8[2] = p0.z; phi8[3] = p0.w;
      phi8[4] = p1.x; phi8[5] = p1.y; phi8[6] = p1.z; phi8[7] = p1.w;
    }
    if (logistic) {
      const float4 y0 = *reinterpret_cast<const float4*>(&s_y[base]);
      const float4 y1 = *reinterpret_cast<const float4*>(&s_y[base + 4]);
      y8[0] = y0.x; y8[1] = y0.y; y8[2] = y0.z; y8[3] = y0.w;
      y8[4] = y1.x; y8[5] = y1.y; y8[6] = y1.z; y8[7] = y1.w;
#pragma unroll
      for (int s = 0; s < kWin; s += 2) {
        const double2 d2 = *reinterpret_cast<const double2*>(&s_dl0[base + s]);
        dl08[s] = d2.x;
        dl08[s + 1] = d2.y;
      }
    }
#pragma unroll
    for (int s = 0; s < kWin; s += 2) {
      const double2 r2 = *reinterpret_cast<const double2*>(&s_rho[base + s]);
      rho[s] = r2.x;
      rho[s + 1] = r2.y;
    }
    {
      const int nb = (base + kWin) & kMask;
      const int4 i0 = *reinterpret_cast<const int4*>(&s_idx[nb]);
      const int4 i1 = *reinterpret_cast<const int4*>(&s_idx[nb + 4]);
      nidx[0] = i0.x; nidx[1] = i0.y; nidx[2] = i0.z; nidx[3] = i0.w;
      nidx[4] = i1.x; nidx[5] = i1.y; nidx[6] = i1.z; nidx[7] = i1.w;
    }
    // Take this window's fragments out of the load buffer (shift / mask them into place)
    // before anything new is requested: the wait for them then never covers the loads of
    // the next window, which stay in flight for the whole window.
    uint32_t xw[kWin][NDW];
#pragma unroll
    for (int s = 0; s < kWin; ++s) {
#pragma unroll
      for (int k = 0; k < NDW; ++k) xw[s][k] = (UPL == 1 ? xr[s][k] >> half_sh : xr[s][k]) & xmask[k];
    }
    __builtin_amdgcn_sched_barrier(0);
    // fragments of the next window
#pragma unroll
    for (int s = 0; s < kWin; ++s) {
      if (FULL || t0 + kWin + s < T) request(xnext[s], __builtin_amdgcn_readfirstlane(nidx[s]));
    }
    // rounding bits: one Philox block per strip serves the whole window
#pragma unroll
    for (int u = 0; u < UPL; ++u)
      zr[u] = zround_block(seed, a.epoch, (uint32_t)(s0 + u), (uint32_t)(t0 >> 3));

#pragma unroll
    for (int s = 0; s < kWin; ++s) {
      const int64_t t = t0 + s;
      if (FULL || t < T) {
        // low-precision dot product x_i^T z
        int xe[CPL];
        short2r xp[UPL];
        int part = 0, part_hi = 0;
        if (PK) {
          // the strip's two bytes go to the high bytes of the two halves and are shifted back
          // down with their signs; one packed dot per strip
#pragma unroll
          for (int u = 0; u < UPL; ++u) {
            const uint32_t up = __builtin_amdgcn_perm(0u, xw[s][u / 2], (u & 1) ? 0x030C020Cu : 0x010C000Cu);
            xp[u] = __builtin_bit_cast(short2r, up) >> (short2r)(8);
            part = __builtin_amdgcn_sdot2(xp[u], zp[u], part, false);
          }
        } else {
#pragma unroll
          for (int k = 0; k < CPL; ++k) {
            const uint32_t xv = xw[s][(k * BITS) / 32];
            const int sh = (k * BITS) % 32;
            xe[k] = BITS == 8 ? (int)(int8_t)(xv >> sh) : (int)(int16_t)(xv >> sh);
            if (BITS == 8) part = mad24(xe[k], z[k], part);
          }
        }
        AccT D;
        if (BITS == 8 && NWT > 1) {
          // the fold leaves the wave's sum in lane 63, which hands it to the other waves itself
          // (see below): no lane read, no scalar register on the way (the same at 16 bits)
          D = (AccT)wave_fold_i32(part);
        } else if (BITS == 8) {
          D = (AccT)wave_sum_i32(part);
        } else {
          // 16 bits: a product of two 16-bit factors, or the sum of two, fits 32 bits.  Each is
          // cut into its low 16 bits and the rest, and the two kinds are summed apart: both
          // sums stay far inside 32 bits over a whole wave, so two plain folds give the exact
          // 64-bit dot product.
          if (CPL == 1) {
            const int p = mad24(xe[0], z[0], 0);
            part = p & 0xFFFF;
            part_hi = p >> 16;
          } else {
#pragma unroll
            for (int k = 0; k + 1 < CPL; k += 2) {
              const int p = mad24(xe[k], z[k], mad24(xe[k + 1], z[k + 1], 0));
              part += p & 0xFFFF;
              part_hi += p >> 16;
            }
          }
          const int lo = NWT > 1 ? wave_fold_i32(part) : wave_sum_i32(part);
          const int hi = NWT > 1 ? wave_fold_i32(part_hi) : wave_sum_i32(part_hi);
          D = (AccT)(((long long)hi << 16) + (long long)lo);
        }
        if (NWT > 1) {
          // every lane stores, so no lane mask is set up: lane 63 (the holder of the sum) into
          // the wave's slot, the others into a dump row
          *((s & 1) ? slot1 : slot0) = D;
          __syncthreads();
          AccT q[NWT];
#pragma unroll
          for (int w2 = 0; w2 < NWT; ++w2) q[w2] = s_part[s & 1][w2];
#pragma unroll
          for (int w = NWT / 2; w >= 1; w /= 2) {  // pairwise: two levels of adds for four waves
#pragma unroll
            for (int k = 0; k < w; ++k) q[k] += q[k + w];
          }
          D = q[0];
        }
        // beta = alpha (l'(phi_i + x_i^T z) - l'(phi_i)), gamma = Q_(delta_s, b)(beta)
        const double delta = __dmul_rn(dscale, (double)D);
        double diff = delta;  // squared loss of Algorithm 4: (phi + Delta - y) - (phi - y)
        if (logistic) {
          // Algorithm 4 moves the margin by x^T z; in Algorithm 2 x^T w is the whole margin
          const double a0 = (double)phi8[s], yi = (double)y8[s];
          const double a1 = lp ? delta : __dadd_rn(a0, delta);
          diff = __dadd_rn(logistic_dl(a1, yi), -dl08[s]);  // l'(phi_i) comes with the batch
        } else if (need_phi) {  // squared loss of Algorithm 2: (x^T w - y) - (phi - y)
          diff = __dadd_rn(delta, -(double)phi8[s]);
        }
        const double beta = __dmul_rn(aB, diff);
        const double f = floor(__dadd_rn(__dmul_rn(beta, inv_s), rho[s]));
        // -gamma = clamp(-f) taken in integers: the conversion saturates at the ends of int32,
        // far outside [-QMAX, -QMIN], so one integer median does what two fp64 ops did
        int nf;
        asm("v_cvt_i32_f64 %0, -%1" : "=v"(nf) : "v"(f));
        const int ng = min(max(nf, -QMAX), -QMIN);
        n_gclamp += (nf != ng) ? 1u : 0u;
        int cl = 0;
        if (REGW) {
          cl = __builtin_amdgcn_readfirstlane(creg[s]);
          n_reg += cl != 0 ? 1u : 0u;
        }
        // u = z - gamma x - h~ (- c_lambda z), z = Q_(delta_m, b)(u)
        if (PK) {
          // per half: floor((-gamma x + r + hl) / 256) + hh + z.  |gamma x| <= 128 * 128 and
          // r + hl < 512, so the numerator fits 16 bits, and so does the sum that is clamped.
          const short2r ngp = short2r{(short)ng, (short)ng};
          short2r zu[UPL];
          uint32_t moved = 0;  // bits in which some clamp changed a value
#pragma unroll
          for (int u = 0; u < UPL; ++u) {
            const uint32_t word = pick(zr[u], (uint32_t)(s >> 1));
            const uint32_t rp = __builtin_amdgcn_perm(0u, word, (s & 1) ? 0x0C030C02u : 0x0C010C00u);
            short2r v = xp[u] * ngp + (__builtin_bit_cast(short2r, rp) + hlp[u]);
            v = (v >> (short2r)(8)) + (hhp[u] + zp[u]);  // the sum in brackets does not wait for gamma
            const short2r zc = __builtin_elementwise_min(__builtin_elementwise_max(v, (short2r)(QMIN)),
                                                         (short2r)(QMAX));
            moved |= __builtin_bit_cast(uint32_t, v) ^ __builtin_bit_cast(uint32_t, zc);
            zu[u] = v;
            zp[u] = zc;
          }
          if (COUNT && __ballot(moved != 0) != 0) {  // rare: count the clamped coordinates exactly
#pragma unroll
            for (int u = 0; u < UPL; ++u) {
              const uint32_t df = __builtin_bit_cast(uint32_t, zu[u]) ^ __builtin_bit_cast(uint32_t, zp[u]);
              n_zclamp_wave += (unsigned int)__builtin_popcountll(__ballot((df & 0xFFFFu) != 0)) +
                               (unsigned int)__builtin_popcountll(__ballot((df >> 16) != 0));
            }
          }
        }
#pragma unroll
        for (int k = 0; k < (PK ? 0 : CPL); ++k) {
          const uint32_t word = pick(zr[k / CT], (uint32_t)(s >> 1));
          const int sh = 16 * (s & 1) + (k % CT) * BITS;
          const int re = (int)((word >> sh) & (BITS == 8 ? 0xFFu : 0xFFFFu));
          int zu;
          if (BITS == 8) {
            int v = mad24(ng, xe[k], hv[k] + re);
            if (REGW) v = mad24(-cl, z[k], v);
            zu = z[k] + (v >> 8);
          } else {
            // with h~ = 2^16 hh + hl, 0 <= hl < 2^16:
            // floor((-gamma x + r - h~ - c z) / 2^16) = floor((-gamma x + r - hl - c z) / 2^16) - hh,
            // and the numerator on the right stays below 2^31 in magnitude
            int v = mad24(ng, xe[k], re - (hv[k] & 0xFFFF));
            if (REGW) v = mad24(-cl, z[k], v);
            zu = z[k] + (v >> 16) - (hv[k] >> 16);
          }
          const int zc = min(max(zu, QMIN), QMAX);
          if (COUNT) {
            // one wave per chain is the shape of many chains per SIMD, where a count on the
            // scalar unit (lanes of the compare's mask) frees a vector issue slot
            if (PKF) n_zclamp_wave += (unsigned int)__builtin_popcountll(__ballot(zu != zc));
            else n_zclamp += (zu != zc) ? 1u : 0u;
          }
          z[k] = zc;
        }
      }
    }
    if (!PK) pack_z();
  };

  int64_t t0 = 0;
  auto refill = [&](int64_t tt) {
    if ((tt & (kBatch - 1)) == 0 && tt > 0) {
      // every wave has finished batch tt/256 - 1; its half is refilled with batch tt/256 + 1
      __syncthreads();
      fill_batch(tt / kBatch + 1);
      __syncthreads();
    }
  };
  // the L2 draws of a window; true if any is non-zero (rare: alpha lambda 2^b is tiny)
  auto load_creg = [&](int64_t tt, int (&creg)[kWin]) -> bool {
#pragma unroll
    for (int s = 0; s < kWin; ++s) creg[s] = 0;
    if (!use_reg) return false;
    const int base = (int)(tt & kMask);
    const int4 c0 = *reinterpret_cast<const int4*>(&s_creg[base]);
    const int4 c1 = *reinterpret_cast<const int4*>(&s_creg[base + 4]);
    creg[0] = c0.x; creg[1] = c0.y; creg[2] = c0.z; creg[3] = c0.w;
    creg[4] = c1.x; creg[5] = c1.y; creg[6] = c1.z; creg[7] = c1.w;
    const int any = c0.x | c0.y | c0.z | c0.w | c1.x | c1.y | c1.z | c1.w;
    return __builtin_amdgcn_readfirstlane(any) != 0;
  };
  int creg[kWin];
  // even windows run on xa and fill xb, odd windows the other way round
  for (; t0 + 3 * kWin <= T; t0 += 2 * kWin) {
    refill(t0);
    if (load_creg(t0, creg)) window(t0, std::true_type{}, std::true_type{}, creg, xa, xb);
    else window(t0, std::true_type{}, std::false_type{}, creg, xa, xb);
    refill(t0 + kWin);
    if (load_creg(t0 + kWin, creg)) window(t0 + kWin, std::true_type{}, std::true_type{}, creg, xb, xa);
    else window(t0 + kWin, std::true_type{}, std::false_type{}, creg, xb, xa);
  }
  for (; t0 < T; t0 += kWin) {
    refill(t0);
    load_creg(t0, creg);
    if (((t0 >> 3) & 1) == 0) window(t0, std::false_type{}, std::true_type{}, creg, xa, xb);
    else window(t0, std::false_type{}, std::true_type{}, creg, xb, xa);
  }

  // ---- w~ <- w~ + delta_m z (option I); hand z out
  unpack_z();
#pragma unroll
  for (int k = 0; k < CPL; ++k) {
    const int j = j0 + k;
    if (j < d) {
      zg[j] = (XT)z[k];
      const double step = __dmul_rn(delta_m, (double)z[k]);
      wg[j] = lp ? (float)step : (float)__dadd_rn((double)wg[j], step);  // Alg. 2: w~ = delta w
    }
  }
  if (COUNT && n_zclamp) atomicAdd(&s_cnt[0], (unsigned long long)n_zclamp);
  if (COUNT && lane == 0 && n_zclamp_wave) atomicAdd(&s_cnt[0], (unsigned long long)n_zclamp_wave);
  if (tid == 0) {
    s_cnt[1] = n_gclamp;  // gamma is uniform over the workgroup: count it once
    s_cnt[2] = n_reg;
  }
  __syncthreads();
  if (tid < 4) cnt_out[tid] = tid < 3 ? s_cnt[tid] : 0ull;
}

template <int BITS, int UPL, int NWT>
int launch_one(const InArgs& a, int R, bool packed, hipStream_t s) {
  const dim3 grid(R), block(64 * NWT);
  if constexpr (BITS == 8 && NWT == 1) {
    if (packed) {
      if (a.loss == HALP_LOSS_SQUARED && a.lp)
        hipLaunchKernelGGL((inner_reg_kernel<BITS, kLossSquaredWithMargins, UPL, NWT, true>), grid, block, 0, s, a);
      else if (a.loss == HALP_LOSS_SQUARED)
        hipLaunchKernelGGL((inner_reg_kernel<BITS, HALP_LOSS_SQUARED, UPL, NWT, true>), grid, block, 0, s, a);
      else
        hipLaunchKernelGGL((inner_reg_kernel<BITS, HALP_LOSS_LOGISTIC, UPL, NWT, true>), grid, block, 0, s, a);
      return hip_ok(hipGetLastError());
    }
  }
  if (a.loss == HALP_LOSS_SQUARED && a.lp)
    hipLaunchKernelGGL((inner_reg_kernel<BITS, kLossSquaredWithMargins, UPL, NWT>), grid, block, 0, s, a);
  else if (a.loss == HALP_LOSS_SQUARED)
    hipLaunchKernelGGL((inner_reg_kernel<BITS, HALP_LOSS_SQUARED, UPL, NWT>), grid, block, 0, s, a);
  else
    hipLaunchKernelGGL((inner_reg_kernel<BITS, HALP_LOSS_LOGISTIC, UPL, NWT>), grid, block, 0, s, a);
  return hip_ok(hipGetLastError());
}

// every (strips per lane, waves per chain) pair the library launches
template <int BITS>
int launch_bits(const InArgs& a, int nw, int upl, int R, bool packed, hipStream_t s) {
#define HALP_CASE(U_, W_) \
  if (upl == U_ && nw == W_) return launch_one<BITS, U_, W_>(a, R, packed, s);
  HALP_CASE(1, 1) HALP_CASE(2, 1) HALP_CASE(4, 1) HALP_CASE(8, 1)
  HALP_CASE(1, 2) HALP_CASE(2, 2) HALP_CASE(4, 2) HALP_CASE(8, 2)
  HALP_CASE(1, 4) HALP_CASE(2, 4) HALP_CASE(4, 4) HALP_CASE(8, 4)
  HALP_CASE(4, 8) HALP_CASE(8, 8) HALP_CASE(4, 16) HALP_CASE(8, 16)
#undef HALP_CASE
  return HALP_ERR_UNSUPPORTED;
}

}  // namespace innerreg
}  // namespace halp
