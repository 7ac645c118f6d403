// Inner loop of Algorithm 4 (LM-HALP), register-resident form for few chains:
// one sampled row per step (B = 1), one class, NW "chain" waves that carry z
// plus NW "helper" waves, one beside each chain wave on the same SIMD.
//
// With one chain per CU a step is bound by its dependent chain
//   dot -> DPP fold -> LDS word per wave + barrier -> fp64 scalar path -> update,
// and every other instruction a chain wave issues lengthens it.  Whatever does not
// depend on z is therefore made by the helper waves, two steps ahead, and handed
// over through LDS as one record per lane and step:
//   xe[k]  the row's values at the lane's coordinates, sign-extended
//   hr[k]  the rounding term of the update, -h~ + r at 8 bits, r - (h~ mod 2^16) at 16
// A helper draws the Philox block of its strips (spread over the eight steps before
// the block's window), requests row fragments 16 steps before they are turned into a
// record, and its first wave also refills the 256-step batches of step-indexed draws
// (sample indices, rounding draws of gamma and of the L2 term, margins and labels of
// the sampled rows).  A chain wave is left with the chain itself, one LDS read of the
// next record and the count of clamped coordinates.  The per-step barrier that the
// chain waves need anyway orders every hand-over: helper iteration j writes the record
// of step j + 2 before barrier j, chain waves read the record of step j + 1 after it,
// and a ring of four records is never overwritten while it can still be read.
//
// Results are those of inner_reg_kernel bit for bit; this header holds the kernel
// template, inner_reg_helped_b8.hip / _b16.hip instantiate it.
#pragma once

#include "inner_reg_impl.hpp"

namespace halp {
namespace innerhelp {

using innerreg::kBatch;
using innerreg::kLossSquaredWithMargins;
using innerreg::kWin;
using innerreg::logistic_dl;
using innerreg::mad24;

constexpr int kRing = 4;    // records in flight per lane
constexpr int kAhead = 16;  // steps between a row request and the record made from it

template <int BITS, int LOSS, int UPL, int NWT>
__global__ __launch_bounds__(128 * NWT) void inner_reg_helped_kernel(InArgs a) {
  using XT = typename std::conditional<BITS == 8, int8_t, int16_t>::type;
  using HT = typename std::conditional<BITS == 8, int16_t, int32_t>::type;
  using AccT = typename std::conditional<BITS == 8, int, long long>::type;
  constexpr int CT = 16 / BITS;       // coordinates per strip
  constexpr int CPL = UPL * CT;       // coordinates per lane
  constexpr int NDW = (UPL + 1) / 2;  // dwords of row data per lane and step
  constexpr int QMAX = (1 << (BITS - 1)) - 1, QMIN = -(1 << (BITS - 1));
  constexpr int kMask = 2 * kBatch - 1;
  constexpr uint32_t kFieldMask = BITS == 8 ? 0xFFu : 0xFFFFu;
  typedef int RecT __attribute__((ext_vector_type(2 * CPL)));
  const int chain = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool helper = wave >= NWT;
  const int cw = helper ? wave - NWT : wave;  // the chain wave whose strips this wave works on
  const int d = a.d;
  const int U = (d + CT - 1) / CT;
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
  __shared__ __attribute__((aligned(16))) float s_phi[2 * kBatch];
  __shared__ __attribute__((aligned(16))) float s_y[2 * kBatch];
  // logistic loss: l'(phi_i) of the sampled rows, evaluated four per lane when a batch is drawn
  __shared__ __attribute__((aligned(16))) double s_dl0[LOSS == HALP_LOSS_LOGISTIC ? 2 * kBatch : 2];
  __shared__ __attribute__((aligned(16))) AccT s_part[2][16];
  __shared__ unsigned long long s_cnt[3];
  __shared__ AccT s_dump[64 * NWT];  // where lanes 0..62 of a chain wave put their partial folds
  __shared__ __attribute__((aligned(16))) RecT s_rec[kRing][64 * NWT];

  const double delta_m = sc[0], inv_s = sc[5];
  const double dscale = __dmul_rn(a.delta_d, delta_m);
  const double aB = a.hyper[2 * chain];  // B = 1: alpha / 1
  const bool use_reg = a.lambda > 0;
  constexpr bool logistic = LOSS == HALP_LOSS_LOGISTIC;
  constexpr bool need_phi = LOSS != HALP_LOSS_SQUARED;
  const bool lp = a.lp != 0;
  const double al = __dmul_rn(aB, a.lambda);

  const int ln = cw * 64 + lane;  // the lane's place among the chain's lanes
  const int s0 = ln * UPL;        // first strip of the lane
  const int j0c = s0 * CT;        // first coordinate
  const bool lane_ok = s0 < U;

  // draws that depend on the step number only, 256 steps per batch (made by one wave)
  auto fill_batch = [&](int64_t bb) {
    const int half = (int)(bb & 1) * kBatch;
    const uint64_t blk = (uint64_t)bb * 64 + (uint64_t)lane;
    const U4 ri = stream_block(seed, kIdx, a.epoch, blk);
    const U4 rg = stream_block(seed, kGamma, a.epoch, blk);
    int4 iv;
    iv.x = (int)__umulhi(ri.x, N); iv.y = (int)__umulhi(ri.y, N);
    iv.z = (int)__umulhi(ri.z, N); iv.w = (int)__umulhi(ri.w, N);
    *reinterpret_cast<int4*>(&s_idx[half + 4 * lane]) = iv;
    if (need_phi) {
      float4 pv;
      pv.x = phi[iv.x]; pv.y = phi[iv.y]; pv.z = phi[iv.z]; pv.w = phi[iv.w];
      *reinterpret_cast<float4*>(&s_phi[half + 4 * lane]) = pv;
    }
    if (logistic) {
      float4 yv;
      yv.x = y[iv.x]; yv.y = y[iv.y]; yv.z = y[iv.z]; yv.w = y[iv.w];
      *reinterpret_cast<float4*>(&s_y[half + 4 * lane]) = yv;
      const float4 pw = *reinterpret_cast<const float4*>(&s_phi[half + 4 * lane]);
      s_dl0[half + 4 * lane + 0] = logistic_dl((double)pw.x, (double)yv.x);
      s_dl0[half + 4 * lane + 1] = logistic_dl((double)pw.y, (double)yv.y);
      s_dl0[half + 4 * lane + 2] = logistic_dl((double)pw.z, (double)yv.z);
      s_dl0[half + 4 * lane + 3] = logistic_dl((double)pw.w, (double)yv.w);
    }
    s_rho[half + 4 * lane + 0] = __dmul_rn((double)rg.x, 0x1p-32);
    s_rho[half + 4 * lane + 1] = __dmul_rn((double)rg.y, 0x1p-32);
    s_rho[half + 4 * lane + 2] = __dmul_rn((double)rg.z, 0x1p-32);
    s_rho[half + 4 * lane + 3] = __dmul_rn((double)rg.w, 0x1p-32);
    if (use_reg) {
      const U4 rr = stream_block(seed, kReg, a.epoch, blk);
      const double two_b = (double)(1 << BITS);
      int4 cv;
      cv.x = (int)quantize_real(al, two_b, rr.x, 0.0, (double)QMAX, nullptr);
      cv.y = (int)quantize_real(al, two_b, rr.y, 0.0, (double)QMAX, nullptr);
      cv.z = (int)quantize_real(al, two_b, rr.z, 0.0, (double)QMAX, nullptr);
      cv.w = (int)quantize_real(al, two_b, rr.w, 0.0, (double)QMAX, nullptr);
      *reinterpret_cast<int4*>(&s_creg[half + 4 * lane]) = cv;
    }
  };
  if (tid < 3) s_cnt[tid] = 0;
  if (tid < 32) (&s_part[0][0])[tid] = 0;
  if (wave == NWT) {
    fill_batch(0);
    fill_batch(1);
  }
  __syncthreads();

  if (helper) {
    // =========================== helper wave ===========================
    int hv[CPL];          // -h~ when b = 8; h~ itself when b = 16
    uint32_t xmask[NDW];  // bytes of a fragment that are coordinates < d
#pragma unroll
    for (int k = 0; k < NDW; ++k) xmask[k] = 0;
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
      const int j = j0c + k;
      const bool ok = j < d;
      hv[k] = ok ? (BITS == 8 ? -(int)hg[j] : (int)hg[j]) : 0;
      if (ok) xmask[(k * BITS) / 32] |= kFieldMask << ((k * BITS) % 32);
    }
    // byte offset of the lane's fragment inside a row; a 2-byte fragment is fetched as the
    // aligned dword around it and shifted into place.  Lanes past the end of the row re-read
    // its first bytes and mask them away, so loads never diverge.
    const int lane_off = lane_ok ? (UPL == 1 ? (s0 * 2) & ~3 : s0 * 2) : 0;
    const int half_sh = (UPL == 1 && lane_ok) ? ((s0 * 2) & 2) * 8 : 0;
    const int64_t last = T > 0 ? T - 1 : 0;
    uint32_t fr[kAhead][NDW];  // row fragments in flight, slot r % 16 for the record of step r
    // the sample index of step r, read from LDS one iteration before it is used
    auto index_of = [&](int64_t r) -> int {
      const int64_t rc = r < last ? r : last;  // past the end: any valid row, never used
      return s_idx[(int)(rc & kMask)];
    };
    auto request = [&](uint32_t (&dst)[NDW], int iv) {
      const int i = __builtin_amdgcn_readfirstlane(iv);
      const unsigned char* rowp = Xq + (int64_t)i * row_bytes;  // uniform
      if (UPL <= 2) {
        dst[0] = *reinterpret_cast<const uint32_t*>(rowp + (uint32_t)lane_off);
      } else {
        const uint2 v = *reinterpret_cast<const uint2*>(rowp + (uint32_t)lane_off);
        dst[0] = v.x;
        dst[NDW > 1 ? 1 : 0] = v.y;
      }
    };
    U4 zr[UPL], zn[UPL];  // rounding blocks of the window being served, and of the next one
    auto philox_rounds = [&](int r0, int r1, uint32_t blkno) {
#pragma unroll
      for (int r = r0; r < r1; ++r) {
        const uint32_t k0 = (uint32_t)seed + (uint32_t)r * 0x9E3779B9u;
        const uint32_t k1 = (uint32_t)(seed >> 32) + (uint32_t)r * 0xBB67AE85u;
#pragma unroll
        for (int u = 0; u < UPL; ++u) {
          const U4 c = r == 0 ? U4{(uint32_t)(s0 + u), blkno, a.epoch, (uint32_t)kZround} : zn[u];
          const uint64_t p0 = (uint64_t)0xD2511F53u * c.x;
          const uint64_t p1 = (uint64_t)0xCD9E8D57u * c.z;
          zn[u] = U4{(uint32_t)(p1 >> 32) ^ c.y ^ k0, (uint32_t)p1, (uint32_t)(p0 >> 32) ^ c.w ^ k1,
                     (uint32_t)p0};
        }
      }
    };
    // the record of a step: `frag` is its row fragment, sn its place in its window
    auto make_record = [&](const uint32_t (&frag)[NDW], int sn, int ring) {
      RecT rec;
#pragma unroll
      for (int k = 0; k < CPL; ++k) {
        const uint32_t fv = frag[(k * BITS) / 32];
        const uint32_t xv = (UPL == 1 ? fv >> half_sh : fv) & xmask[(k * BITS) / 32];
        const int sh = (k * BITS) % 32;
        rec[k] = BITS == 8 ? (int)(int8_t)(xv >> sh) : (int)(int16_t)(xv >> sh);
        const uint32_t word = pick(zr[k / CT], (uint32_t)(sn >> 1));
        const int re = (int)((word >> (16 * (sn & 1) + (k % CT) * BITS)) & kFieldMask);
        rec[CPL + k] = BITS == 8 ? hv[k] + re : re - (hv[k] & 0xFFFF);
      }
      s_rec[ring][ln] = rec;
    };
    // one helper iteration: what has to be in place before barrier j.  The record goes first,
    // so that its LDS store is under way while the rest is issued and the wave reaches the
    // barrier before the chain waves do.
    int nidx = 0;  // sample index of the row requested next
    auto iteration = [&](int64_t j, auto s_tag) {
      constexpr int s = decltype(s_tag)::value;  // j % 16
      constexpr int p = (s + 2) & 7;             // place of step j + 2 in its window
      const int64_t r = j + 2;
      if (p == 0) {
#pragma unroll
        for (int u = 0; u < UPL; ++u) zr[u] = zn[u];
      }
      make_record(fr[(s + 2) & 15], p, (s + 2) & 3);
      request(fr[(s + 2) & 15], nidx);
      nidx = index_of(r + 1 + kAhead);
      // ten rounds of the next window's blocks over the eight steps of this one
      philox_rounds(p == 0 ? 0 : (p < 5 ? p + 1 : p + 2), p < 4 ? p + 2 : (p == 4 ? 7 : p + 3),
                    (uint32_t)(r >> 3) + 1u);
      if (s == 0 && wave == NWT && (j & (kBatch - 1)) == 0 && j > 0) fill_batch(j / kBatch + 1);
      __syncthreads();
    };

#pragma unroll
    for (int r = 0; r < kAhead; ++r) request(fr[r], index_of(r));
#pragma unroll
    for (int u = 0; u < UPL; ++u) zr[u] = zround_block(seed, a.epoch, (uint32_t)(s0 + u), 0u);
    philox_rounds(0, 3, 1u);  // as far as the places 0 and 1 of a window bring the next block
    make_record(fr[0], 0, 0);
    request(fr[0], index_of(kAhead));
    make_record(fr[1], 1, 1);
    request(fr[1], index_of(kAhead + 1));
    nidx = index_of(kAhead + 2);
    __syncthreads();

    int64_t j = 0;
    for (; j + 16 <= T; j += 16) {
      iteration(j + 0, std::integral_constant<int, 0>{});
      iteration(j + 1, std::integral_constant<int, 1>{});
      iteration(j + 2, std::integral_constant<int, 2>{});
      iteration(j + 3, std::integral_constant<int, 3>{});
      iteration(j + 4, std::integral_constant<int, 4>{});
      iteration(j + 5, std::integral_constant<int, 5>{});
      iteration(j + 6, std::integral_constant<int, 6>{});
      iteration(j + 7, std::integral_constant<int, 7>{});
      iteration(j + 8, std::integral_constant<int, 8>{});
      iteration(j + 9, std::integral_constant<int, 9>{});
      iteration(j + 10, std::integral_constant<int, 10>{});
      iteration(j + 11, std::integral_constant<int, 11>{});
      iteration(j + 12, std::integral_constant<int, 12>{});
      iteration(j + 13, std::integral_constant<int, 13>{});
      iteration(j + 14, std::integral_constant<int, 14>{});
      iteration(j + 15, std::integral_constant<int, 15>{});
    }
#define HALP_TAIL(S_) \
  if (j + S_ < T) iteration(j + S_, std::integral_constant<int, S_>{});
    HALP_TAIL(0) HALP_TAIL(1) HALP_TAIL(2) HALP_TAIL(3) HALP_TAIL(4) HALP_TAIL(5) HALP_TAIL(6)
    HALP_TAIL(7) HALP_TAIL(8) HALP_TAIL(9) HALP_TAIL(10) HALP_TAIL(11) HALP_TAIL(12) HALP_TAIL(13)
    HALP_TAIL(14)
#undef HALP_TAIL
    __syncthreads();  // the chain waves' counters
    return;
  }

  // ============================= chain wave =============================
  using LdsAcc = __attribute__((address_space(3))) AccT;
  LdsAcc* const slot0 = (LdsAcc*)((lane != 63) ? &s_dump[tid] : &s_part[0][wave]);
  LdsAcc* const slot1 = (LdsAcc*)((lane != 63) ? &s_dump[tid] : &s_part[1][wave]);
  int z[CPL];
  int hh[CPL];  // 16 bits: the high half of h~, which the record's rounding term leaves out
#pragma unroll
  for (int k = 0; k < CPL; ++k) {
    const int j = j0c + k;
    const bool ok = j < d;
    z[k] = ok ? (int)zg[j] : 0;
    hh[k] = (ok && BITS == 16) ? ((int)hg[j] >> 16) : 0;
  }
  unsigned int n_zclamp = 0, n_gclamp = 0, n_reg = 0;
  int zu_p[CPL];  // unclamped values of the step before: clamps are counted one step late,
  int nf_p = 0, ng_p = 0;  // while the wave waits for its LDS store
#pragma unroll
  for (int k = 0; k < CPL; ++k) zu_p[k] = z[k];
  auto count_pending = [&]() {
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
      n_zclamp += (zu_p[k] != z[k]) ? 1u : 0u;
      zu_p[k] = z[k];
    }
    n_gclamp += (nf_p != ng_p) ? 1u : 0u;
    nf_p = ng_p;
  };
  __syncthreads();  // the records of steps 0 and 1 are in place
  RecT nxt = s_rec[0][ln];
  __builtin_amdgcn_s_setprio(3);  // a chain wave that can issue goes before the helper on its SIMD

  // One window of 8 steps from t0 (a multiple of 8).  FULL: all 8 steps exist.  REGW: some
  // step of the window has c_lambda != 0.
  auto window = [&](int64_t t0, auto full_tag, auto reg_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    constexpr bool REGW = decltype(reg_tag)::value;
    const int base = (int)(t0 & kMask);
    double rho[kWin];
    float phi8[kWin], y8[kWin];
    double dl08[kWin];
    int creg[kWin];
#pragma unroll
    for (int s = 0; s < kWin; ++s) {
      dl08[s] = 0.0;
      phi8[s] = y8[s] = 0.f;
      creg[s] = 0;
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
    if (REGW) {
      const int4 c0 = *reinterpret_cast<const int4*>(&s_creg[base]);
      const int4 c1 = *reinterpret_cast<const int4*>(&s_creg[base + 4]);
      creg[0] = c0.x; creg[1] = c0.y; creg[2] = c0.z; creg[3] = c0.w;
      creg[4] = c1.x; creg[5] = c1.y; creg[6] = c1.z; creg[7] = c1.w;
    }
#pragma unroll
    for (int s = 0; s < kWin; s += 2) {
      const double2 r2 = *reinterpret_cast<const double2*>(&s_rho[base + s]);
      rho[s] = r2.x;
      rho[s + 1] = r2.y;
    }
#pragma unroll
    for (int s = 0; s < kWin; ++s) {
      if (FULL || t0 + s < T) {
        int xe[CPL], hr[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
          xe[k] = nxt[k];
          hr[k] = nxt[CPL + k];
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- dot, fold, the wave's sum into its LDS word
        int part = 0, part_hi = 0;
        AccT D;
        if (BITS == 8) {
#pragma unroll
          for (int k = 0; k < CPL; ++k) part = mad24(xe[k], z[k], part);
          D = (AccT)wave_fold_i32(part);
        } else {
          // a product of two 16-bit factors is cut into its low 16 bits and the rest, and the
          // two kinds are summed apart: two plain folds give the exact 64-bit dot product
          if (CPL == 1) {
            const int pr = mad24(xe[0], z[0], 0);
            part = pr & 0xFFFF;
            part_hi = pr >> 16;
          } else {
#pragma unroll
            for (int k = 0; k + 1 < CPL; k += 2) {
              const int pr = mad24(xe[k], z[k], mad24(xe[k + 1], z[k + 1], 0));
              part += pr & 0xFFFF;
              part_hi += pr >> 16;
            }
          }
          const int lo = wave_fold_i32(part);
          const int hi = wave_fold_i32(part_hi);
          D = (AccT)(((long long)hi << 16) + (long long)lo);
        }
        *((s & 1) ? slot1 : slot0) = D;
        __builtin_amdgcn_sched_barrier(0);
        count_pending();
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        AccT q[NWT];
#pragma unroll
        for (int w2 = 0; w2 < NWT; ++w2) q[w2] = s_part[s & 1][w2];
        nxt = s_rec[(s + 1) & (kRing - 1)][ln];  // t0 is a multiple of 8: (t + 1) % 4 = (s + 1) % 4
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int w = NWT / 2; w >= 1; w /= 2) {
#pragma unroll
          for (int k = 0; k < w; ++k) q[k] += q[k + w];
        }
        D = q[0];
        // beta = alpha (l'(phi_i + x_i^T z) - l'(phi_i)), gamma = Q_(delta_s, b)(beta)
        const double delta = __dmul_rn(dscale, (double)D);
        double diff = delta;
        if (logistic) {
          const double a0 = (double)phi8[s], yi = (double)y8[s];
          const double a1 = lp ? delta : __dadd_rn(a0, delta);
          diff = __dadd_rn(logistic_dl(a1, yi), -dl08[s]);  // l'(phi_i) comes with the batch
        } else if (need_phi) {
          diff = __dadd_rn(delta, -(double)phi8[s]);
        }
        const double beta = __dmul_rn(aB, diff);
        const double f = floor(__dadd_rn(__dmul_rn(beta, inv_s), rho[s]));
        int nf;
        asm("v_cvt_i32_f64 %0, -%1" : "=v"(nf) : "v"(f));
        const int ng = min(max(nf, -QMAX), -QMIN);
        nf_p = nf;
        ng_p = ng;
        int cl = 0;
        if (REGW) {
          cl = __builtin_amdgcn_readfirstlane(creg[s]);
          n_reg += cl != 0 ? 1u : 0u;
        }
        // u = z - gamma x - h~ (- c_lambda z), z = Q_(delta_m, b)(u)
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
          int v = mad24(ng, xe[k], hr[k]);
          if (REGW) v = mad24(-cl, z[k], v);
          const int zu = BITS == 8 ? z[k] + (v >> 8) : z[k] + (v >> 16) - hh[k];
          zu_p[k] = zu;
          z[k] = min(max(zu, QMIN), QMAX);
        }
      }
    }
  };
  // true if some step of the window at tt has an L2 draw (rare: alpha lambda 2^b is tiny)
  auto any_creg = [&](int64_t tt) -> bool {
    if (!use_reg) return false;
    const int base = (int)(tt & kMask);
    const int4 c0 = *reinterpret_cast<const int4*>(&s_creg[base]);
    const int4 c1 = *reinterpret_cast<const int4*>(&s_creg[base + 4]);
    const int any = c0.x | c0.y | c0.z | c0.w | c1.x | c1.y | c1.z | c1.w;
    return __builtin_amdgcn_readfirstlane(any) != 0;
  };
  int64_t t0 = 0;
  for (; t0 + kWin <= T; t0 += kWin) {
    if (any_creg(t0)) window(t0, std::true_type{}, std::true_type{});
    else window(t0, std::true_type{}, std::false_type{});
  }
  if (t0 < T) {
    if (use_reg) window(t0, std::false_type{}, std::true_type{});
    else window(t0, std::false_type{}, std::false_type{});
  }
  count_pending();

  // ---- w~ <- w~ + delta_m z (option I); hand z out
#pragma unroll
  for (int k = 0; k < CPL; ++k) {
    const int j = j0c + k;
    if (j < d) {
      zg[j] = (XT)z[k];
      const double step = __dmul_rn(delta_m, (double)z[k]);
      wg[j] = lp ? (float)step : (float)__dadd_rn((double)wg[j], step);  // Alg. 2: w~ = delta w
    }
  }
  if (n_zclamp) atomicAdd(&s_cnt[0], (unsigned long long)n_zclamp);
  if (tid == 0) {
    s_cnt[1] = n_gclamp;  // gamma is uniform over the workgroup: count it once
    s_cnt[2] = n_reg;
  }
  __syncthreads();
  if (tid < 4) cnt_out[tid] = tid < 3 ? s_cnt[tid] : 0ull;
}

template <int BITS, int UPL, int NWT>
int launch_one(const InArgs& a, int R, hipStream_t s) {
  const dim3 grid(R), block(128 * NWT);
  if (a.loss == HALP_LOSS_SQUARED && a.lp)
    hipLaunchKernelGGL((inner_reg_helped_kernel<BITS, kLossSquaredWithMargins, UPL, NWT>), grid, block, 0, s, a);
  else if (a.loss == HALP_LOSS_SQUARED)
    hipLaunchKernelGGL((inner_reg_helped_kernel<BITS, HALP_LOSS_SQUARED, UPL, NWT>), grid, block, 0, s, a);
  else
    hipLaunchKernelGGL((inner_reg_helped_kernel<BITS, HALP_LOSS_LOGISTIC, UPL, NWT>), grid, block, 0, s, a);
  return hip_ok(hipGetLastError());
}

// every (strips per lane, chain waves) pair this form is built for
template <int BITS>
int launch_bits(const InArgs& a, int nw, int upl, int R, hipStream_t s) {
  if (upl == 1 && nw == 2) return launch_one<BITS, 1, 2>(a, R, s);
  if (upl == 2 && nw == 2) return launch_one<BITS, 2, 2>(a, R, s);
  if (upl == 1 && nw == 4) return launch_one<BITS, 1, 4>(a, R, s);
  if (upl == 2 && nw == 4) return launch_one<BITS, 2, 4>(a, R, s);
  return HALP_ERR_UNSUPPORTED;
}

}  // namespace innerhelp
}  // namespace halp
