// Inner loop of Algorithm 4 (LM-HALP), register-resident form for one chain per CU at
// 8 bits: one sampled row per step (B = 1), one class, ONE "chain" wave that carries
// the whole of z, and helper waves on the other SIMDs of the CU.
//
// With a chain to itself a CU is bound by the step's dependent chain.  Several waves per
// chain shorten the update but pay an LDS word and a barrier per step to add their dot
// products up; one wave with all the coordinates pays nothing across waves, and at 8 bits
// its arithmetic packs two coordinates into a register:
//   dot     one packed 16-bit dot per strip (two coordinates), DPP fold, sum read from lane 63
//   scalar  beta and gamma = Q_(delta_s,b)(beta) in fp64, wave-uniform
//   update  per strip: floor((-gamma x + r + hl) / 256) + hh + z on packed halves, clamp
//           (-h~ = 256 hh + hl, 0 <= hl < 256; |gamma x| <= 2^14 and r + hl < 512, so
//           every intermediate fits 16 bits)
// Whatever does not depend on z is made by the helpers, a window of 8 steps ahead, and
// handed over through LDS as one record per lane and step: per strip the sign-extended
// pair of row values and the pair of rounding bytes with hl added.  A helper serves one or
// two of the strips of every lane: it draws their Philox blocks, requests the row fragments
// three windows ahead and writes its dwords of the records.  Where -h~ / 256 is small in
// every coordinate the records carry r - h~ whole (it fits 16 bits beside -gamma x) and the
// chain wave adds no hh.  A service wave refills the 256-step batches of step-indexed draws
// (sample indices, rounding draws of gamma and of the L2 term, margins and labels of the
// sampled rows) and counts the clamped coordinates: the chain wave stores the unclamped strips
// of a step in LDS instead of comparing them with the clamped ones, and the service wave
// counts the halves outside [-128, 127] a window later.  One barrier per window orders every
// hand-over: in period w the chain wave consumes window w from one half of the record ring
// and fills one half of the log, while the helpers fill the other half of the ring with
// window w + 1 and the service wave reads the other half of the log (window w - 1).
//
// The chain wave is wave 0; the helpers and the service wave are placed on the other three
// SIMDs (waves w and w + 4 of a workgroup share a SIMD: wave 4 only keeps the barriers).
//
// Results are those of inner_reg_kernel bit for bit; this header holds the kernel template,
// inner_reg_lone_b8.hip instantiates it.
#pragma once

#include "inner_reg_impl.hpp"

namespace halp {
namespace innerlone {

using innerreg::kBatch;
using innerreg::kLossSquaredWithMargins;
using innerreg::kWin;
using innerreg::logistic_dl;
using innerreg::mad24;
using innerreg::short2r;

typedef int int4r __attribute__((ext_vector_type(4)));

template <int LOSS>
constexpr bool logistic_c = LOSS == HALP_LOSS_LOGISTIC;

// waves of a workgroup: chain, helpers, the service wave, and wave 4 kept idle when there is one
constexpr int waves_of(int upl) { return upl == 2 ? 4 : (upl == 4 ? 7 : 8); }

// PAIR: built for two workgroups per CU (more chains than CUs): their 14 waves need four wave
// slots on two of the SIMDs, i.e. at most 128 registers per lane, which costs the single
// workgroup of a CU a few spills (2.59 against 2.50 ms per 16384 steps at 4 strips per lane).
template <int LOSS, int UPL, bool PAIR>
__global__ __launch_bounds__(64 * waves_of(UPL), PAIR ? 4 : 2) void inner_reg_lone_kernel(InArgs a) {
  static_assert(UPL == 2 || UPL == 4 || UPL == 8, "two, four or eight strips per lane");
  constexpr int BITS = 8;
  constexpr int NQ = UPL / 2;           // 16-byte quads of a record: UPL value pairs, then UPL rounding pairs
  constexpr int QMAX = 127, QMIN = -128;
  constexpr int kMask = 2 * kBatch - 1;
  const int chain = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Roles by wave.  Waves w and w + 4 share a SIMD and wave 0 is the chain wave, so wave 4 only
  // keeps the barriers.  2 strips per lane: waves 1, 2 serve one strip each, wave 3 is the
  // service wave.  4: waves 1, 2, 3, 5 one strip each, service wave 6.  8: waves 1, 2, 3 two
  // strips each, waves 5, 6 one each (three strips on two SIMDs, two and the service wave 7 on
  // the third).
  int first_strip = -1, strips_here = 0;
  bool is_service = false;
  if (UPL == 2) {
    if (wave == 1 || wave == 2) { first_strip = wave - 1; strips_here = 1; }
    is_service = wave == 3;
  } else if (UPL == 4) {
    if (wave >= 1 && wave <= 3) { first_strip = wave - 1; strips_here = 1; }
    if (wave == 5) { first_strip = 3; strips_here = 1; }
    is_service = wave == 6;
  } else {
    if (wave >= 1 && wave <= 3) { first_strip = 2 * (wave - 1); strips_here = 2; }
    if (wave == 5 || wave == 6) { first_strip = wave + 1; strips_here = 1; }
    is_service = wave == 7;
  }
  const int d = a.d;
  const int U = (d + 1) / 2;  // strips in a row
  const uint32_t N = (uint32_t)a.N;
  const int64_t row_bytes = a.ldxq;
  const unsigned char* __restrict__ Xq =
      reinterpret_cast<const unsigned char*>(a.Xq) + (int64_t)chain * a.xq_chain_stride;
  const float* __restrict__ phi = a.phi + (int64_t)chain * a.N;
  const float* __restrict__ y =
      reinterpret_cast<const float*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const int16_t* __restrict__ hg = reinterpret_cast<const int16_t*>(a.h) + (int64_t)chain * d;
  int8_t* __restrict__ zg = reinterpret_cast<int8_t*>(a.z) + (int64_t)chain * d;
  float* __restrict__ wg = a.w + (int64_t)chain * d;
  const double* sc = a.scales + (int64_t)chain * 8;
  uint64_t* cnt_out = a.counters + (int64_t)chain * 4;
  const uint64_t seed = a.seed + (uint64_t)chain;
  const int64_t T = epoch_steps(seed, a.epoch, a.T, a.option2);
  const int64_t nwin = (T + kWin - 1) / kWin;

  if (sc[7] != 0.0) {  // converged or unusable gradient: the epoch is a no-op
    if (tid < 4) cnt_out[tid] = 0;
    return;
  }

  __shared__ __attribute__((aligned(16))) int s_idx[2 * kBatch];
  __shared__ __attribute__((aligned(16))) double s_rho[2 * kBatch];
  __shared__ __attribute__((aligned(16))) int s_creg[2 * kBatch];
  __shared__ __attribute__((aligned(16))) float s_phi[2 * kBatch];
  __shared__ __attribute__((aligned(16))) float s_y[2 * kBatch];
  // logistic loss: l'(phi_i) of the sampled rows, which no step has to evaluate itself
  __shared__ __attribute__((aligned(16))) double s_dl0[logistic_c<LOSS> ? 2 * kBatch : 2];
  __shared__ unsigned long long s_cnt[4];
  __shared__ int s_fold;  // 1: the whole of -h~ rides in the records (set by the chain wave before the first barrier)
  // records: [half of the ring][step of the window][quad][lane], 16 bytes each
  extern __shared__ __attribute__((aligned(16))) int4r s_rec[];
  auto rec_at = [&](int half, int s, int q) -> int4r* { return s_rec + ((half * kWin + s) * NQ + q) * 64 + lane; };
  // behind it, what the chain wave hands back: the unclamped strips of every step, [half][step][quad][lane]
  constexpr int NQV = UPL >= 4 ? UPL / 4 : 1;
  int4r* const s_vlog = s_rec + 2 * kWin * NQ * 64;
  auto vlog_at = [&](int half, int s, int q) -> int4r* { return s_vlog + ((half * kWin + s) * NQV + q) * 64 + lane; };

  const double delta_m = sc[0], inv_s = sc[5];
  const double dscale = __dmul_rn(a.delta_d, delta_m);
  const double aB = a.hyper[2 * chain];  // B = 1: alpha / 1
  const bool use_reg = a.lambda > 0;
  constexpr bool logistic = LOSS == HALP_LOSS_LOGISTIC;
  constexpr bool need_phi = LOSS != HALP_LOSS_SQUARED;
  const bool lp = a.lp != 0;
  const double al = __dmul_rn(aB, a.lambda);

  const int s0 = lane * UPL;  // first strip of the lane
  const int j0 = s0 * 2;      // first coordinate

  if (tid < 4) s_cnt[tid] = 0;

  if (is_service) {
    // ============================ service wave ============================
    // draws that depend on the step number only, 256 steps per batch
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
        const float4 pv = *reinterpret_cast<const float4*>(&s_phi[half + 4 * lane]);
        s_dl0[half + 4 * lane + 0] = logistic_dl((double)pv.x, (double)yv.x);
        s_dl0[half + 4 * lane + 1] = logistic_dl((double)pv.y, (double)yv.y);
        s_dl0[half + 4 * lane + 2] = logistic_dl((double)pv.z, (double)yv.z);
        s_dl0[half + 4 * lane + 3] = logistic_dl((double)pv.w, (double)yv.w);
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
    // Clamped coordinates: the chain wave stores the unclamped strips of a step (one LDS store)
    // instead of comparing them with the clamped ones; they are counted here, a window later.
    // A half outside [-128, 127] has a bit set above its low byte once 128 is added.
    unsigned int n_lane = 0;  // this lane's count
    auto count_window = [&](int64_t w) {
      const int half = (int)(w & 1);
      const int64_t left = T - w * kWin;
      const short2r k128 = short2r{128, 128};
      short2r acc = short2r{0, 0};  // at most 8 UPL per half and window
#pragma unroll
      for (int s = 0; s < kWin; ++s) {
        if (s < left) {
#pragma unroll
          for (int q = 0; q < NQV; ++q) {
            const int4r v4 = *vlog_at(half, s, q);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              if (4 * q + k < UPL) {
                const int vk = v4[k];
                typedef unsigned short ushort2r __attribute__((ext_vector_type(2)));
                const ushort2r t = __builtin_bit_cast(ushort2r, __builtin_bit_cast(short2r, vk) + k128) >> (ushort2r)(8);
                acc += __builtin_bit_cast(short2r, __builtin_elementwise_min(t, (ushort2r)(1)));
              }
            }
          }
        }
      }
      n_lane += (unsigned int)(unsigned short)acc[0] + (unsigned int)(unsigned short)acc[1];
    };
    fill_batch(0);
    fill_batch(1);
    __syncthreads();  // P0: the first two batches are in place
    __syncthreads();  // P1: the records of window 0 are in place
    for (int64_t w = 0; w < nwin; ++w) {
      // window w = 32 m: every reader has left batch m - 1, whose half takes batch m + 1
      if ((w & (kBatch / kWin - 1)) == 0 && w > 0) fill_batch(w / (kBatch / kWin) + 1);
      if (w > 0) count_window(w - 1);
      __syncthreads();
    }
    if (nwin > 0) count_window(nwin - 1);
    const unsigned int total = (unsigned int)wave_sum_i32((int)n_lane);
    if (lane == 0) s_cnt[0] = total;
    __syncthreads();  // the counters
    return;
  }

  if (first_strip >= 0) {
    // ============================ helper wave =============================
    auto helper_body = [&](auto sph_c) {
      constexpr int SPH = decltype(sph_c)::value;  // strips of a lane this wave serves
      const int u0 = first_strip;               // the first of them
      const int g0 = s0 + u0;                   // ... in the row
      const bool frag_ok = g0 < U;              // the fragment starts inside the row
      const uint32_t frag_off = frag_ok ? (uint32_t)(2 * g0) : 0u;  // lanes past the row re-read its first bytes
      short2r hlp[SPH];                         // what a record adds to the rounding bytes: the low byte of
      short2r hfp[SPH];                         // -h~, or the whole of it where every -h~ / 256 is small
      uint32_t xmask = 0;                       // bytes of the fragment that are coordinates < d
#pragma unroll
      for (int i = 0; i < SPH; ++i) {
        int hl[2], hf[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int j = 2 * (g0 + i) + e;
          const bool ok = j < d;
          const int hneg = ok ? -(int)hg[ok ? j : 0] : 0;
          hl[e] = hneg & 0xFF;
          hf[e] = hneg;
          if (ok) xmask |= 0xFFu << (16 * i + 8 * e);
        }
        hlp[i] = short2r{(short)hl[0], (short)hl[1]};
        hfp[i] = short2r{(short)hf[0], (short)hf[1]};
      }
      // The rows of a window: its eight sample indices in two LDS reads (every entry of the
      // index ring is a valid row at any time, so windows past the end of the epoch fetch
      // rows that are never used), then one load per step.
      auto request = [&](uint32_t (&dst)[kWin], int64_t win) {
        const int base = (int)((win * kWin) & kMask);
        const int4 i0 = *reinterpret_cast<const int4*>(&s_idx[base]);
        const int4 i1 = *reinterpret_cast<const int4*>(&s_idx[base + 4]);
        const int iv[kWin] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
#pragma unroll
        for (int s = 0; s < kWin; ++s) {
          const int i = __builtin_amdgcn_readfirstlane(iv[s]);
          const unsigned char* rowp = Xq + (int64_t)i * row_bytes;  // uniform
          if (SPH == 1) dst[s] = (uint32_t) * reinterpret_cast<const uint16_t*>(rowp + frag_off);
          else dst[s] = *reinterpret_cast<const uint32_t*>(rowp + frag_off);
        }
      };
      uint32_t f0[kWin], f1[kWin], f2[kWin];  // row fragments in flight: window v in set v % 3
      U4 zr[SPH], zn[SPH];  // rounding blocks of window 0, and of the window whose records are made next
      auto blocks = [&](U4 (&dst)[SPH], int64_t win) {
#pragma unroll
        for (int i = 0; i < SPH; ++i) dst[i] = zround_block(seed, a.epoch, (uint32_t)(g0 + i), (uint32_t)win);
      };
      // the records of a window into a half of the ring
      auto make_window = [&](const uint32_t (&fr)[kWin], const U4 (&zb)[SPH], int half) {
#pragma unroll
        for (int s = 0; s < kWin; ++s) {
          const uint32_t fv = fr[s] & xmask;
#pragma unroll
          for (int i = 0; i < SPH; ++i) {
            // the strip's two bytes go to the high bytes of the halves and come back down with their signs
            const uint32_t up = __builtin_amdgcn_perm(0u, fv, i ? 0x030C020Cu : 0x010C000Cu);
            const short2r xp = __builtin_bit_cast(short2r, up) >> (short2r)(8);
            const uint32_t word = pick(zb[i], (uint32_t)(s >> 1));
            const uint32_t rp = __builtin_amdgcn_perm(0u, word, (s & 1) ? 0x0C030C02u : 0x0C010C00u);
            const short2r crp = __builtin_bit_cast(short2r, rp) + hlp[i];
            const int u = u0 + i;
            reinterpret_cast<int*>(rec_at(half, s, u / 4))[u % 4] = __builtin_bit_cast(int, xp);
            reinterpret_cast<int*>(rec_at(half, s, (UPL + u) / 4))[(UPL + u) % 4] = __builtin_bit_cast(int, crp);
          }
        }
      };
      __syncthreads();  // P0: the first two batches are in place
      if (s_fold) {
#pragma unroll
        for (int i = 0; i < SPH; ++i) hlp[i] = hfp[i];
      }
      request(f0, 0);
      request(f1, 1);
      request(f2, 2);
      blocks(zr, 0);
      make_window(f0, zr, 0);
      blocks(zn, 1);
      __syncthreads();  // P1: the records of window 0 are in place
      // Period w: the rows of window w + 3 are requested into the set window w left, the records
      // of window w + 1 are made, then the blocks of window w + 2.  Three periods per trip, so that
      // the fragment sets rotate by name.
      // (nothing may be scheduled across the borders of a period: left to itself the compiler
      // masks the fragments of all three sets at the top of the loop, i.e. waits for every load)
      auto period = [&](int64_t w, uint32_t (&freq)[kWin], const uint32_t (&fuse)[kWin]) {
        __builtin_amdgcn_sched_barrier(0);
        request(freq, w + 3);
        __builtin_amdgcn_sched_barrier(0);
        make_window(fuse, zn, (int)((w + 1) & 1));
        blocks(zn, w + 2);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      };
      int64_t w = 0;
      for (; w + 3 <= nwin; w += 3) {
        period(w, f0, f1);
        period(w + 1, f1, f2);
        period(w + 2, f2, f0);
      }
      if (w < nwin) period(w, f0, f1);
      if (w + 1 < nwin) period(w + 1, f1, f2);
      __syncthreads();  // the chain wave's counters
    };
    if (strips_here == 2) helper_body(std::integral_constant<int, 2>{});
    else helper_body(std::integral_constant<int, 1>{});
    return;
  }

  if (wave != 0) {
    // ============================== idle wave ==============================
    __syncthreads();
    __syncthreads();
    for (int64_t w = 0; w < nwin; ++w) __syncthreads();
    __syncthreads();
    return;
  }

  // ============================== chain wave ==============================
  short2r zp[UPL], hhp[UPL];  // z, and the high part of -h~, two coordinates per register
#pragma unroll
  for (int u = 0; u < UPL; ++u) {
    int zv[2], hh[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int j = j0 + 2 * u + e;
      const bool ok = j < d;
      zv[e] = ok ? (int)zg[ok ? j : 0] : 0;
      hh[e] = ok ? (-(int)hg[ok ? j : 0]) >> 8 : 0;
    }
    zp[u] = short2r{(short)zv[0], (short)zv[1]};
    hhp[u] = short2r{(short)hh[0], (short)hh[1]};
  }
  // With -h~ = 256 hh + hl the update adds hh behind the shift.  Where every hh lies in
  // [-64, 62], -gamma x + r - h~ itself fits 16 bits (|gamma x| <= 2^14, 0 <= r < 256): the
  // records then carry r - h~ whole and the chain wave saves the addition of hh, one
  // instruction per strip and step.
  bool hh_small = true;
#pragma unroll
  for (int u = 0; u < UPL; ++u)
#pragma unroll
    for (int e = 0; e < 2; ++e) hh_small = hh_small && (int)hhp[u][e] >= -64 && (int)hhp[u][e] <= 62;
  const bool fold = __ballot(!hh_small) == 0;  // uniform
  if (lane == 0) s_fold = fold ? 1 : 0;
  unsigned int n_zclamp = 0, n_reg = 0;  // uniform over the wave
  unsigned int n_gclamp_v = 0;          // per lane, the same in every lane
  __syncthreads();  // P0
  __syncthreads();  // P1: the records of window 0 are in place
  __builtin_amdgcn_s_setprio(3);

  // step-indexed draws of a window (rounding draws of gamma, margins and labels of its rows),
  // read from the batch ring one window before they are used
  double rho_n[kWin], dl0_n[kWin];
  float phi_n[kWin], y_n[kWin];
#pragma unroll
  for (int s = 0; s < kWin; ++s) {
    phi_n[s] = y_n[s] = 0.f;
    dl0_n[s] = 0.0;
  }
  auto load_draws = [&](int64_t tt) {
    const int base = (int)(tt & kMask);
    if (need_phi) {
      const float4 p0 = *reinterpret_cast<const float4*>(&s_phi[base]);
      const float4 p1 = *reinterpret_cast<const float4*>(&s_phi[base + 4]);
      phi_n[0] = p0.x; phi_n[1] = p0.y; phi_n[2] = p0.z; phi_n[3] = p0.w;
      phi_n[4] = p1.x; phi_n[5] = p1.y; phi_n[6] = p1.z; phi_n[7] = p1.w;
    }
    if (logistic) {
      const float4 y0 = *reinterpret_cast<const float4*>(&s_y[base]);
      const float4 y1 = *reinterpret_cast<const float4*>(&s_y[base + 4]);
      y_n[0] = y0.x; y_n[1] = y0.y; y_n[2] = y0.z; y_n[3] = y0.w;
      y_n[4] = y1.x; y_n[5] = y1.y; y_n[6] = y1.z; y_n[7] = y1.w;
#pragma unroll
      for (int s = 0; s < kWin; s += 2) {
        const double2 d2 = *reinterpret_cast<const double2*>(&s_dl0[base + s]);
        dl0_n[s] = d2.x;
        dl0_n[s + 1] = d2.y;
      }
    }
#pragma unroll
    for (int s = 0; s < kWin; s += 2) {
      const double2 r2 = *reinterpret_cast<const double2*>(&s_rho[base + s]);
      rho_n[s] = r2.x;
      rho_n[s + 1] = r2.y;
    }
  };
  load_draws(0);

  auto window = [&](int64_t t0, auto full_tag, auto reg_tag, auto fold_tag) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full_tag)::value;
    constexpr bool REGW = decltype(reg_tag)::value;  // some step of the window may have c_lambda != 0
    constexpr bool FOLD = decltype(fold_tag)::value;  // the records carry the whole of -h~
    const int base = (int)(t0 & kMask);
    const int half = (int)((t0 >> 3) & 1);
    double rho[kWin], dl08[kWin];
    float phi8[kWin], y8[kWin];
    int creg[kWin];
#pragma unroll
    for (int s = 0; s < kWin; ++s) {
      dl08[s] = dl0_n[s];
      rho[s] = rho_n[s];
      phi8[s] = phi_n[s];
      y8[s] = y_n[s];
      creg[s] = 0;
    }
    if (REGW) {
      const int4 c0 = *reinterpret_cast<const int4*>(&s_creg[base]);
      const int4 c1 = *reinterpret_cast<const int4*>(&s_creg[base + 4]);
      creg[0] = c0.x; creg[1] = c0.y; creg[2] = c0.z; creg[3] = c0.w;
      creg[4] = c1.x; creg[5] = c1.y; creg[6] = c1.z; creg[7] = c1.w;
    }
    int4r rq[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) rq[q] = *rec_at(half, 0, q);
    load_draws(t0 + kWin);  // (any window has its place in the ring, also past the end of the epoch)
#pragma unroll
    for (int s = 0; s < kWin; ++s) {
      if (FULL || t0 + s < T) {
        short2r xp[UPL], crp[UPL];
#pragma unroll
        for (int u = 0; u < UPL; ++u) {
          // (element by value first: a bit cast applied to a vector's element reads element 0)
          const int xv = rq[u / 4][u % 4], cv = rq[(UPL + u) / 4][(UPL + u) % 4];
          xp[u] = __builtin_bit_cast(short2r, xv);
          crp[u] = __builtin_bit_cast(short2r, cv);
        }
        if (s + 1 < kWin) {  // the next step's record, one step ahead
#pragma unroll
          for (int q = 0; q < NQ; ++q) rq[q] = *rec_at(half, s + 1, q);
        }
        // low-precision dot product x_i^T z: one packed dot per strip, two accumulators
        int p0 = 0, p1 = 0;
#pragma unroll
        for (int u = 0; u < UPL; u += 2) {
          p0 = __builtin_amdgcn_sdot2(xp[u], zp[u], p0, false);
          p1 = __builtin_amdgcn_sdot2(xp[u + 1], zp[u + 1], p1, false);
        }
        const int D = wave_sum_i32(p0 + p1);
        // beta = alpha (l'(phi_i + x_i^T z) - l'(phi_i)), gamma = Q_(delta_s, b)(beta)
        const double delta = __dmul_rn(dscale, (double)D);
        double diff = delta;
        if (logistic) {
          const double a0 = (double)phi8[s], yi = (double)y8[s];
          const double a1 = lp ? delta : __dadd_rn(a0, delta);
          diff = __dadd_rn(logistic_dl(a1, yi), -dl08[s]);  // l'(phi_i) comes with the draws
        } else if (need_phi) {
          diff = __dadd_rn(delta, -(double)phi8[s]);
        }
        const double beta = __dmul_rn(aB, diff);
        const double f = floor(__dadd_rn(__dmul_rn(beta, inv_s), rho[s]));
        int nfv;
        asm("v_cvt_i32_f64 %0, -%1" : "=v"(nfv) : "v"(f));
        const int ng = min(max(nfv, -QMAX), -QMIN);
        n_gclamp_v += (nfv != ng) ? 1u : 0u;  // the same in every lane
        int cl = 0;
        if (REGW) {
          cl = __builtin_amdgcn_readfirstlane(creg[s]);
          n_reg += cl != 0 ? 1u : 0u;
        }
        // u = z - gamma x - h~ (- c_lambda z), z = Q_(delta_m, b)(u)
        if (!REGW || cl == 0) {
          // Clamped coordinates are not looked for here (comparing the strips before and after the
          // clamp costs 70 of 410 cycles per step at 4 strips per lane): the unclamped strips go to
          // LDS in one store and the service wave counts a window later.
          const short2r ngp = short2r{(short)ng, (short)ng};
          int4r vq[NQV];
#pragma unroll
          for (int q = 0; q < NQV; ++q) vq[q] = int4r{0, 0, 0, 0};
#pragma unroll
          for (int u = 0; u < UPL; ++u) {
            short2r v = xp[u] * ngp + crp[u];
            if (FOLD) v = (v >> (short2r)(8)) + zp[u];
            else v = (v >> (short2r)(8)) + (hhp[u] + zp[u]);  // the sum in brackets does not wait for gamma
            vq[u / 4][u % 4] = __builtin_bit_cast(int, v);
            zp[u] = __builtin_elementwise_min(__builtin_elementwise_max(v, (short2r)(QMIN)), (short2r)(QMAX));
          }
#pragma unroll
          for (int q = 0; q < NQV; ++q) *vlog_at(half, s, q) = vq[q];
        } else {
          // a step with an L2 draw (rare): 32-bit arithmetic on the unpacked halves,
          // -h~ + r = 256 hh + (hl + r); its clamps are counted here and its log entry is empty
#pragma unroll
          for (int q = 0; q < NQV; ++q) *vlog_at(half, s, q) = int4r{0, 0, 0, 0};
#pragma unroll
          for (int u = 0; u < UPL; ++u) {
            int zn2[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              const int zk = (int)zp[u][e], xk = (int)xp[u][e];
              const int hr = FOLD ? (int)crp[u][e] : ((int)hhp[u][e] << 8) + (int)crp[u][e];
              const int v = mad24(-cl, zk, mad24(ng, xk, hr));
              const int zuk = zk + (v >> 8);
              const int zc = min(max(zuk, QMIN), QMAX);
              n_zclamp += (unsigned int)__builtin_popcountll(__ballot(zuk != zc));
              zn2[e] = zc;
            }
            zp[u] = short2r{(short)zn2[0], (short)zn2[1]};
          }
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
  auto run = [&](auto fold_tag) __attribute__((always_inline)) {
    for (; t0 + kWin <= T; t0 += kWin) {
      if (any_creg(t0)) window(t0, std::true_type{}, std::true_type{}, fold_tag);
      else window(t0, std::true_type{}, std::false_type{}, fold_tag);
      __syncthreads();  // window t0 / 8 is consumed, the records of the next one are in place
    }
    if (t0 < T) {
      if (use_reg) window(t0, std::false_type{}, std::true_type{}, fold_tag);
      else window(t0, std::false_type{}, std::false_type{}, fold_tag);
      __syncthreads();
    }
  };
  if (fold) run(std::true_type{});
  else run(std::false_type{});

  // ---- w~ <- w~ + delta_m z (option I); hand z out
#pragma unroll
  for (int u = 0; u < UPL; ++u)
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int j = j0 + 2 * u + e;
      if (j < d) {
        const int zk = (int)zp[u][e];
        zg[j] = (int8_t)zk;
        const double step = __dmul_rn(delta_m, (double)zk);
        wg[j] = lp ? (float)step : (float)__dadd_rn((double)wg[j], step);  // Alg. 2: w~ = delta w
      }
    }
  if (lane == 0) {
    s_cnt[3] = n_zclamp;  // clamps of the steps with an L2 draw; the service wave puts the others into s_cnt[0]
    s_cnt[1] = n_gclamp_v;
    s_cnt[2] = n_reg;
  }
  __syncthreads();
  if (tid < 4) cnt_out[tid] = tid == 0 ? s_cnt[0] + s_cnt[3] : (tid < 3 ? s_cnt[tid] : 0ull);
}

// the record ring (two windows of 8 steps, 8 UPL bytes per lane and step) and the log of
// unclamped strips behind it (4 UPL bytes, 16 at least)
constexpr size_t ring_bytes(int upl) {
  return (size_t)2 * kWin * (upl / 2) * 64 * 16 + (size_t)2 * kWin * (upl >= 4 ? upl / 4 : 1) * 64 * 16;
}

template <int UPL, bool PAIR>
int launch_one(const InArgs& a, int R, hipStream_t s) {
  const dim3 grid(R), block(64 * waves_of(UPL));
  const size_t smem = ring_bytes(UPL);
#define HALP_LONE(LOSS_)                                                                          \
  do {                                                                                            \
    auto kern = inner_reg_lone_kernel<LOSS_, UPL, PAIR>;                                          \
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                  \
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess) \
      return HALP_ERR_HIP;                                                                        \
    hipLaunchKernelGGL(kern, grid, block, smem, s, a);                                            \
  } while (0)
  if (a.loss == HALP_LOSS_SQUARED && a.lp) HALP_LONE(kLossSquaredWithMargins);
  else if (a.loss == HALP_LOSS_SQUARED) HALP_LONE(HALP_LOSS_SQUARED);
  else HALP_LONE(HALP_LOSS_LOGISTIC);
#undef HALP_LONE
  return hip_ok(hipGetLastError());
}

}  // namespace innerlone
}  // namespace halp
