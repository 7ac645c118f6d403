// Inner loop of Algorithm 4 (LM-HALP) for softmax regression (K classes, one
// sampled row per step), register-resident form with specialised waves.
//
// One workgroup per chain: K / CPW class waves and one service wave (CPW = 1 up to 15
// classes; CPW = 2, two rows of z per class wave, for the 16 classes that would need a
// seventeenth wave).
//
// Class wave c owns row c of z ([K][d]): lane l holds the UPL consecutive strips
// (16 rounding bits each; UPL up to 8 at 8 bits, up to 16 at 16 bits) starting at l * UPL,
// with -h~ and the strips' Philox blocks of the current window of 8 steps, in registers for
// the whole epoch.
//
// The service wave owns everything that does not scale with d: it draws the
// sample indices, fetches the sampled rows of the quantized data and their margins
// two windows ahead and stages them in LDS, draws the rounding words of gamma and
// of the L2 term, and evaluates the softmax.  It holds no part of z, so its
// double-precision work has the register file to itself.
//
// One step:
//   class waves   x_i^T z_c (24-bit multiply-adds, DPP fold), one LDS word each      | barrier
//   service wave  softmax before and after the offset, one class per lane (lanes c    |
//                 and 16 + c), gamma_c = Q_(delta_s,b)(beta_c) into LDS;              |
//   class waves   meanwhile: operands of the update that do not need gamma, and one   |
//                 Philox block of the next window (parked in LDS until it starts)     | barrier
//   class waves   integer update of row c of z;
//   service wave  meanwhile, once per window: stage the next window, request the one after.
#include "halp_device.hpp"
#include "inner_args.hpp"

namespace halp {
namespace {

constexpr int kWin = 8;   // steps per window
constexpr int kKC = 16;   // classes are padded to one DPP row

__device__ __forceinline__ int mad24(int a, int b, int c) {
  int r;
  asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// the value of lane ^ 16 (the two rows of each half-wave trade places)
__device__ __forceinline__ double swap16_f64(double v) {
  const uint64_t u = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_swizzle((int)(uint32_t)u, 0x401F);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_swizzle((int)(u >> 32), 0x401F);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

template <typename F>
__device__ __forceinline__ double row_fold_f64(double v, F op) {
  auto step = [&](double x, auto mv) {
    const uint64_t u = __builtin_bit_cast(uint64_t, x);
    const uint32_t lo = (uint32_t)mv((int)(uint32_t)u), hi = (uint32_t)mv((int)(u >> 32));
    return op(x, __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo));
  };
  v = step(v, [](int t) { return dpp_quad_swap1(t); });
  v = step(v, [](int t) { return dpp_quad_swap2(t); });
  v = step(v, [](int t) { return dpp_half_mirror(t); });
  v = step(v, [](int t) { return dpp_row_mirror(t); });
  return v;
}

// Sum over each row of 16 lanes, left in every lane of the row: lanes are joined in
// adjacent pairs, the pairs' sums in adjacent pairs, and so on (a + b and b + a round
// alike, so every lane of a group holds the same bits).
__device__ __forceinline__ double row_sum_f64(double v) {
  return row_fold_f64(v, [](double x, double y) { return __dadd_rn(x, y); });
}

// maximum over each row of 16 lanes, left in every lane of the row
__device__ __forceinline__ double row_max_f64(double v) {
  return row_fold_f64(v, [](double x, double y) { return fmax(x, y); });
}

template <int BITS, int UPL, int KT, int CPW>
__global__ __launch_bounds__(64 * KT) void inner_softmax_kernel(InArgs a) {
  using XT = typename std::conditional<BITS == 8, int8_t, int16_t>::type;
  using HT = typename std::conditional<BITS == 8, int16_t, int32_t>::type;
  using AccT = typename std::conditional<BITS == 8, int, long long>::type;
  constexpr int CT = 16 / BITS;
  constexpr int CPL = UPL * CT;
  constexpr int NDW = (UPL + 1) / 2;
  constexpr int PQ = UPL >= 4 ? UPL / 4 : 1;  // 16-byte slots per word of a lane's parked blocks
  constexpr int BPS = (CPW * UPL + 7) / 8;    // Philox blocks of the next window made per step
  constexpr int kRowQ = UPL > 8 ? 8 : 4;      // dwords of a row per service lane: rows up to 1 / 2 KB
  // 16 strips per lane leave no registers for operands prepared ahead of gamma: the sampled
  // row stays packed and everything else of the update is formed after the second barrier
  // (and so does a second row of z per wave)
  constexpr bool LEAN = UPL > 8 || CPW > 1;
  // 8 bits: the two coordinates of a strip are kept and updated as the 16-bit halves of one
  // register (the class waves share their SIMDs three deep and are bound by issue slots)
  constexpr bool PK = BITS == 8 && !LEAN;
  typedef short S2 __attribute__((ext_vector_type(2)));
  constexpr int QMAX = (1 << (BITS - 1)) - 1, QMIN = -(1 << (BITS - 1));
  const int chain = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int d = a.d, K = a.K;
  const int U = (d + CT - 1) / CT;
  const int NACT = (U + UPL - 1) / UPL;  // lanes of a class wave that hold part of the row
  const int NP = K * NACT;               // ... of all class waves: slots of the parked blocks
  const int NCW = K / CPW;               // class waves; wave NCW is the service wave
  const int64_t T = epoch_steps(a.seed + (uint64_t)blockIdx.x, a.epoch, a.T, a.option2);
  const int64_t row_bytes = a.ldxq * (BITS / 8);
  const int row_dw = (int)(row_bytes / 4);
  const double* sc = a.scales + (int64_t)chain * 8;
  uint64_t* cnt_out = a.counters + (int64_t)chain * 4;
  const uint64_t seed = a.seed + (uint64_t)chain;
  const bool lp = a.lp != 0;  // Algorithm 2 (LP-SVRG): z is the model itself

  if (sc[7] != 0.0) {
    if (tid < 4) cnt_out[tid] = 0;
    return;
  }

  __shared__ __attribute__((aligned(16))) uint32_t s_rho[2][kWin][kKC];  // words of the gamma stream
  __shared__ __attribute__((aligned(16))) float s_phi[2][kWin][kKC];     // margins of the sampled rows
  __shared__ int s_creg[2][kWin];                                        // c_lambda
  __shared__ __attribute__((aligned(16))) AccT s_D[2][kKC];              // x_i^T z_c
  __shared__ int s_ng[2][kKC];                                           // -gamma_c
  __shared__ AccT s_dumpD[64];  // partial folds of lanes 0..62 of every class wave (never read)
  __shared__ unsigned long long s_cnt[3];
  // [2][kWin][row_dw] staged rows (coordinates past d staged as zeros), 32 bytes of zeros that
  // the lanes past the row read instead, then the parked Philox blocks: [word][slot][active
  // class lane] of 16 bytes, so that a wave reads consecutive addresses; a lane reads only its own
  extern __shared__ __attribute__((aligned(16))) uint32_t s_ring[];
  uint32_t* s_zero = s_ring + ((2 * kWin * row_dw + 3) & ~3);
  uint32_t* s_park = s_zero + 8;

  if (tid < 3) s_cnt[tid] = 0;
  if (tid < 8) s_zero[tid] = 0;
  const bool use_reg = a.lambda > 0;

  if (wave == NCW) {
    // ===================================================================== service wave
    // every class wave waits for this one at the step's second barrier: it goes first
    // wherever it shares a SIMD with class waves
    __builtin_amdgcn_s_setprio(3);
    const uint32_t N = (uint32_t)a.N;
    const unsigned char* __restrict__ Xq = reinterpret_cast<const unsigned char*>(a.Xq) +
                                           (int64_t)chain * a.xq_chain_stride * (BITS / 8);
    const float* __restrict__ phi = a.phi + (int64_t)chain * a.N * K;
    const double delta_m = sc[0], inv_s = sc[5];
    const double dscale = __dmul_rn(a.delta_d, delta_m);
    const double aB = a.hyper[2 * chain];  // alpha / B, B = 1
    const double al = __dmul_rn(aB, a.lambda);
    unsigned int n_gclamp = 0, n_reg = 0;

    // sample index of step tw + (lane & 7): any step number names a valid row, so windows
    // past T are fetched like the others and never used
    auto draw_idx = [&](int64_t tw) {
      const uint64_t t = (uint64_t)tw + (uint64_t)(lane & 7);
      const U4 r = stream_block(seed, kIdx, a.epoch, t >> 2);
      return (int)__umulhi(pick(r, (uint32_t)(t & 3)), N);
    };
    uint32_t xn[kWin][kRowQ];
    float phin[2];
    // coordinates of dword lane + 64 q that lie inside the row's d
    uint32_t smask[kRowQ];
#pragma unroll
    for (int q = 0; q < kRowQ; ++q) {
      const int nv = d - (lane + 64 * q) * (32 / BITS);
      smask[q] = nv >= 32 / BITS ? 0xFFFFFFFFu : (nv <= 0 ? 0u : (1u << (nv * BITS)) - 1u);
    }
    // dwords lane, lane + 64, ... of the window's rows; 8K margins, two per lane
    auto request = [&](int idxv) {
#pragma unroll
      for (int s = 0; s < kWin; ++s) {
        const int i = __builtin_amdgcn_readlane(idxv, s);
        const uint32_t* row = reinterpret_cast<const uint32_t*>(Xq + (int64_t)i * row_bytes);
#pragma unroll
        for (int q = 0; q < kRowQ; ++q) xn[s][q] = row[min(lane + 64 * q, row_dw - 1)];
      }
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int e = min(lane + 64 * q, kWin * K - 1);
        const int s = e / K, c = e - s * K;
        phin[q] = phi[(int64_t)__shfl(idxv, s) * K + c];
      }
    };
    auto stage = [&](int buf) {
#pragma unroll
      for (int s = 0; s < kWin; ++s)
#pragma unroll
        for (int q = 0; q < kRowQ; ++q)
          if (lane + 64 * q < row_dw)
            s_ring[(buf * kWin + s) * row_dw + lane + 64 * q] = xn[s][q] & smask[q];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int e = lane + 64 * q;
        if (e < kWin * K) {
          const int s = e / K, c = e - s * K;
          s_phi[buf][s][c] = phin[q];
        }
      }
    };
    // rounding words of gamma (word t*K + c of that stream; a window starts at a multiple
    // of 4 words) and c_lambda = Q_(2^-b, b)(alpha lambda) for the window starting at tw
    auto draw_scalars = [&](int64_t tw, int buf) {
      const uint64_t n0 = (uint64_t)tw * (uint64_t)K;
      if (lane < 2 * K) {
        const U4 rg = stream_block(seed, kGamma, a.epoch, (n0 >> 2) + (uint64_t)lane);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int rel = 4 * lane + e;  // = step * K + class
          const int s = rel / K;
          s_rho[buf][s][rel - s * K] = pick(rg, e);
        }
      }
      if (use_reg && lane < kWin) {
        const uint64_t t = (uint64_t)tw + (uint64_t)lane;
        const U4 rr = stream_block(seed, kReg, a.epoch, t >> 2);
        const int cl = (int)quantize_real(al, (double)(1 << BITS), pick(rr, (uint32_t)(t & 3)), 0.0,
                                          (double)QMAX, nullptr);
        s_creg[buf][lane] = cl;
        n_reg += (cl != 0 && (int64_t)t < T) ? 1u : 0u;
      }
    };

    // window 0 staged, window 1 requested
    request(draw_idx(0));
    stage(0);
    draw_scalars(0, 0);
    request(draw_idx(kWin));
    __syncthreads();

    const int lc = lane & 15;
    const bool after = (lane & 16) != 0;
    const bool live = lc < K;
    for (int64_t t0 = 0; t0 < T; t0 += kWin) {
      const int buf = (int)((t0 >> 3) & 1);
      for (int s = 0; s < kWin && t0 + s < T; ++s) {
        __syncthreads();  // the dot products of this step are in LDS
        double val = -INFINITY;
        uint32_t rw = 0;
        if (live) {
          const double a0 = (double)s_phi[buf][s][lc];
          // Algorithm 4 moves the margins by x^T z; in Algorithm 2 (LP-SVRG) x^T w is the margin
          const double moved = __dmul_rn(dscale, (double)s_D[s & 1][lc]);
          val = after ? (lp ? moved : __dadd_rn(a0, moved)) : a0;
          rw = s_rho[buf][s][lc];
        }
        const double mx = row_max_f64(val);
        const double e = live ? halp_exp(__dadd_rn(val, -mx)) : 0.0;
        // normaliser: pairwise over adjacent classes, the order the DPP fold gives
        const double p = __ddiv_rn(e, row_sum_f64(e));
        const double diff = __dadd_rn(swap16_f64(p), -p);  // lanes 0..15: p_after - p_before
        // beta_c = alpha (p_c(phi + x^T z) - p_c(phi)), gamma_c = Q_(delta_s, b)(beta_c)
        const double beta = __dmul_rn(aB, diff);
        const double rho = __dmul_rn((double)rw, 0x1p-32);
        const double f = floor(__dadd_rn(__dmul_rn(beta, inv_s), rho));
        const double fc = fmin(fmax(f, (double)QMIN), (double)QMAX);
        if (lane < K) {
          n_gclamp += (f != fc) ? 1u : 0u;
          s_ng[s & 1][lane] = (int)(-fc);
        }
        __syncthreads();  // gamma is out; the class waves update z
        if (s == 0) {
          // The other buffers were last read in the previous window: stage the next window
          // there, and request the one after it, which has eight steps to arrive.
          stage(buf ^ 1);
          draw_scalars(t0 + kWin, buf ^ 1);
          request(draw_idx(t0 + 2 * kWin));
        }
      }
    }
    if (n_gclamp) atomicAdd(&s_cnt[1], (unsigned long long)n_gclamp);
    if (n_reg) atomicAdd(&s_cnt[2], (unsigned long long)n_reg);
  } else {
    // ======================================================================= class wave
    // rows cls0 .. cls0 + CPW - 1 of z
    const int cls0 = wave * CPW;
    auto row0_of = [&](int cc) { return ((int64_t)chain * K + cls0 + cc) * d; };
    const int s0 = lane * UPL;
    const int j0 = s0 * CT;
    const bool lane_ok = s0 < U;  // = lane < NACT
    int z[CPW][CPL];
    int hv[CPW][CPL];  // -h~ at b = 8, h~ at b = 16
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
      const HT* __restrict__ hg = reinterpret_cast<const HT*>(a.h) + row0_of(cc);
      const XT* __restrict__ zg = reinterpret_cast<const XT*>(a.z) + row0_of(cc);
#pragma unroll
      for (int k = 0; k < CPL; ++k) {
        const int j = j0 + k;
        const bool ok = j < d;
        z[cc][k] = ok ? (int)zg[j] : 0;
        hv[cc][k] = ok ? (BITS == 8 ? -(int)hg[j] : (int)hg[j]) : 0;
      }
    }
    // packed form: z, and -h~ = 256 hh + hl with 0 <= hl < 256, two coordinates per register
    S2 zp[PK ? UPL : 1], hlp[PK ? UPL : 1], hhp[PK ? UPL : 1];
    if (PK) {
#pragma unroll
      for (int u = 0; u < UPL; ++u) {
        const int k0 = (2 * u) % CPL, k1 = (2 * u + 1) % CPL;
        zp[PK ? u : 0] = S2{(short)z[0][k0], (short)z[0][k1]};
        hlp[PK ? u : 0] = S2{(short)(hv[0][k0] & 0xFF), (short)(hv[0][k1] & 0xFF)};
        hhp[PK ? u : 0] = S2{(short)(hv[0][k0] >> 8), (short)(hv[0][k1] >> 8)};
      }
    }
    const int frag_dw = lane_ok ? (s0 * 2) >> 2 : 0;  // dword index of the fragment in a row
    const int half_sh = (UPL == 1 && lane_ok) ? ((s0 * 2) & 2) * 8 : 0;
    // first strip of this lane in row cc, and the slot of its parked blocks (lanes on the row only)
    auto strip0_of = [&](int cc) { return (uint32_t)((cls0 + cc) * U + s0); };
    auto pidx_of = [&](int cc) { return (cls0 + cc) * NACT + lane; };
    using LdsAcc = __attribute__((address_space(3))) AccT;
    LdsAcc* slotD[CPW][2];
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc)
#pragma unroll
      for (int par = 0; par < 2; ++par)
        slotD[cc][par] = (LdsAcc*)(lane == 63 ? &s_D[par][cls0 + cc] : &s_dumpD[lane]);
    const uint4* park = reinterpret_cast<const uint4*>(s_park);

    uint32_t zrw[CPW][4][UPL];  // the window's rounding words: [row][word of the block][strip]
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc)
#pragma unroll
      for (int u = 0; u < UPL; ++u) {
        const U4 r = zround_block(seed, a.epoch, strip0_of(cc) + (uint32_t)u, 0u);
        zrw[cc][0][u] = r.x; zrw[cc][1][u] = r.y; zrw[cc][2][u] = r.z; zrw[cc][3][u] = r.w;
      }
    unsigned long long n_zclamp = 0;
    __syncthreads();

    for (int64_t t0 = 0; t0 < T; t0 += kWin) {
      const int buf = (int)((t0 >> 3) & 1);
      const bool more = t0 + kWin < T;
      if (t0 > 0 && lane_ok) {  // the blocks parked during the previous window
#pragma unroll
        for (int cc = 0; cc < CPW; ++cc)
#pragma unroll
          for (int wd = 0; wd < 4; ++wd)
#pragma unroll
            for (int q = 0; q < PQ; ++q) {
              const uint4 v = park[(wd * PQ + q) * NP + pidx_of(cc)];
              if (4 * q + 0 < UPL) zrw[cc][wd][(4 * q + 0) % UPL] = v.x;
              if (4 * q + 1 < UPL) zrw[cc][wd][(4 * q + 1) % UPL] = v.y;
              if (4 * q + 2 < UPL) zrw[cc][wd][(4 * q + 2) % UPL] = v.z;
              if (4 * q + 3 < UPL) zrw[cc][wd][(4 * q + 3) % UPL] = v.w;
            }
      }
#pragma unroll
      for (int s = 0; s < kWin; ++s) {
        if (t0 + s < T) {
          // this lane's fragment of the row, from the ring (zeros for the lanes past the row)
          uint32_t xw[NDW];
          {
            const uint32_t* rp =
                lane_ok ? s_ring + (buf * kWin + s) * row_dw + frag_dw : s_zero;
            if (NDW == 1) {
              xw[0] = rp[0];
              if (UPL == 1) xw[0] = (xw[0] >> half_sh) & 0xFFFFu;
            } else if (NDW == 2) {
              const uint2 v = *reinterpret_cast<const uint2*>(rp);
              xw[0] = v.x; xw[NDW > 1 ? 1 : 0] = v.y;
            } else {
#pragma unroll
              for (int q = 0; q < NDW / 4; ++q) {
                const uint4 v = reinterpret_cast<const uint4*>(rp)[q];
                xw[4 * q] = v.x; xw[NDW > 1 ? 4 * q + 1 : 0] = v.y;
                xw[NDW > 2 ? 4 * q + 2 : 0] = v.z; xw[NDW > 3 ? 4 * q + 3 : 0] = v.w;
              }
            }
          }
          auto x_of = [&](int k) {
            const uint32_t xv = xw[(k * BITS) / 32];
            const int xs = (k * BITS) % 32;
            return BITS == 8 ? (int)(int8_t)(xv >> xs) : (int)(int16_t)(xv >> xs);
          };
          int xe[LEAN ? 1 : CPL];
          S2 xp[PK ? UPL : 1];
          AccT part[CPW];
#pragma unroll
          for (int cc = 0; cc < CPW; ++cc) part[cc] = 0;
          if (PK) {
            // the strip's two bytes go to the high bytes of the halves and come back down with
            // their signs; one packed dot per strip
#pragma unroll
            for (int u = 0; u < UPL; ++u) {
              const uint32_t up = __builtin_amdgcn_perm(0u, xw[u / 2], (u & 1) ? 0x030C020Cu : 0x010C000Cu);
              xp[PK ? u : 0] = __builtin_bit_cast(S2, up) >> (S2)(8);
              part[0] = (AccT)__builtin_amdgcn_sdot2(xp[PK ? u : 0], zp[PK ? u : 0], (int)part[0], false);
            }
          } else if (!LEAN) {
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
              xe[LEAN ? 0 : k] = x_of(k);
              if (BITS == 8) part[0] = (AccT)mad24(xe[LEAN ? 0 : k], z[0][k], (int)part[0]);
            }
          } else if (BITS == 8) {
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
              const int xk = x_of(k);
#pragma unroll
              for (int cc = 0; cc < CPW; ++cc) part[cc] = (AccT)mad24(xk, z[cc][k], (int)part[cc]);
            }
          }
          if (BITS == 16) {
            // two products of 16-bit factors fit 32 bits; their sums are added in 64
#pragma unroll
            for (int cc = 0; cc < CPW; ++cc) {
              if (CPL == 1) {
                part[cc] = (AccT)mad24(x_of(0), z[cc][0], 0);
              } else {
#pragma unroll
                for (int k = 0; k + 1 < CPL; k += 2)
                  part[cc] += (AccT)mad24(x_of(k), z[cc][k], mad24(x_of(k + 1), z[cc][k + 1], 0));
              }
            }
          }
          // the fold leaves the sum in lane 63, which stores it; the other lanes store their
          // partial folds into a dump row, so that no lane mask is set up and no lane is read
#pragma unroll
          for (int cc = 0; cc < CPW; ++cc) {
            AccT D;
            if (BITS == 8) D = (AccT)wave_fold_i32((int)part[cc]);
            else D = (AccT)wave_fold_i64((long long)part[cc]);
            *slotD[cc][s & 1] = D;
          }
          __syncthreads();
          // While the service wave evaluates the softmax: the part of the update that does
          // not need gamma, and the Philox blocks of the next window.
          // b = 8: hr = -h~ + rounding bits.  b = 16: with h~ = 2^16 hh + hl, 0 <= hl < 2^16,
          // floor((-gamma x + bits - h~) / 2^16) = floor((-gamma x + bits - hl) / 2^16) - hh, and
          // the numerator on the right fits 32 bits; hr = bits - hl.
          auto hr_of = [&](int cc, int k) {
            const uint32_t word = zrw[cc][s >> 1][k / CT];
            const int sh = 16 * (s & 1) + (k % CT) * BITS;
            const int re = (int)((word >> sh) & (BITS == 8 ? 0xFFu : 0xFFFFu));
            if (BITS == 16) asm volatile("" : "+v"(hv[cc][k]));  // keeps hl, hh from being hoisted into registers
            return BITS == 8 ? hv[cc][k] + re : re - (hv[cc][k] & 0xFFFF);
          };
          int hr[LEAN ? 1 : CPL];
          S2 crp[PK ? UPL : 1], zh[PK ? UPL : 1];
          if (PK) {
#pragma unroll
            for (int u = 0; u < UPL; ++u) {
              const uint32_t rp = __builtin_amdgcn_perm(0u, zrw[0][s >> 1][u], (s & 1) ? 0x0C030C02u : 0x0C010C00u);
              crp[PK ? u : 0] = __builtin_bit_cast(S2, rp) + hlp[PK ? u : 0];  // rounding bits + hl
              zh[PK ? u : 0] = hhp[PK ? u : 0] + zp[PK ? u : 0];
            }
          } else if (!LEAN) {
#pragma unroll
            for (int k = 0; k < CPL; ++k) hr[LEAN ? 0 : k] = hr_of(0, k);
          }
#pragma unroll
          for (int q = 0; q < BPS; ++q) {
            if (q > 0) __builtin_amdgcn_sched_barrier(0);  // one block's temporaries at a time
            const int ub = s * BPS + q;  // block number within the window: row ub / UPL, strip ub % UPL
            if (ub < CPW * UPL && more) {
              const int cc = ub / UPL, u = ub % UPL;
              const U4 r = zround_block(seed, a.epoch, strip0_of(cc) + (uint32_t)u, (uint32_t)(t0 >> 3) + 1u);
              if (lane_ok) {
                uint32_t* slot = s_park + ((size_t)((u / 4) * NP + pidx_of(cc))) * 4 + (u % 4);
                const size_t word_stride = (size_t)PQ * NP * 4;
                slot[0] = r.x; slot[word_stride] = r.y; slot[2 * word_stride] = r.z; slot[3 * word_stride] = r.w;
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
          __syncthreads();
          int ng[CPW];
#pragma unroll
          for (int cc = 0; cc < CPW; ++cc) ng[cc] = s_ng[s & 1][cls0 + cc];
          const int cl = use_reg ? __builtin_amdgcn_readfirstlane(s_creg[buf][s]) : 0;
          // u = z - gamma x - h~ (- c_lambda z), z = Q_(delta_m, b)(u)
          auto update = [&](auto with_l2) {
#pragma unroll
            for (int cc = 0; cc < CPW; ++cc)
#pragma unroll
              for (int k = 0; k < CPL; ++k) {
                int hk = LEAN ? hr_of(cc, k) : hr[LEAN ? 0 : k];
                if (decltype(with_l2)::value) hk = mad24(-cl, z[cc][k], hk);
                const int xk = LEAN ? x_of(k) : xe[LEAN ? 0 : k];
                int zu;
                if (BITS == 8) zu = z[cc][k] + (mad24(ng[cc], xk, hk) >> 8);
                else zu = z[cc][k] + (mad24(ng[cc], xk, hk) >> 16) - (hv[cc][k] >> 16);
                const int zc = min(max(zu, QMIN), QMAX);
                // clamps are counted on the scalar unit: one compare here, the rest is wave-wide
                n_zclamp += (unsigned long long)__builtin_popcountll(__ballot(zu != zc));
                z[cc][k] = zc;
              }
          };
          if (PK && cl == 0) {
            // per half: floor((-gamma x + r + hl) / 256) + hh + z; |gamma x| <= 2^14 and
            // r + hl < 512, so every intermediate fits 16 bits
            const S2 ngp = S2{(short)ng[0], (short)ng[0]};
            S2 vu[PK ? UPL : 1];
            uint32_t moved = 0;
#pragma unroll
            for (int u = 0; u < (PK ? UPL : 0); ++u) {
              S2 v = xp[u] * ngp + crp[u];
              v = (v >> (S2)(8)) + zh[u];
              const S2 zc = __builtin_elementwise_min(__builtin_elementwise_max(v, (S2)(QMIN)), (S2)(QMAX));
              moved |= __builtin_bit_cast(uint32_t, v) ^ __builtin_bit_cast(uint32_t, zc);
              vu[u] = v;
              zp[u] = zc;
            }
            if (__ballot(moved != 0) != 0) {  // rare: count the clamped coordinates exactly
#pragma unroll
              for (int u = 0; u < (PK ? UPL : 0); ++u) {
                const uint32_t df = __builtin_bit_cast(uint32_t, vu[u]) ^ __builtin_bit_cast(uint32_t, zp[u]);
                n_zclamp += (unsigned long long)__builtin_popcountll(__ballot((df & 0xFFFFu) != 0)) +
                            (unsigned long long)__builtin_popcountll(__ballot((df >> 16) != 0));
              }
            }
          } else if (PK) {  // a step with an L2 draw: unpack, the scalar form, pack again
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
              z[0][k] = (int)zp[(k / 2) % UPL][k % 2];
              xe[LEAN ? 0 : k] = (int)xp[(k / 2) % UPL][k % 2];
              hr[LEAN ? 0 : k] = hr_of(0, k);
            }
            update(std::true_type{});
#pragma unroll
            for (int u = 0; u < (PK ? UPL : 0); ++u) zp[u] = S2{(short)z[0][(2 * u) % CPL], (short)z[0][(2 * u + 1) % CPL]};
          } else if (cl != 0) update(std::true_type{});  // the L2 term is rare: c_lambda is mostly 0
          else update(std::false_type{});
        }
        __builtin_amdgcn_sched_barrier(0);  // keep one step's temporaries from overlapping the next's
      }
    }

    // ---- w~ <- w~ + delta_m z (option I); hand z out
    if (PK) {
#pragma unroll
      for (int k = 0; k < CPL; ++k) z[0][k] = (int)zp[(k / 2) % UPL][k % 2];
    }
    const double delta_m = sc[0];
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
      XT* __restrict__ zg = reinterpret_cast<XT*>(a.z) + row0_of(cc);
      float* __restrict__ wg = a.w + row0_of(cc);
      float wv[CPL];
#pragma unroll
      for (int k = 0; k < CPL; ++k) wv[k] = wg[min(j0 + k, d - 1)];  // all loads in flight at once
#pragma unroll
      for (int k = 0; k < CPL; ++k) {
        const int j = j0 + k;
        if (j < d) {
          zg[j] = (XT)z[cc][k];
          const double step = __dmul_rn(delta_m, (double)z[cc][k]);
          wg[j] = lp ? (float)step : (float)__dadd_rn((double)wv[k], step);  // Alg. 2: w~ = delta w
        }
      }
    }
    if (lane == 0 && n_zclamp) atomicAdd(&s_cnt[0], n_zclamp);  // wave-wide count
  }
  __syncthreads();
  if (tid < 4) cnt_out[tid] = tid < 3 ? s_cnt[tid] : 0ull;
}

template <int BITS, int UPL>
int launch_kt(const InArgs& a, int R, size_t smem, hipStream_t s) {
  // one row of z per class wave up to 15 classes; 16 classes: two rows per wave, 8 + 1 waves
  const int cpw = a.K > 15 ? 2 : 1;
  const dim3 grid(R), block(64 * (a.K / cpw + 1));
#define HALP_SM(KT_, CPW_)                                                                        \
  do {                                                                                            \
    auto kern = inner_softmax_kernel<BITS, UPL, KT_, CPW_>;                                       \
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                  \
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess) \
      return HALP_ERR_HIP;                                                                        \
    hipLaunchKernelGGL(kern, grid, block, smem, s, a);                                            \
  } while (0)
  if (cpw == 2) {
    if constexpr (UPL <= 8) HALP_SM(12, 2);
    else return HALP_ERR_UNSUPPORTED;
  } else if (a.K + 1 <= 4) HALP_SM(4, 1);
  else if (a.K + 1 <= 8) HALP_SM(8, 1);
  else if (a.K + 1 <= 12) HALP_SM(12, 1);
  else HALP_SM(16, 1);
#undef HALP_SM
  return hip_ok(hipGetLastError());
}

template <int BITS>
int launch_upl(const InArgs& a, int upl, int R, size_t smem, hipStream_t s) {
  switch (upl) {
    case 1: return launch_kt<BITS, 1>(a, R, smem, s);
    case 2: return launch_kt<BITS, 2>(a, R, smem, s);
    case 4: return launch_kt<BITS, 4>(a, R, smem, s);
    case 8: return launch_kt<BITS, 8>(a, R, smem, s);
    default: return HALP_ERR_UNSUPPORTED;
  }
}

// 16 strips per lane exist at 16 bits only (16 coordinates per lane; at 8 bits they would be 32)
int launch_upl16(const InArgs& a, int R, size_t smem, hipStream_t s) {
  return launch_kt<16, 16>(a, R, smem, s);
}

int strips_per_lane(const halp_params& p) {
  const int ct = 16 / p.b;
  const int U = (p.d + ct - 1) / ct;
  const int upl = (U + 63) / 64;
  int u2 = 1;
  while (u2 < upl) u2 *= 2;
  return u2;
}

// the ring of staged rows, 32 bytes of zeros, and the parked Philox blocks (16 bytes per
// strip, 64 at least, per class lane that holds part of the row)
size_t dynamic_lds(const halp_params& p, int64_t row_bytes) {
  const int upl = strips_per_lane(p);
  const int ct = 16 / p.b;
  const int U = (p.d + ct - 1) / ct;
  const int nact = (U + upl - 1) / upl;
  const size_t ring = (((size_t)2 * kWin * (size_t)row_bytes) + 15) / 16 * 16;
  return ring + 32 + (size_t)nact * p.K * 16 * (size_t)(upl >= 4 ? upl : 4);
}

}  // namespace

// softmax, one row per step, up to 15 classes one wave each plus the service wave, 16 classes
// two to a wave (8 strips per lane at most then, for the registers of two rows of z), a
// class's row of z within one wave (8 strips per lane at most at 8 bits, 16 at 16 bits), data
// rows up to 1 KB (2 KB at 16 strips per lane), everything staged within the LDS of a CU
int inner_softmax_supported(const halp_handle& h) {
  const halp_params& p = h.p;
  if (p.loss != HALP_LOSS_SOFTMAX || p.B != 1 || p.K < 2 || p.K > 16) return HALP_ERR_UNSUPPORTED;
  if (p.b == 8 && p.d > 131071) return HALP_ERR_UNSUPPORTED;  // int32 dot product stays exact
  const int upl = strips_per_lane(p);
  if (upl > (p.b == 16 && p.K <= 15 ? 16 : 8)) return HALP_ERR_UNSUPPORTED;
  if (!h.bound || !h.buf.Xq) return HALP_ERR_NOT_BOUND;
  const int64_t row_bytes = h.buf.ldxq * (p.b / 8);
  const int ct = 16 / p.b;
  const int U = (p.d + ct - 1) / ct;
  // fragments are read whole (2 * UPL bytes, up to 16) from the staged row
  const int frag = upl >= 8 ? 16 : (upl == 4 ? 8 : 4);
  if (row_bytes % frag != 0 || row_bytes / 4 > 64 * (upl > 8 ? 8 : 4)) return HALP_ERR_UNSUPPORTED;
  if ((int64_t)((U + upl - 1) / upl) * upl * 2 > row_bytes) return HALP_ERR_UNSUPPORTED;
  if (dynamic_lds(p, row_bytes) > 156 * 1024) return HALP_ERR_UNSUPPORTED;  // 160 KB less the static part
  return HALP_OK;
}

int launch_inner_softmax(const halp_handle& h, uint32_t epoch, hipStream_t s) {
  const halp_params& p = h.p;
  const int rc = inner_softmax_supported(h);
  if (rc != HALP_OK) return rc;
  const InArgs a = make_inner_args(h, epoch);
  const int upl = strips_per_lane(p);
  const size_t smem = dynamic_lds(p, h.buf.ldxq * (p.b / 8));
  if (upl == 16) return launch_upl16(a, p.R, smem, s);
  return p.b == 8 ? launch_upl<8>(a, upl, p.R, smem, s) : launch_upl<16>(a, upl, p.R, smem, s);
}

}  // namespace halp
