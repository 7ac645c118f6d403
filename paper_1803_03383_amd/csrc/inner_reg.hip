// Inner loop of Algorithm 4 (LM-HALP), register-resident form for one sampled
// row per step (B = 1) and one class (squared or logistic loss).
//
// One workgroup per chain, NW waves.  A lane owns GPL groups of coordinates; a
// group is the 64/b coordinates that share 64 rounding bits, i.e. 8 bytes of a
// data row.  z (unpacked and packed), -h~ and a ring of prefetched data rows
// stay in registers for the whole epoch; nothing but the sampled rows is read
// from memory inside the loop.  Per step:
//   dot      v_dot4 (b=8) / v_dot2 (b=16) on packed z, folded across the wave
//            with DPP and across waves through one LDS word per wave
//   scalar   beta and gamma = Q_(delta_s,b)(beta) in fp64, wave-uniform
//   update   u = -gamma x - h~ (- c_lambda z) in (delta_i, 2b), stochastic
//            rounding with b Philox bits per coordinate, clamp to the box
// Sample indices and the gamma / L2 rounding words are pure functions of the
// step number, so they are produced 256 steps at a time into LDS and rows are
// requested PF steps before they are needed.
#include "halp_device.hpp"
#include "inner_args.hpp"

namespace halp {
namespace {

typedef short short2v __attribute__((ext_vector_type(2)));

constexpr int kBatch = 256;  // steps per batch of precomputed draws
constexpr int kPF = 8;       // rows in flight

__device__ __forceinline__ double logistic_dl(double a, double y) {
  return __ddiv_rn(-y, __dadd_rn(1.0, exp(__dmul_rn(y, a))));
}

template <int BITS, int LOSS, int GPL, bool RAGGED, bool COUNT, int MAXT>
__global__ __launch_bounds__(MAXT) void inner_reg_kernel(InArgs a) {
  using XT = typename std::conditional<BITS == 8, int8_t, int16_t>::type;
  using HT = typename std::conditional<BITS == 8, int16_t, int32_t>::type;
  using AccT = typename std::conditional<BITS == 8, int, long long>::type;
  constexpr int CPG = 64 / BITS;
  constexpr int QMAX = (1 << (BITS - 1)) - 1, QMIN = -(1 << (BITS - 1));
  const int chain = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int NW = blockDim.x >> 6;
  const int d = a.d;
  const int G = (d + CPG - 1) / CPG;
  const int64_t N = a.N;
  const int64_t row_bytes = a.ldxq * (BITS / 8);
  const unsigned char* __restrict__ Xq = reinterpret_cast<const unsigned char*>(a.Xq) +
                                         (int64_t)chain * a.xq_chain_stride * (BITS / 8);
  const float* __restrict__ phi = a.phi + (int64_t)chain * N;
  const float* __restrict__ y =
      reinterpret_cast<const float*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const HT* __restrict__ hg = reinterpret_cast<const HT*>(a.h) + (int64_t)chain * d;
  XT* __restrict__ zg = reinterpret_cast<XT*>(a.z) + (int64_t)chain * d;
  float* __restrict__ wg = a.w + (int64_t)chain * d;
  const double* sc = a.scales + (int64_t)chain * 8;
  uint64_t* cnt_out = a.counters + (int64_t)chain * 4;
  const uint64_t seed = a.seed + (uint64_t)chain;

  if (sc[7] != 0.0) {
    if (tid < 4) cnt_out[tid] = 0;
    return;
  }

  __shared__ int s_idx[2 * kBatch];
  __shared__ uint32_t s_rho[2 * kBatch];
  __shared__ int s_creg[2 * kBatch];
  __shared__ AccT s_part[2][16];
  __shared__ unsigned long long s_cnt[3];

  const double delta_m = sc[0], inv_s = sc[5];
  const double dscale = __dmul_rn(a.delta_d, delta_m);
  const double aB = a.alpha;  // B = 1: alpha / 1
  const bool use_reg = a.lambda > 0;
  const double al = __dmul_rn(a.alpha, a.lambda);

  // ---- per-lane state
  int gidx[GPL];   // group index (also the Philox counter word 0)
  bool gok[GPL];
  int z[GPL][CPG];
  int nh[GPL][CPG];  // -h~ when b = 8 (fits), h~ itself when b = 16 (its negation may not fit)
  uint32_t zp[GPL][2];
  uint32_t xmask[GPL][2];
#pragma unroll
  for (int q = 0; q < GPL; ++q) {
    gidx[q] = wave * 64 + lane + q * 64 * NW;
    gok[q] = gidx[q] < G;
    zp[q][0] = zp[q][1] = 0;
    xmask[q][0] = xmask[q][1] = 0;
#pragma unroll
    for (int e = 0; e < CPG; ++e) {
      const int j = gidx[q] * CPG + e;
      const bool ok = gok[q] && j < d;
      z[q][e] = ok ? (int)zg[j] : 0;
      nh[q][e] = ok ? (BITS == 8 ? -(int)hg[j] : (int)hg[j]) : 0;
      if (ok) xmask[q][(e * BITS) / 32] |= (BITS == 8 ? 0xFFu : 0xFFFFu) << ((e * BITS) % 32);
    }
  }
  auto repack = [&]() {
#pragma unroll
    for (int q = 0; q < GPL; ++q) {
      if (BITS == 8) {
        zp[q][0] = (uint32_t)(z[q][0] & 0xFF) | ((uint32_t)(z[q][1] & 0xFF) << 8) |
                   ((uint32_t)(z[q][2] & 0xFF) << 16) | ((uint32_t)z[q][3] << 24);
        zp[q][1] = (uint32_t)(z[q][4 % CPG] & 0xFF) | ((uint32_t)(z[q][5 % CPG] & 0xFF) << 8) |
                   ((uint32_t)(z[q][6 % CPG] & 0xFF) << 16) | ((uint32_t)z[q][7 % CPG] << 24);
      } else {
        zp[q][0] = (uint32_t)(z[q][0] & 0xFFFF) | ((uint32_t)z[q][1] << 16);
        zp[q][1] = (uint32_t)(z[q][2 % CPG] & 0xFFFF) | ((uint32_t)z[q][3 % CPG] << 16);
      }
    }
  };
  repack();

  // ---- draws that depend on the step number only, 256 steps per batch
  auto fill_batch = [&](int64_t bb) {
    const int half = (int)(bb & 1) * kBatch;
    if (tid < 64) {
      const uint64_t blk = (uint64_t)bb * 64 + (uint64_t)tid;
      const U4 ri = stream_block(seed, kIdx, a.epoch, blk);
      const U4 rg = stream_block(seed, kGamma, a.epoch, blk);
      s_idx[half + 4 * tid + 0] = (int)__umulhi(ri.x, (uint32_t)N);
      s_idx[half + 4 * tid + 1] = (int)__umulhi(ri.y, (uint32_t)N);
      s_idx[half + 4 * tid + 2] = (int)__umulhi(ri.z, (uint32_t)N);
      s_idx[half + 4 * tid + 3] = (int)__umulhi(ri.w, (uint32_t)N);
      s_rho[half + 4 * tid + 0] = rg.x;
      s_rho[half + 4 * tid + 1] = rg.y;
      s_rho[half + 4 * tid + 2] = rg.z;
      s_rho[half + 4 * tid + 3] = rg.w;
      if (use_reg) {
        const U4 rr = stream_block(seed, kReg, a.epoch, blk);
        const double two_b = (double)(1 << BITS);
        s_creg[half + 4 * tid + 0] = (int)quantize_real(al, two_b, rr.x, 0.0, (double)QMAX, nullptr);
        s_creg[half + 4 * tid + 1] = (int)quantize_real(al, two_b, rr.y, 0.0, (double)QMAX, nullptr);
        s_creg[half + 4 * tid + 2] = (int)quantize_real(al, two_b, rr.z, 0.0, (double)QMAX, nullptr);
        s_creg[half + 4 * tid + 3] = (int)quantize_real(al, two_b, rr.w, 0.0, (double)QMAX, nullptr);
      }
    }
  };
  if (tid < 3) s_cnt[tid] = 0;
  fill_batch(0);
  fill_batch(1);
  __syncthreads();

  // ---- ring of prefetched rows
  uint32_t xr[kPF][GPL][2];
  float ring_phi[kPF], ring_y[kPF];
  auto request = [&](int slot, int64_t t) {
    const int i = s_idx[t & (2 * kBatch - 1)];
    const unsigned char* rp = Xq + (int64_t)i * row_bytes;
#pragma unroll
    for (int q = 0; q < GPL; ++q) {
      uint2 v = make_uint2(0u, 0u);
      if (gok[q]) v = *reinterpret_cast<const uint2*>(rp + (int64_t)gidx[q] * 8);
      xr[slot][q][0] = v.x;
      xr[slot][q][1] = v.y;
    }
    if (LOSS == HALP_LOSS_LOGISTIC) {
      ring_phi[slot] = phi[i];
      ring_y[slot] = y[i];
    }
  };
#pragma unroll
  for (int s = 0; s < kPF; ++s) {
    if (s < a.T) request(s, s);
  }

  unsigned int n_zclamp = 0, n_gclamp = 0, n_reg = 0;
  U4 zr[GPL];

  auto step = [&](int slot, int64_t t) {
    // low-precision dot product x_i^T z
    AccT part = 0;
#pragma unroll
    for (int q = 0; q < GPL; ++q) {
      uint32_t x0 = xr[slot][q][0], x1 = xr[slot][q][1];
      if (RAGGED) { x0 &= xmask[q][0]; x1 &= xmask[q][1]; xr[slot][q][0] = x0; xr[slot][q][1] = x1; }
      if (BITS == 8) {
        part = __builtin_amdgcn_sdot4((int)x0, (int)zp[q][0], (int)part, false);
        part = __builtin_amdgcn_sdot4((int)x1, (int)zp[q][1], (int)part, false);
      } else {
        part += (AccT)__builtin_amdgcn_sdot2(__builtin_bit_cast(short2v, x0),
                                             __builtin_bit_cast(short2v, zp[q][0]), 0, false);
        part += (AccT)__builtin_amdgcn_sdot2(__builtin_bit_cast(short2v, x1),
                                             __builtin_bit_cast(short2v, zp[q][1]), 0, false);
      }
    }
    AccT D;
    if (BITS == 8) D = (AccT)wave_sum_i32((int)part);
    else D = (AccT)wave_sum_i64((long long)part);
    if (NW > 1) {
      if (lane == 0) s_part[t & 1][wave] = D;
      __syncthreads();
      AccT tot = 0;
      for (int w2 = 0; w2 < NW; ++w2) tot += s_part[t & 1][w2];
      D = tot;
    }
    // beta = alpha (l'(phi_i + x_i^T z) - l'(phi_i)), gamma = Q_(delta_s, b)(beta)
    const double delta = __dmul_rn(dscale, (double)D);
    double diff;
    if (LOSS == HALP_LOSS_SQUARED) {
      diff = delta;
    } else {
      const double a0 = (double)ring_phi[slot], yi = (double)ring_y[slot];
      diff = __dadd_rn(logistic_dl(__dadd_rn(a0, delta), yi), -logistic_dl(a0, yi));
    }
    const double beta = __dmul_rn(aB, diff);
    bool ghit = false;
    const int gamma = (int)quantize_real(beta, inv_s, s_rho[t & (2 * kBatch - 1)], (double)QMIN,
                                         (double)QMAX, &ghit);
    n_gclamp += ghit ? 1u : 0u;
    const int ng = -gamma;
    int cl = 0;
    if (use_reg) {
      cl = s_creg[t & (2 * kBatch - 1)];
      n_reg += cl != 0 ? 1u : 0u;
    }
    // rounding bits: one Philox block per group serves steps 2s and 2s+1
    if ((slot & 1) == 0) {  // kPF is even and t - slot a multiple of kPF: slot parity is t parity
#pragma unroll
      for (int q = 0; q < GPL; ++q) zr[q] = zround_block(seed, a.epoch, (uint32_t)gidx[q], (uint32_t)(t >> 1));
    }
    // u = z - gamma x - h~ (- c_lambda z), z = Q_(delta_m, b)(u)
#pragma unroll
    for (int q = 0; q < GPL; ++q) {
      const uint32_t b0 = (slot & 1) ? zr[q].z : zr[q].x, b1 = (slot & 1) ? zr[q].w : zr[q].y;
#pragma unroll
      for (int e = 0; e < CPG; ++e) {
        const uint32_t xw = xr[slot][q][(e * BITS) / 32];
        const uint32_t bw = (e * BITS) / 32 ? b1 : b0;
        const int sh = (e * BITS) % 32;
        int xe, re;
        if (BITS == 8) {
          xe = (int)(int8_t)(xw >> sh);
          re = (int)((bw >> sh) & 0xFFu);
        } else {
          xe = (int)(int16_t)(xw >> sh);
          re = (int)((bw >> sh) & 0xFFFFu);
        }
        int zu;
        if (BITS == 8) {
          int v = ng * xe + nh[q][e];
          if (use_reg) v -= cl * z[q][e];
          zu = z[q][e] + ((v + re) >> 8);
        } else {
          long long v = (long long)ng * (long long)xe - (long long)nh[q][e];
          if (use_reg) v -= (long long)cl * (long long)z[q][e];
          zu = z[q][e] + (int)((v + (long long)re) >> 16);
        }
        const int zc = min(max(zu, QMIN), QMAX);
        if (COUNT) n_zclamp += (zu != zc) ? 1u : 0u;
        z[q][e] = zc;
      }
    }
    repack();
  };

  const int64_t T = a.T;
  for (int64_t t0 = 0; t0 < T; t0 += kPF) {
    if ((t0 & (kBatch - 1)) == 0 && t0 > 0) {
      // every wave has finished batch t0/256 - 1; refill its half with batch t0/256 + 1
      __syncthreads();
      fill_batch(t0 / kBatch + 1);
      __syncthreads();
    }
#pragma unroll
    for (int s = 0; s < kPF; ++s) {
      const int64_t t = t0 + s;
      if (t < T) {
        step(s, t);
        if (t + kPF < T) request(s, t + kPF);
      }
    }
  }

  // ---- w~ <- w~ + delta_m z (option I); hand z out
#pragma unroll
  for (int q = 0; q < GPL; ++q) {
#pragma unroll
    for (int e = 0; e < CPG; ++e) {
      const int j = gidx[q] * CPG + e;
      if (gok[q] && j < d) {
        zg[j] = (XT)z[q][e];
        wg[j] = (float)__dadd_rn((double)wg[j], __dmul_rn(delta_m, (double)z[q][e]));
      }
    }
  }
  if (COUNT && n_zclamp) atomicAdd(&s_cnt[0], (unsigned long long)n_zclamp);
  if (tid == 0) {
    s_cnt[1] = n_gclamp;  // gamma is wave-uniform: count it once
    s_cnt[2] = n_reg;
  }
  __syncthreads();
  if (tid < 4) {
    unsigned long long v = tid < 3 ? s_cnt[tid] : 0ull;
    if (tid == 0 && !COUNT) v = ~0ull;
    cnt_out[tid] = v;
  }
}

struct Shape {
  int nw, gpl;
};

Shape pick_shape(const halp_params& p) {
  const int cpg = 64 / p.b;
  const int G = (p.d + cpg - 1) / cpg;
  int nw = 1;
  while (nw < 4 && nw * 64 < G) nw *= 2;
  int gpl = (G + 64 * nw - 1) / (64 * nw);
  int g2 = 1;
  while (g2 < gpl) g2 *= 2;
  // more than 4 groups per lane: widen the workgroup instead, up to 16 waves
  while (g2 > 4 && nw < 16) {
    nw *= 2;
    gpl = (G + 64 * nw - 1) / (64 * nw);
    g2 = 1;
    while (g2 < gpl) g2 *= 2;
  }
  return Shape{nw, g2};
}

template <int BITS, int LOSS, int GPL>
int launch_shape(const InArgs& a, int nw, bool ragged, bool count, int R, hipStream_t s) {
  const dim3 grid(R), block(64 * nw);
#define HALP_LAUNCH(RG, CT)                                                                 \
  do {                                                                                      \
    if (nw <= 4)                                                                            \
      hipLaunchKernelGGL((inner_reg_kernel<BITS, LOSS, GPL, RG, CT, 256>), grid, block, 0, s, a); \
    else                                                                                    \
      hipLaunchKernelGGL((inner_reg_kernel<BITS, LOSS, GPL, RG, CT, 1024>), grid, block, 0, s, a); \
  } while (0)
  if (ragged) {
    if (count) HALP_LAUNCH(true, true); else HALP_LAUNCH(true, false);
  } else {
    if (count) HALP_LAUNCH(false, true); else HALP_LAUNCH(false, false);
  }
#undef HALP_LAUNCH
  return hip_ok(hipGetLastError());
}

template <int BITS, int LOSS>
int launch_gpl(const InArgs& a, Shape sh, bool ragged, bool count, int R, hipStream_t s) {
  switch (sh.gpl) {
    case 1: return launch_shape<BITS, LOSS, 1>(a, sh.nw, ragged, count, R, s);
    case 2: return launch_shape<BITS, LOSS, 2>(a, sh.nw, ragged, count, R, s);
    case 4: return launch_shape<BITS, LOSS, 4>(a, sh.nw, ragged, count, R, s);
    default: return HALP_ERR_UNSUPPORTED;
  }
}

}  // namespace

int inner_reg_supported(const halp_params& p) {
  if (p.B != 1 || p.K != 1) return HALP_ERR_UNSUPPORTED;
  if (p.loss != HALP_LOSS_SQUARED && p.loss != HALP_LOSS_LOGISTIC) return HALP_ERR_UNSUPPORTED;
  if (p.b == 8 && p.d > 131071) return HALP_ERR_UNSUPPORTED;  // int32 dot product stays exact
  const Shape sh = pick_shape(p);
  if (sh.gpl > 4) return HALP_ERR_UNSUPPORTED;
  return HALP_OK;
}

int launch_inner_reg(const halp_handle& h, uint32_t epoch, hipStream_t s) {
  const halp_params& p = h.p;
  int rc = inner_reg_supported(p);
  if (rc != HALP_OK) return rc;
  const InArgs a = make_inner_args(h, epoch);
  const Shape sh = pick_shape(p);
  const int cpg = 64 / p.b;
  const bool ragged = (p.d % cpg) != 0;
  const bool count = h.count_clamps;
  if (p.b == 8) {
    if (p.loss == HALP_LOSS_SQUARED) return launch_gpl<8, HALP_LOSS_SQUARED>(a, sh, ragged, count, p.R, s);
    return launch_gpl<8, HALP_LOSS_LOGISTIC>(a, sh, ragged, count, p.R, s);
  }
  if (p.loss == HALP_LOSS_SQUARED) return launch_gpl<16, HALP_LOSS_SQUARED>(a, sh, ragged, count, p.R, s);
  return launch_gpl<16, HALP_LOSS_LOGISTIC>(a, sh, ragged, count, p.R, s);
}

}  // namespace halp
