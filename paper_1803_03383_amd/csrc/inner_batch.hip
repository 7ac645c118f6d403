// Inner loop of Algorithm 4 (LM-HALP) with a minibatch of B rows per step (K = 1):
// all rows of a step see the same z, each has its own gamma, z is quantized once per step.
//
// One workgroup per chain, or -- when chains are few -- P workgroups per chain, each holding
// a slice of the coordinates.  The P partial dots of a row then meet in global memory once
// per step: every workgroup publishes its 64 partial sums, each tagged with the step, waits
// (bounded) for the tagged sums of the others, adds them and goes on alone; the update needs
// nothing from the others.
//
// A thread owns the coordinates of one 4/8/16-byte fragment of a row (CPT of them)
// with z, h~ and the window's Philox words in registers.  A step:
//   pass 1   per row: packed integer dot of the fragment with z (v_dot4 at 8 bits; at 16
//            bits v_dot2 against a low and a high part of z separately, so that
//            32-bit sums stay exact), eight wave sums at a time, one LDS slot per row | barrier
//   scalars  wave 0, one row per lane: D_m (with the other workgroups' shares), beta_m,
//            gamma_m = Q_(delta_s,b)(beta_m) into LDS                               | barrier
//   pass 2   per row: sum_m gamma_m x_m accumulated per coordinate (gamma split into its
//            low and high byte at 16 bits), then the rounding of z
// Wave 0 also draws the indices two steps ahead and gathers the margins and labels of the
// next step's rows.  The barriers wait for LDS only, loads stay in flight across them.
//
// Chunked form: the waves of a workgroup sit side by side along the row.  The B rows of a
// step (512 KB at B = 64, d = 4096, b = 16: a CU's register file) cannot stay on chip, so
// they travel twice, in chunks of 8 through two register buffers: from HBM for the dots,
// from L2 for the update.  Full-step form: see the kernel template below.
#include "halp_device.hpp"
#include "inner_args.hpp"

namespace halp {
namespace {

constexpr int kMaxB = 64;   // rows per step: one per service lane
constexpr int kChunk = 8;   // rows in flight per worker thread
constexpr int kMaxParts = kBatchMaxParts;
constexpr int kRowsPerWave = 16;    // full-step form: rows of a step one wave takes at most

typedef short short2v __attribute__((ext_vector_type(2)));

// workgroup barrier that waits for this wave's LDS traffic only: global loads may stay in
// flight across it (their registers are waited for where they are used)
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ int mad24(int a, int b, int c) {
  int r;
  asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Sums of 8 values over the 64 lanes of a wave at once: v[m] is this lane's share of sum m.
// Three exchange steps inside each group of 8 lanes (partner lane ^ 7, ^ 2, ^ 1) halve the
// number of values a lane carries while doubling the lanes each covers, leaving lane l with
// sum l % 8 over its group; three more (lane ^ 8, ^ 16, ^ 32) add the groups.  Every lane
// returns the complete sum number l % 8.  Integer sums: the order does not matter.
__device__ __forceinline__ int wave_sums8_i32(const int (&v)[8], int lane) {
  const bool f2 = (lane & 4) != 0, f1 = (lane & 2) != 0, f0 = (lane & 1) != 0;
  int w[4], u[2];
#pragma unroll
  for (int m = 0; m < 4; ++m) w[m] = (f2 ? v[m + 4] : v[m]) + dpp_half_mirror(f2 ? v[m] : v[m + 4]);
#pragma unroll
  for (int m = 0; m < 2; ++m) u[m] = (f1 ? w[m + 2] : w[m]) + dpp_quad_swap2(f1 ? w[m] : w[m + 2]);
  int r = (f0 ? u[1] : u[0]) + dpp_quad_swap1(f0 ? u[0] : u[1]);
  r += __builtin_amdgcn_update_dpp(0, r, 0x128, 0xF, 0xF, false);  // row_ror:8 = lane ^ 8
  r += __builtin_amdgcn_ds_swizzle(r, 0x401F);                      // lane ^ 16
  r += __shfl_xor(r, 32);
  return r;
}

__device__ __forceinline__ double logistic_dl(double a, double y) {
  return __ddiv_rn(-y, __dadd_rn(1.0, halp_exp(__dmul_rn(y, a))));
}

// NDW: dwords of a row per thread; KT: most waves of the workgroup.
// FS, the full-step form: a workgroup holds ONE slice of 64 NDW dwords of the row, and its
// nwk waves of z all hold that same slice and split the ROWS of the step between them (16
// each at most).  A wave keeps its rows' fragments in registers, loaded a whole step ahead, so
// the rows are read from memory once and a wave's per-row work covers a quarter of the batch.
// The price: the waves add up their sums over rows through LDS before the update, which each
// of them then performs on its own copy of z (same inputs, same result).
template <int BITS, int NDW, int KT, bool FS>
__global__ __launch_bounds__(64 * KT) void inner_batch_kernel(InArgs a, int nwk, int P, long long* xbuf,
                                                              int spin_limit, int poll_delay) {
  using XT = typename std::conditional<BITS == 8, int8_t, int16_t>::type;
  using HT = typename std::conditional<BITS == 8, int16_t, int32_t>::type;
  constexpr int EPD = 32 / BITS;       // elements per dword
  constexpr int CPT = NDW * EPD;       // coordinates per thread
  constexpr int CT = 16 / BITS;        // coordinates per strip of 16 rounding bits
  constexpr int UPL = CPT / CT;        // strips per thread (= 2 NDW)
  constexpr int QMAX = (1 << (BITS - 1)) - 1, QMIN = -(1 << (BITS - 1));
  const int chain = (int)blockIdx.x / P;         // P workgroups per chain, nwk waves of z each
  const int part = (int)blockIdx.x - chain * P;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int d = a.d, B = a.B;
  const int64_t T = epoch_steps(a.seed + (uint64_t)chain, a.epoch, a.T, a.option2);
  const int64_t row_bytes = a.ldxq * (BITS / 8);
  const unsigned char* __restrict__ Xq = reinterpret_cast<const unsigned char*>(a.Xq) +
                                         (int64_t)chain * a.xq_chain_stride * (BITS / 8);
  const double* sc = a.scales + (int64_t)chain * 8;
  uint64_t* cnt_out = a.counters + (int64_t)chain * 4;
  const uint64_t seed = a.seed + (uint64_t)chain;

  if (sc[7] != 0.0) {
    if (tid < 4) cnt_out[tid] = 0;
    return;
  }
  // polls of the other workgroups' sums before a wait is given up for good; below 0: never wait
  unsigned int n_timeout = spin_limit < 0 ? 1u : 0u;
  constexpr int kWarm = 8;   // cache lines of the widest slice (64 threads of 16 bytes)
  uint32_t warm[kWarm] = {};  // full-step form: what wave 0 reads to warm the caches, never used

  __shared__ int s_idx[4][kMaxB];            // sampled rows of steps t .. t+2, slot = step % 4
  __shared__ int s_part[2][16][kMaxB];       // per wave and row: low / high partial dot
  __shared__ int s_gam[kMaxB];               // gamma_m
  __shared__ int s_acc[FS ? 4 : 1][FS ? 2 * CPT : 1][64];  // full-step form: the waves' sums over their rows
  __shared__ int s_cl;                       // c_lambda of the step
  __shared__ uint32_t s_rw[2][kMaxB];        // full-step form: rounding words of gamma_m and the L2
  __shared__ int s_cln[2];                   // draw of the next step, made by wave 1 for wave 0
  __shared__ unsigned long long s_cnt[3];
  if (tid < 3) s_cnt[tid] = 0;
  const bool use_reg = a.lambda > 0;
  const bool lp = a.lp != 0;

  // ---- scalar duties (one row of the step per lane): wave 0, beside its share of z.  (A wave
  // of its own for them would put two waves on one SIMD and halve every wave's registers.)
  const bool svc = wave == 0;
  const int wv = wave;        // this wave's place among the nwk waves that hold z
  const bool worker = true;
  // Full-step form with more than one wave: what can be drawn ahead (the next step's rounding
  // words, the indices two steps ahead) is drawn by wave 1 while wave 0 runs the scalar stage.
  const bool helper = FS && nwk > 1 && wave == 1;
  const bool self_prepare = !(FS && nwk > 1);
  const uint32_t N = (uint32_t)a.N;
  const float* __restrict__ phi = a.phi + (int64_t)chain * a.N;
  const float* __restrict__ y = reinterpret_cast<const float*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const double inv_s = sc[5];
  const double dscale = __dmul_rn(a.delta_d, sc[0]);
  const double alpha = a.hyper[2 * chain];
  const double aB = __ddiv_rn(alpha, (double)B);
  const double al = __dmul_rn(alpha, a.lambda);
  const bool row = lane < B;
  const bool need_phi = a.loss != HALP_LOSS_SQUARED || lp;
  unsigned int n_gclamp = 0, n_reg = 0;
  auto draw_idx = [&](int64_t t) {  // row `lane` of step t (any t names a valid row)
    const uint64_t n = (uint64_t)t * (uint64_t)B + (uint64_t)min(lane, B - 1);
    const U4 r = stream_block(seed, kIdx, a.epoch, n >> 2);
    return (int)__umulhi(pick(r, (uint32_t)(n & 3)), N);
  };
  float phi_c = 0.f, y_c = 0.f;
  int i_next = 0;
  // A chain cut across workgroups: every workgroup evaluates all scalars of a step, but only
  // part 0 gathers the margins and labels of the sampled rows (a 128-byte line per 4-byte
  // value and workgroup otherwise).  It does so a step before it needs them and ships them with
  // the sums of the step in between, as two more tagged words per row.
  const bool shipper = P > 1 && part == 0;
  const bool receiver = P > 1 && part != 0;
  float phi_g = 0.f, y_g = 0.f;  // part 0: margins and labels gathered for the step after this one
  if (svc) {
    const int i0 = draw_idx(0), i1 = draw_idx(1);
    if (row) { s_idx[0][lane] = i0; s_idx[1][lane] = i1; }
    phi_c = need_phi ? phi[i0] : 0.f;
    y_c = a.loss == HALP_LOSS_LOGISTIC ? y[i0] : 0.f;
    i_next = i1;
    if (shipper) {
      phi_g = need_phi ? phi[i1] : 0.f;
      y_g = a.loss == HALP_LOSS_LOGISTIC ? y[i1] : 0.f;
    }
  }
  {
    // ========================================================================= worker
    const HT* __restrict__ hg = reinterpret_cast<const HT*>(a.h) + (int64_t)chain * d;
    XT* __restrict__ zg = reinterpret_cast<XT*>(a.z) + (int64_t)chain * d;
    float* __restrict__ wg = a.w + (int64_t)chain * d;
    // chunked form: the waves of a workgroup (and the workgroups of a chain) hold consecutive
    // slices; full-step form: one slice per workgroup, the same in all its waves
    const int j0 = !worker ? d : (FS ? (part * 64 + lane) * CPT : (part * 64 * nwk + wv * 64 + lane) * CPT);
    // full-step form: the rows of a step are dealt to the waves in runs of 8 or 16
    const int rpw = FS ? 8 * ((((B + nwk - 1) / nwk) + 7) / 8) : 0;
    const int row0 = FS && worker ? wv * rpw : 0;
    const bool active = j0 < d;
    // Rows are padded to whole 8-byte groups; a 16-byte fragment is only used when rows are
    // 16-byte multiples (checked on the host), so a fragment that starts below d lies inside
    // the row.  Threads past the row re-read its first fragment; their z stays 0.
    const int frag_off = active ? j0 * (BITS / 8) : 0;
    int z[CPT], hv[CPT];
    bool ok[CPT];
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      ok[k] = j0 + k < d;
      const int j = min(j0 + k, d - 1);
      z[k] = ok[k] ? (int)zg[j] : 0;
      hv[k] = ok[k] ? (int)hg[j] : 0;
    }
    const uint32_t strip0 = (uint32_t)(j0 / CT);
    // At 8 strips per thread the window's 8 Philox blocks (32 registers) are parked in LDS
    // as [word][strips 0..3 | 4..7][thread] of 16 bytes (a wave reads consecutive addresses;
    // a thread reads only what it wrote) and the words of two steps are fetched at a time.
    constexpr bool kPark = UPL == 8;
    extern __shared__ __attribute__((aligned(16))) uint4 s_zr[];
    const int nworkers = 64 * nwk;      // threads that hold z
    const int wtid = wv * 64 + lane;    // this thread's place among them
    U4 zr[kPark ? 1 : UPL];
    uint32_t zw[kPark ? UPL : 1];
    unsigned long long n_zclamp = 0;
    auto load_frag = [&](uint32_t (&dst)[NDW], int i) {
      const unsigned char* rp = Xq + (int64_t)i * row_bytes + frag_off;
      if (NDW == 1) {
        dst[0] = *reinterpret_cast<const uint32_t*>(rp);
      } else if (NDW == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(rp);
        dst[0] = v.x; dst[NDW > 1 ? 1 : 0] = v.y;
      } else {
        const uint4 v = *reinterpret_cast<const uint4*>(rp);
        dst[0] = v.x; dst[NDW > 1 ? 1 : 0] = v.y; dst[NDW > 2 ? 2 : 0] = v.z; dst[NDW > 3 ? 3 : 0] = v.w;
      }
    };
    uint32_t xa[kChunk][NDW], xb[kChunk][NDW];
    auto load_chunk = [&](uint32_t (&dst)[kChunk][NDW], const int* idx, int m0) {
      const int mine = idx[min(m0 + (lane & (kChunk - 1)), B - 1)];  // lane r: row m0 + r, one LDS read
#pragma unroll
      for (int r = 0; r < kChunk; ++r)  // the row number is uniform: scalar address arithmetic
        load_frag(dst[r], __builtin_amdgcn_readlane(mine, r));
    };
    // FS: the fragments of all rows of this step and of the next one
    constexpr int RPW = FS ? kRowsPerWave : 1;
    // Full-step form with fragments of at most 8 bytes: three register sets, the rows of a step
    // are requested two steps before their dots (a step ahead is less than a trip to memory for
    // a random row, and a workgroup whose rows are late makes every workgroup of the chain wait)
    constexpr bool kDeep = FS && NDW <= 2;
    uint32_t xc[RPW][NDW], xn[RPW][NDW], xf[kDeep ? RPW : 1][NDW];
    auto load_step = [&](uint32_t (&dst)[RPW][NDW], const int* idx) {
      // lane r fetches the index of the wave's row r (one LDS read for all); rows past B
      // repeat the last one and are not used
      const int mine = idx[min(row0 + (lane & (RPW - 1)), B - 1)];
#pragma unroll
      for (int r = 0; r < RPW; ++r) load_frag(dst[r], __builtin_amdgcn_readlane(mine, r));
    };
    __syncthreads();
    if (FS) {
      if (worker) load_step(xc, s_idx[0]);
      if (kDeep && worker) load_step(xn, s_idx[1]);
    } else {
      load_chunk(xa, s_idx[0], 0);
    }

    // wave 0: the rounding word of gamma_m and the L2 draw of a step, made a step ahead
    uint32_t rw_next = 0;
    int cl_next = 0;
    auto draw_scalars = [&](int64_t tn) {
      const uint64_t n = (uint64_t)tn * (uint64_t)B + (uint64_t)min(lane, B - 1);
      rw_next = pick(stream_block(seed, kGamma, a.epoch, n >> 2), (uint32_t)(n & 3));
      cl_next = 0;
      if (use_reg) {
        const uint32_t rr = pick(stream_block(seed, kReg, a.epoch, (uint64_t)tn >> 2), (uint32_t)(tn & 3));
        cl_next = (int)quantize_real(al, (double)(1 << BITS), rr, 0.0, (double)QMAX, nullptr);
      }
    };
    if (svc) draw_scalars(0);

    auto one_step = [&](int64_t t, uint32_t (&cur)[RPW][NDW], uint32_t (&nxt)[RPW][NDW]) {
      const int* idx = s_idx[t & 3];
      // wave 0: what the scalar stage needs and does not depend on the dots — margins and
      // labels of the next step's rows (used after the next barrier pair), the rounding word
      // of gamma_m, the L2 draw
      float phi_n = 0.f, y_n = 0.f;
      uint32_t rw = 0;
      int cl_draw = 0;
      if (svc) {
        if (P == 1) {
          const int inx = self_prepare ? i_next : s_idx[(t + 1) & 3][min(lane, B - 1)];
          phi_n = need_phi ? phi[inx] : 0.f;
          y_n = a.loss == HALP_LOSS_LOGISTIC ? y[inx] : 0.f;
        } else if (shipper) {  // gathered after the last step's gamma (before the loop for step 0)
          phi_n = phi_g;
          y_n = y_g;
        }  // the other parts receive them with the sums below
        if (self_prepare || t == 0) {  // drawn during the previous step (or before the first)
          rw = rw_next;
          cl_draw = cl_next;
        } else {
          rw = s_rw[t & 1][lane];
          cl_draw = s_cln[t & 1];
        }
        n_reg += (lane == 0 && cl_draw != 0) ? 1u : 0u;
      }
      // What wave 0 prepares for later steps: with several workgroups per chain it runs while
      // the wave waits for the others' sums, else here, while the other waves take the dots.
      auto prepare_ahead = [&]() {
        draw_scalars(t + 1);
        if (FS) {  // the indices two steps ahead (slot (t + 2) % 4 was last read in step t - 2)
          const int i2 = draw_idx(t + 2);
          if (row) s_idx[(t + 2) & 3][lane] = i2;
          i_next = i2;
          // Touch this workgroup's slice of those rows, one row per lane and one load per
          // cache line: the address translations and the lines are on their way into L2 a step
          // before the other waves ask for them.  The values are not used (taken up a step
          // later, so that nothing here waits for them).
#pragma unroll
          for (int k = 0; k < kWarm; ++k) asm volatile("" ::"v"(warm[k]));
          const int64_t part_off = (int64_t)part * 64 * NDW * 4;
          const int slice = (int)min((int64_t)64 * NDW * 4, row_bytes - part_off);
          if (!kDeep && slice >= 4) {  // kDeep: the rows themselves are requested at that distance
            const unsigned char* wp = Xq + (int64_t)i2 * row_bytes + part_off;
#pragma unroll
            for (int k = 0; k < kWarm; ++k)  // unconditional, the last line repeated
              warm[k] = *reinterpret_cast<const uint32_t*>(wp + min(k * 128, slice - 4));
          }
        }
      };
      if (svc && P == 1 && self_prepare) prepare_ahead();
      if (worker && (t & 7) == 0) {
        if (kPark) {
#pragma unroll
          for (int q = 0; q < UPL / 4; ++q) {
            U4 blk[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
              blk[u] = zround_block(seed, a.epoch, strip0 + (uint32_t)(4 * q + u), (uint32_t)(t >> 3));
#pragma unroll
            for (int wd = 0; wd < 4; ++wd)
              s_zr[(wd * (UPL / 4) + q) * nworkers + wtid] =
                  make_uint4(pick(blk[0], wd), pick(blk[1], wd), pick(blk[2], wd), pick(blk[3], wd));
          }
        } else {
#pragma unroll
          for (int u = 0; u < (kPark ? 1 : UPL); ++u)
            zr[u] = zround_block(seed, a.epoch, strip0 + (uint32_t)u, (uint32_t)(t >> 3));
        }
      }
      if (kPark && worker && (t & 1) == 0) {  // the block word that serves steps t and t + 1
#pragma unroll
        for (int q = 0; q < UPL / 4; ++q) {
          const uint4 v = s_zr[(((int)(t & 7) >> 1) * (UPL / 4) + q) * nworkers + wtid];
          zw[(4 * q) % UPL] = v.x; zw[(4 * q + 1) % UPL] = v.y;
          zw[(4 * q + 2) % UPL] = v.z; zw[(4 * q + 3) % UPL] = v.w;
        }
      }
      // z packed for the dots: bytes at 8 bits; low parts and high parts apart at 16 bits
      uint32_t zp[NDW], zq[NDW];
#pragma unroll
      for (int q = 0; q < NDW; ++q) {
        if (BITS == 8) {
          zp[q] = (uint32_t)(z[4 * q] & 0xFF) | ((uint32_t)(z[4 * q + 1] & 0xFF) << 8) |
                  ((uint32_t)(z[4 * q + 2] & 0xFF) << 16) | ((uint32_t)(z[4 * q + 3] & 0xFF) << 24);
          zq[q] = 0;
        } else {
          // z = 256 zh + zl with zl in [-128, 127]: both parts at most 128 in magnitude, so a
          // wave's sum of 512 products with |x| <= 32767 stays below 2^31
          const int za = z[(2 * q) % CPT], zb = z[(2 * q + 1) % CPT];
          const int ha = (za + 128) >> 8, hb = (zb + 128) >> 8;
          const int la = za - 256 * ha, lb = zb - 256 * hb;
          zp[q] = (uint32_t)(la & 0xFFFF) | ((uint32_t)lb << 16);
          zq[q] = (uint32_t)(ha & 0xFFFF) | ((uint32_t)hb << 16);
        }
      }
      // Rows come in chunks of 8 through two register buffers: while one chunk is worked on
      // the next is in flight, across the passes and across the steps (the chunk after the
      // last of pass 1 is the first of pass 2; after pass 2, the first of the next step).
      // ---- pass 1: dots
      auto dots = [&](uint32_t (&xf)[kChunk][NDW], int m0) {
        int lo[kChunk], hi[kChunk];
#pragma unroll
        for (int r = 0; r < kChunk; ++r) {
          lo[r] = hi[r] = 0;
#pragma unroll
          for (int q = 0; q < NDW; ++q) {
            if (BITS == 8) {
              lo[r] = __builtin_amdgcn_sdot4((int)xf[r][q], (int)zp[q], lo[r], false);
            } else {
              const short2v xv = __builtin_bit_cast(short2v, xf[r][q]);
              lo[r] = __builtin_amdgcn_sdot2(xv, __builtin_bit_cast(short2v, zp[q]), lo[r], false);
              hi[r] = __builtin_amdgcn_sdot2(xv, __builtin_bit_cast(short2v, zq[q]), hi[r], false);
            }
          }
        }
        const int slo = wave_sums8_i32(lo, lane);  // row m0 + lane % 8
        const int shi = BITS == 16 ? wave_sums8_i32(hi, lane) : 0;
        if (lane < kChunk && m0 + lane < B) {
          s_part[0][FS ? 0 : wv][m0 + lane] = slo;  // full-step form: one wave per row, one slot
          if (BITS == 16) s_part[1][FS ? 0 : wv][m0 + lane] = shi;
        }
      };
      if constexpr (FS) {
        if (worker) {
#pragma unroll
          for (int c0 = 0; c0 < RPW; c0 += kChunk)
            if (c0 < rpw && row0 + c0 < B) dots(reinterpret_cast<uint32_t(&)[kChunk][NDW]>(cur[c0]), row0 + c0);
        }
      } else {
        for (int m0 = 0; m0 < B; m0 += 2 * kChunk) {
          load_chunk(xb, idx, m0 + kChunk);
          dots(xa, m0);
          load_chunk(xa, idx, m0 + 2 * kChunk < B ? m0 + 2 * kChunk : 0);
          if (m0 + kChunk < B) dots(xb, m0 + kChunk);
        }
      }
      lds_barrier();  // the partial dots of this step are in LDS
      if (helper) {
        prepare_ahead();
        s_rw[(t + 1) & 1][lane] = rw_next;
        if (lane == 0) s_cln[(t + 1) & 1] = cl_next;
      }
      if (svc) {
        // l'(phi_m) does not depend on the dots: evaluated here, ahead of the wait for the other
        // workgroups' sums, so that only l'(phi_m + x_m^T z) follows it
        const double a0 = (double)phi_c, yi = (double)y_c;
        double rho_m = __dmul_rn((double)rw, 0x1p-32);  // the rounding draw of gamma_m
        asm volatile("" : "+v"(rho_m));
        double dl0 = 0.0;
        if (P == 1) {
          if (a.loss == HALP_LOSS_LOGISTIC) dl0 = logistic_dl(a0, yi);
          asm volatile("" : "+v"(dl0));  // stays where it is written
        }
        long long D = 0;
        for (int w2 = 0; w2 < (FS ? 1 : nwk); ++w2) {
          const long long lo = s_part[0][w2][min(lane, B - 1)];
          const long long hi = BITS == 8 ? 0 : s_part[1][w2][min(lane, B - 1)];
          D += lo + hi * 256;
        }
        if (P > 1) {
          // The other workgroups' shares of the dots.  A share travels as one 64-bit word, the
          // sum in its low 46 bits and a tag of the step above them, written and read with
          // device-scope atomics: a word that carries the step's tag is that step's sum, so no
          // fence (and no write-back or invalidation of a whole L2) is needed.  A word is
          // rewritten two steps later, which its writer only reaches after every workgroup of
          // the chain has read it.
          const unsigned long long tag = (unsigned long long)((t >> 1) % 262143) + 1ull;
          unsigned long long* xb = reinterpret_cast<unsigned long long*>(xbuf) +
                                   (((int64_t)chain * 2 + (int64_t)(t & 1)) * kBatchSlots) * kMaxB;
          __hip_atomic_store(&xb[part * kMaxB + lane],
                             (tag << 46) | ((unsigned long long)D & ((1ull << 46) - 1ull)), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
          const bool logistic = a.loss == HALP_LOSS_LOGISTIC;
          if (shipper && need_phi)
            __hip_atomic_store(&xb[kMaxParts * kMaxB + lane], (tag << 46) | (unsigned long long)__float_as_uint(phi_g),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (shipper && logistic)
            __hip_atomic_store(&xb[(kMaxParts + 1) * kMaxB + lane], (tag << 46) | (unsigned long long)__float_as_uint(y_g),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          bool want_phi = receiver && need_phi, want_y = receiver && logistic;
          if (logistic) dl0 = logistic_dl(a0, yi);  // behind the publish, ahead of the wait
          asm volatile("" : "+v"(dl0));
          if (self_prepare) prepare_ahead();
          // A published word needs a trip through device memory before another workgroup can
          // see it, so polls that start at once only add traffic: wait out most of that trip
          // first.  Later rounds ask only for the parts that have not arrived yet.
          if (n_timeout == 0) {
            for (int i = 0; i < poll_delay; ++i) __builtin_amdgcn_s_sleep(4);
          }
          long long tot = D;
          long long val[kMaxParts];
#pragma unroll
          for (int p2 = 0; p2 < kMaxParts; ++p2) val[p2] = 0;
          unsigned long long missing = (1ull << P) - 1ull;  // parts whose 64 words do not all carry the tag yet
          for (int spin = 0; n_timeout == 0; ++spin) {  // after one wait ran out, none is tried again
            unsigned long long wd[kMaxParts];
            // all loads of a round in flight at once; the upper half of the slots only for
            // chains cut into more than eight parts
            auto ask = [&](int lo, int hi) {
#pragma unroll
              for (int p2 = 0; p2 < kMaxParts; ++p2) {
                if (p2 < lo || p2 >= hi) continue;
                wd[p2] = 0;
                if ((missing >> p2) & 1ull)
                  wd[p2] = __hip_atomic_load(&xb[p2 * kMaxB + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              }
            };
            auto take = [&](int lo, int hi) {
#pragma unroll
              for (int p2 = 0; p2 < kMaxParts; ++p2) {
                if (p2 < lo || p2 >= hi) continue;
                if ((missing >> p2) & 1ull) {
                  if (__ballot((wd[p2] >> 46) != tag) == 0) {
                    missing &= ~(1ull << p2);
                    val[p2] = (long long)(wd[p2] << 18) >> 18;
                  }
                }
              }
            };
            ask(0, 8);
            if (P > 8) ask(8, kMaxParts);
            unsigned long long wphi = 0, wy = 0;
            if (want_phi)
              wphi = __hip_atomic_load(&xb[kMaxParts * kMaxB + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (want_y)
              wy = __hip_atomic_load(&xb[(kMaxParts + 1) * kMaxB + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            take(0, 8);
            if (P > 8) take(8, kMaxParts);
            if (want_phi && __ballot((wphi >> 46) != tag) == 0) {
              want_phi = false;
              phi_n = __uint_as_float((uint32_t)wphi);
            }
            if (want_y && __ballot((wy >> 46) != tag) == 0) {
              want_y = false;
              y_n = __uint_as_float((uint32_t)wy);
            }
            if (missing == 0 && !want_phi && !want_y) break;
            if (spin >= spin_limit) {  // only if a workgroup of the chain never ran: give up
              n_timeout = 1;
              break;
            }
            __builtin_amdgcn_s_sleep(1);
          }
          if (n_timeout == 0) {
            tot = 0;
#pragma unroll
            for (int p2 = 0; p2 < kMaxParts; ++p2) tot += val[p2];
          }
          D = tot;
        }
        // beta_m = (alpha / B) (l'(phi_m + x_m^T z) - l'(phi_m)), gamma_m = Q_(delta_s, b)(beta_m)
        const double delta = __dmul_rn(dscale, (double)D);
        double diff;
        if (a.loss == HALP_LOSS_LOGISTIC) {
          const double a1 = lp ? delta : __dadd_rn(a0, delta);
          diff = __dadd_rn(logistic_dl(a1, yi), -dl0);
        } else {
          diff = lp ? __dadd_rn(delta, -a0) : delta;
        }
        const double beta = __dmul_rn(aB, diff);
        // gamma_m = Q_(delta_s, b)(beta_m): floor(beta / delta_s + rho), clamped -- the quantizer of
        // quantize_real with its draw converted ahead of the wait and the result taken as a
        // 32-bit integer (it lies in the box after the clamp)
        const double fq = floor(__dadd_rn(__dmul_rn(beta, inv_s), rho_m));
        const double fc = fmin(fmax(fq, (double)QMIN), (double)QMAX);
        const bool hit = fq != fc;
        const int gq = (int)fc;
        if (row) {
          s_gam[lane] = gq;
          n_gclamp += hit ? 1u : 0u;
        }
        if (lane == 0) s_cl = cl_draw;
        if (!FS) {  // indices two steps ahead (slot (t + 2) % 4 was last read in step t - 2)
          const int i2 = draw_idx(t + 2);
          if (row) s_idx[(t + 2) & 3][lane] = i2;
          i_next = i2;
        }
        phi_c = phi_n; y_c = y_n;
      }
      lds_barrier();  // gamma is out
      if (svc && shipper) {  // margins and labels of the rows two steps on, shipped with the next step's sums
        const int i2 = self_prepare ? i_next : s_idx[(t + 2) & 3][min(lane, B - 1)];
        phi_g = need_phi ? phi[i2] : 0.f;
        y_g = a.loss == HALP_LOSS_LOGISTIC ? y[i2] : 0.f;
      }
      // Full-step form: this wave's rows of the next step, requested only now -- what wave 0
      // read from memory for the scalar stage (margins, the other workgroups' sums) must not
      // queue behind them -- and in flight through the update and the next step's start.
      if (FS) load_step(nxt, s_idx[(t + (kDeep ? 2 : 1)) & 3]);  // kDeep: `nxt` is the set two steps on
      // ---- pass 2: sum_m gamma_m x_m per coordinate (low / high byte of gamma apart at 16 bits)
      int acc[CPT], acch[CPT];
#pragma unroll
      for (int k = 0; k < CPT; ++k) acc[k] = acch[k] = 0;
      auto accumulate = [&](uint32_t (&xf)[kChunk][NDW], int m0) {
        int gm[kChunk];
        const int gmine = s_gam[min(m0 + (lane & (kChunk - 1)), kMaxB - 1)];  // lane r: row m0 + r
#pragma unroll
        for (int r = 0; r < kChunk; ++r) gm[r] = m0 + r < B ? __builtin_amdgcn_readlane(gmine, r) : 0;
        if (BITS == 16) {
          // Two rows at a time: v_perm puts coordinate j of both rows into one register, one
          // v_dot2 against the pair of gammas then serves both rows.  gamma = 256 gh + gl with
          // gl in [0, 255]: 64 products of each part stay below 2^31.
#pragma unroll
          for (int r = 0; r < kChunk; r += 2) {
            const uint32_t glp = (uint32_t)(gm[r] & 0xFF) | ((uint32_t)(gm[r + 1] & 0xFF) << 16);
            const uint32_t ghp = (uint32_t)((gm[r] >> 8) & 0xFFFF) | ((uint32_t)(gm[r + 1] >> 8) << 16);
            const short2v gl2 = __builtin_bit_cast(short2v, glp), gh2 = __builtin_bit_cast(short2v, ghp);
#pragma unroll
            for (int q = 0; q < NDW; ++q) {
              const uint32_t xr0 = xf[r][q], xr1 = xf[r + 1][q];
              // (row r, row r + 1) of the even and of the odd coordinate of this dword
              const short2v pe = __builtin_bit_cast(short2v, __builtin_amdgcn_perm(xr1, xr0, 0x05040100u));
              const short2v po = __builtin_bit_cast(short2v, __builtin_amdgcn_perm(xr1, xr0, 0x07060302u));
              acc[(2 * q) % CPT] = __builtin_amdgcn_sdot2(pe, gl2, acc[(2 * q) % CPT], false);
              acch[(2 * q) % CPT] = __builtin_amdgcn_sdot2(pe, gh2, acch[(2 * q) % CPT], false);
              acc[(2 * q + 1) % CPT] = __builtin_amdgcn_sdot2(po, gl2, acc[(2 * q + 1) % CPT], false);
              acch[(2 * q + 1) % CPT] = __builtin_amdgcn_sdot2(po, gh2, acch[(2 * q + 1) % CPT], false);
            }
          }
        } else {
#pragma unroll
          for (int r = 0; r < kChunk; ++r) {
#pragma unroll
            for (int k = 0; k < CPT; ++k) {
              const uint32_t xv = xf[r][k / EPD];
              const int x = (int)(int8_t)(xv >> ((k % EPD) * 8));
              acc[k] = mad24(gm[r], x, acc[k]);
            }
          }
        }
      };
      if constexpr (FS) {
        if (worker) {
#pragma unroll
          for (int c0 = 0; c0 < RPW; c0 += kChunk)
            if (c0 < rpw && row0 + c0 < B)
              accumulate(reinterpret_cast<uint32_t(&)[kChunk][NDW]>(cur[c0]), row0 + c0);
          // this wave's sums over its rows, for the other waves
#pragma unroll
          for (int k = 0; k < CPT; ++k) {
            s_acc[wv][k][lane] = acc[k];
            if (BITS == 16) s_acc[wv][CPT + k][lane] = acch[k];
          }
        }
        lds_barrier();  // every wave's sums are in LDS
        if (worker) {
#pragma unroll
          for (int k = 0; k < CPT; ++k) {
            int pa[4], ph[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {  // every group's slot is read (unused ones hold old sums)
              pa[g] = s_acc[g][k][lane];
              ph[g] = BITS == 16 ? s_acc[g][CPT + k][lane] : 0;
            }
            acc[k] = 0;
            acch[k] = 0;
#pragma unroll
            for (int g = 0; g < 4; ++g) {  // the same order in every wave
              if (g < nwk) {
                acc[k] += pa[g];
                acch[k] += ph[g];
              }
            }
          }
        }
      } else {
        const int* idn = s_idx[(t + 1) & 3];
        for (int m0 = 0; m0 < B; m0 += 2 * kChunk) {
          load_chunk(xb, idx, m0 + kChunk);
          accumulate(xa, m0);
          if (m0 + 2 * kChunk < B) load_chunk(xa, idx, m0 + 2 * kChunk);
          else load_chunk(xa, idn, 0);
          accumulate(xb, m0 + kChunk);
        }
      }
      // ---- u = z - sum gamma x - h~ - c_lambda z in (delta_i, 2b); z = Q_(delta_m, b)(u)
      const int cl = use_reg ? s_cl : 0;
#pragma unroll
      for (int k = 0; k < CPT; ++k) {
        // the strip's 16-bit field of this step: half (t % 2) of word (t % 8) / 2 of its block
        const uint32_t field = kPark ? (zw[(k / CT) % (kPark ? UPL : 1)] >> (16u * (uint32_t)(t & 1))) & 0xFFFFu
                                     : zround_field(zr[kPark ? 0 : k / CT], (uint32_t)t);
        const long long re = (long long)((field >> ((k % CT) * BITS)) & ((1u << BITS) - 1u));
        const long long gsum = (long long)acc[k] + (BITS == 16 ? (long long)acch[k] * 256 : 0);
        const long long v = -(long long)hv[k] - (long long)cl * (long long)z[k] - gsum;
        const long long zu = (long long)z[k] + ((v + re) >> BITS);
        const long long zc = zu > QMAX ? QMAX : (zu < QMIN ? QMIN : zu);
        n_zclamp += (ok[k] && zu != zc && (!FS || wv == 0)) ? 1u : 0u;  // the copies of z count once
        z[k] = ok[k] ? (int)zc : 0;
      }
    };
    if constexpr (kDeep) {  // three register sets in rotation: rows of steps t, t + 1 and the set being filled
      auto& x0 = xc;
      auto& x1 = xn;
      auto& x2 = reinterpret_cast<uint32_t(&)[RPW][NDW]>(xf);
      int64_t t = 0;
      for (; t + 2 < T; t += 3) {
        one_step(t, x0, x2);
        one_step(t + 1, x1, x0);
        one_step(t + 2, x2, x1);
      }
      if (t < T) one_step(t, x0, x2);
      if (t + 1 < T) one_step(t + 1, x1, x0);
    } else if (FS) {  // the two register sets trade places from step to step
      int64_t t = 0;
      for (; t + 1 < T; t += 2) {
        one_step(t, xc, xn);
        one_step(t + 1, xn, xc);
      }
      if (t < T) one_step(t, xc, xn);
    } else {
      for (int64_t t = 0; t < T; ++t) one_step(t, xc, xn);
    }

    // ---- w~ <- w~ + delta_m z (option I; Algorithm 2: w~ = delta z); hand z out
    const double delta_m = sc[0];
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      if (ok[k] && (!FS || wv == 0)) {
        const int j = j0 + k;
        zg[j] = (XT)z[k];
        if (P == 1) {  // several workgroups per chain: batch_split_finish applies the offset
          const double step = __dmul_rn(delta_m, (double)z[k]);
          wg[j] = lp ? (float)step : (float)__dadd_rn((double)wg[j], step);
        }
      }
    }
    if (n_zclamp) atomicAdd(&s_cnt[0], n_zclamp);
    if (n_gclamp) atomicAdd(&s_cnt[1], (unsigned long long)n_gclamp);
    if (n_reg) atomicAdd(&s_cnt[2], (unsigned long long)n_reg);
  }
  __syncthreads();
  if (P == 1) {
    if (tid < 4) cnt_out[tid] = tid < 3 ? s_cnt[tid] : 0ull;
  } else {
    // counters were cleared before the launch: clamped coordinates add up over the parts, the
    // scalar counts are the same in every part, a timed-out wait is flagged in the last word
    if (tid == 0 && s_cnt[0]) atomicAdd(reinterpret_cast<unsigned long long*>(&cnt_out[0]), s_cnt[0]);
    if (part == 0 && (tid == 1 || tid == 2)) cnt_out[tid] = s_cnt[tid];
    if (tid == 0 && n_timeout) atomicMax(reinterpret_cast<unsigned long long*>(&cnt_out[3]), 1ull);
  }
}

// Several workgroups per chain: w~ <- w~ + delta_m z is applied here, after the launch, and only
// for chains none of whose workgroups gave up a wait.  A chain with a wait that ran out keeps
// its w~ (its z is then not a trajectory of the method) and gets status -2 in scales[7].
template <int BITS>
__global__ __launch_bounds__(256) void batch_split_finish(InArgs a, double* scales) {
  using XT = typename std::conditional<BITS == 8, int8_t, int16_t>::type;
  const int chain = blockIdx.y;
  const int j = (int)(blockIdx.x * 256 + threadIdx.x);
  double* sc = scales + (int64_t)chain * 8;
  if (a.counters[(int64_t)chain * 4 + 3] != 0) {
    if (j == 0) sc[7] = -2.0;
    return;
  }
  if (sc[7] != 0.0 || j >= a.d) return;  // a gradient of zero or not finite: the loop did not run
  const XT* zg = reinterpret_cast<const XT*>(a.z) + (int64_t)chain * a.d;
  float* wg = a.w + (int64_t)chain * a.d;
  const double step = __dmul_rn(sc[0], (double)zg[j]);
  wg[j] = a.lp ? (float)step : (float)__dadd_rn((double)wg[j], step);
}

// clears what the split launch accumulates into or waits on
__global__ void batch_split_prepare(long long* xbuf, int nwords, uint64_t* counters, int ncounters) {
  const int k = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (k < nwords) xbuf[k] = 0;
  if (k < ncounters) counters[k] = 0;
}

template <int BITS, int NDW, int KT, bool FS>
int launch_kt(const InArgs& a, int nwk, int P, long long* xbuf, int spin_limit, int poll_delay, dim3 grid, dim3 block,
              size_t smem, hipStream_t s) {
  auto kern = inner_batch_kernel<BITS, NDW, KT, FS>;
  if (smem > 0 && hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                      hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)smem) != hipSuccess)
    return HALP_ERR_HIP;
  hipLaunchKernelGGL(kern, grid, block, smem, s, a, nwk, P, xbuf, spin_limit, poll_delay);
  return hip_ok(hipGetLastError());
}

struct BtShape {
  int ndw, nwk;
};

// dwords per thread and worker waves: the widest fragment the row alignment allows that
// still gives every SIMD a wave, at most 15 worker waves
BtShape pick_shape(const halp_params& p, int64_t row_bytes) {
  const int epd = 32 / p.b;
  int ndw = row_bytes % 16 == 0 ? 4 : 2;
  while (ndw > 1 && (p.d + 64 * ndw * epd - 1) / (64 * ndw * epd) < 4) ndw /= 2;
  int nwk = (p.d + 64 * ndw * epd - 1) / (64 * ndw * epd);
  while (nwk > 16 && ndw < (row_bytes % 16 == 0 ? 4 : 2)) {
    ndw *= 2;
    nwk = (p.d + 64 * ndw * epd - 1) / (64 * ndw * epd);
  }
  return BtShape{ndw, nwk};
}

}  // namespace

// K = 1, 2 <= B <= 64, squared or logistic loss, up to 16 waves of 16-byte fragments
int inner_batch_supported(const halp_handle& h) {
  const halp_params& p = h.p;
  if (p.K != 1 || p.B < 2 || p.B > kMaxB) return HALP_ERR_UNSUPPORTED;
  if (p.loss != HALP_LOSS_SQUARED && p.loss != HALP_LOSS_LOGISTIC) return HALP_ERR_UNSUPPORTED;
  if (p.b == 8 && p.d > 131071) return HALP_ERR_UNSUPPORTED;  // int32 dots stay exact
  if (!h.bound || !h.buf.Xq) return HALP_ERR_NOT_BOUND;
  const int64_t row_bytes = h.buf.ldxq * (p.b / 8);
  const BtShape sh = pick_shape(p, row_bytes);
  if (sh.nwk > 16) return HALP_ERR_UNSUPPORTED;
  // every fragment that starts below d must lie inside the row
  const int cpt = sh.ndw * 32 / p.b;
  if ((int64_t)((p.d + cpt - 1) / cpt) * sh.ndw * 4 > row_bytes) return HALP_ERR_UNSUPPORTED;
  if (sh.ndw == 4 && reinterpret_cast<uintptr_t>(h.buf.Xq) % 16 != 0) return HALP_ERR_UNSUPPORTED;
  return HALP_OK;
}

// Launch shape.  Full-step form (one slice of the row per workgroup, the rows of a step dealt
// to its waves and kept in registers): taken by default whenever the slices of a row are few
// enough for one workgroup each.  Otherwise, and whenever HALP_OPT_INNER_PARTS names a count,
// the chunked form with that many workgroups per chain.  Workgroups of a chain wait for each
// other, so there are only as many as are surely resident at once (at most one per CU).
struct BtLaunch {
  bool fs;
  int ndw, nwk, P;  // nwk: waves of z per workgroup
};

static BtLaunch pick_launch(const halp_handle& h, int64_t row_bytes) {
  const halp_params& p = h.p;
  const BtShape sh = pick_shape(p, row_bytes);
  int most = 1;
  if (h.batch_xbuf) {
    most = kBatchMaxParts;
    while (most > 1 && (int64_t)p.R * most > h.num_cus) most /= 2;
  }
  int most_any = 1;  // any count up to the exchange buffer's slots
  if (h.batch_xbuf) {
    most_any = (int)(h.num_cus / p.R);
    if (most_any > kBatchMaxParts) most_any = kBatchMaxParts;
    if (most_any < 1) most_any = 1;
  }
  if (h.inner_parts == 0) {
    // full-step form: the widest fragment the alignment allows whose slices (one workgroup
    // each) are few enough to be resident together; up to 4 waves share the rows of a step
    const int epd = 32 / p.b;
    const bool al16 = row_bytes % 16 == 0 && reinterpret_cast<uintptr_t>(h.buf.Xq) % 16 == 0;
    const int ndw_max = (al16 && p.b == 16) ? 4 : 2;  // 8 coordinates per thread at most
    auto fits = [&](int ndw, int& P) {
      const int cpt = ndw * epd;
      P = (p.d + 64 * cpt - 1) / (64 * cpt);
      if (P > most_any) return false;
      // several workgroups pay ~2 us per step for their exchange.  Measured: worth it down to
      // steps of 16 KB of rows (3.3 - 4.6 us split against 3.9 - 5.2 on one workgroup; at 64 - 128 KB
      // 3.9 - 4.9 against 9.6 - 11.3)
      if (P > 1 && (int64_t)p.B * row_bytes < 16 * 1024) return false;
      return (int64_t)((p.d + cpt - 1) / cpt) * ndw * 4 <= row_bytes;  // fragments inside the row
    };
    int rg = (p.B + 7) / 8;
    if (rg > 4) rg = 4;
    // A chain cut across workgroups: the narrowest fragment of at least four coordinates whose
    // slices are few enough -- more, narrower slices shorten both passes over the rows of a step
    // (measured: 4096 x 16 bits 6.6 us with 8 slices, 6.2 with 16; 2048 x 16 bits 5.8 / 4.9 with
    // 4 / 8; 4096 x 8 bits 5.4 / 5.2 with 8 / 16; two coordinates per thread lose again).
    for (int ndw = p.b == 16 ? 2 : 1; ndw <= ndw_max; ndw *= 2) {
      int P;
      if (fits(ndw, P) && P > 1) return BtLaunch{true, ndw, rg, P};
    }
    for (int ndw = ndw_max; ndw >= 1; ndw /= 2) {
      int P;
      if (fits(ndw, P)) return BtLaunch{true, ndw, rg, P};
    }
  }
  int P = 1;
  if (h.inner_parts > 0) {
    while (most > sh.nwk) most /= 2;
    P = h.inner_parts < most ? h.inner_parts : (most < 1 ? 1 : most);
  }
  return BtLaunch{false, sh.ndw, (sh.nwk + P - 1) / P, P};
}

int launch_inner_batch(const halp_handle& h, uint32_t epoch, hipStream_t s) {
  const halp_params& p = h.p;
  const int rc = inner_batch_supported(h);
  if (rc != HALP_OK) return rc;
  const InArgs a = make_inner_args(h, epoch);
  const BtLaunch L = pick_launch(h, h.buf.ldxq * (p.b / 8));
  const int nwk = L.nwk, P = L.P;
  const int nwaves = nwk;
  const dim3 grid(p.R * P), block(64 * nwaves);
  if (P > 1) {
    const int nwords = p.R * 2 * kBatchSlots * kMaxB, ncnt = p.R * 4;
    hipLaunchKernelGGL(batch_split_prepare, dim3((nwords + 255) / 256), dim3(256), 0, s, h.batch_xbuf, nwords,
                       h.buf.counters, ncnt);
  }
  // parked Philox blocks: 128 bytes per worker thread at 8 strips per thread (120 KB at most)
  const size_t smem = L.ndw == 4 ? (size_t)64 * nwk * 128 : 0;
#define HALP_BT(BITS_, NDW_, FS_)                                                                  \
  if (p.b == BITS_ && L.ndw == NDW_ && L.fs == FS_) {                                              \
    if (nwaves <= 4)                                                                               \
      return launch_kt<BITS_, NDW_, 4, FS_>(a, nwk, P, h.batch_xbuf, h.spin_limit, h.poll_delay, grid, block, smem, s);         \
    if (nwaves <= 8)                                                                               \
      return launch_kt<BITS_, NDW_, 8, FS_>(a, nwk, P, h.batch_xbuf, h.spin_limit, h.poll_delay, grid, block, smem, s);         \
    if (FS_) return HALP_ERR_UNSUPPORTED;                                                          \
    if (nwaves <= 12)                                                                              \
      return launch_kt<BITS_, NDW_, 12, FS_>(a, nwk, P, h.batch_xbuf, h.spin_limit, h.poll_delay, grid, block, smem, s);        \
    return launch_kt<BITS_, NDW_, 16, FS_>(a, nwk, P, h.batch_xbuf, h.spin_limit, h.poll_delay, grid, block, smem, s);          \
  }
  auto launch_loop = [&]() -> int {
    HALP_BT(8, 1, true) HALP_BT(8, 2, true) HALP_BT(8, 4, true)
    HALP_BT(16, 1, true) HALP_BT(16, 2, true) HALP_BT(16, 4, true)
    HALP_BT(8, 1, false) HALP_BT(8, 2, false) HALP_BT(8, 4, false)
    HALP_BT(16, 1, false) HALP_BT(16, 2, false) HALP_BT(16, 4, false)
    return HALP_ERR_UNSUPPORTED;
  };
#undef HALP_BT
  const int lrc = launch_loop();
  if (lrc != HALP_OK || P == 1) return lrc;
  const dim3 fgrid((p.d + 255) / 256, p.R);
  if (p.b == 8) hipLaunchKernelGGL(batch_split_finish<8>, fgrid, dim3(256), 0, s, a, h.buf.scales);
  else hipLaunchKernelGGL(batch_split_finish<16>, fgrid, dim3(256), 0, s, a, h.buf.scales);
  return hip_ok(hipGetLastError());
}

}  // namespace halp
