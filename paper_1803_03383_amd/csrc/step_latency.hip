// Measurement aid: the dependent chain of one inner-loop step of Algorithm 4 at 8 bits,
// with nothing beside it.  One workgroup per CU, `waves` waves, each lane two coordinates;
// per step: two 24-bit multiply-adds, the DPP fold, the wave's sum through one LDS word and
// a barrier, the add of the waves' sums, the fp64 scalar path of gamma (conversion, three
// products, one sum, floor, conversion, clamp) and the update of the two coordinates
// (multiply-add, shift, add, clamp).  No row is fetched, no random bit drawn, nothing is
// counted: row values and rounding terms are lane constants.  The time per step of this
// kernel is the latency floor of the several-wave register kernels with one chain per CU
// (`waves` = 2 or 4; `waves` = 1 runs the chain of the one-chain-wave form, further down).
#include "halp_device.hpp"
#include "halp_internal.hpp"

namespace halp {
namespace {

__device__ __forceinline__ int mad24(int a, int b, int c) {
  int r;
  asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

template <int NW>
__global__ __launch_bounds__(64 * NW) void step_latency_kernel(int64_t steps, double dscale, double aB,
                                                              double inv_s, uint32_t* out) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  __shared__ __attribute__((aligned(16))) int s_part[2][16];
  __shared__ int s_dump[64 * NW];
  using Lds = __attribute__((address_space(3))) int;
  if (tid < 32) (&s_part[0][0])[tid] = 0;
  __syncthreads();
  Lds* const slot0 = (Lds*)((lane != 63) ? &s_dump[tid] : &s_part[0][wave]);
  Lds* const slot1 = (Lds*)((lane != 63) ? &s_dump[tid] : &s_part[1][wave]);
  int z0 = (lane * 7 + 1) & 7, z1 = -((lane * 3 + 1) & 3);
  int xs[8][2];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    xs[s][0] = ((lane * 13 + s * 5 + 1) % 11) - 5;
    xs[s][1] = ((lane * 17 + s * 3 + 1) % 13) - 6;
  }
  const int hv0 = (lane * 29 + 1) & 1023, hv1 = (lane * 31 + 1) & 511;
  const double rho = 0.37;
  for (int64_t t = 0; t < steps; t += 8) {
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const int x0 = xs[s][0], x1 = xs[s][1];
      int D = wave_fold_i32(mad24(x0, z0, mad24(x1, z1, 0)));
      if (NW > 1) {
        *((s & 1) ? slot1 : slot0) = D;
        __syncthreads();
        int q[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) q[w] = s_part[s & 1][w];
#pragma unroll
        for (int w = NW / 2; w >= 1; w /= 2) {
#pragma unroll
          for (int k = 0; k < w; ++k) q[k] += q[k + w];
        }
        D = q[0];
      } else {
        D = __builtin_amdgcn_readlane(D, 63);
      }
      const double delta = __dmul_rn(dscale, (double)D);
      const double beta = __dmul_rn(aB, delta);
      const double f = floor(__dadd_rn(__dmul_rn(beta, inv_s), rho));
      int nf;
      asm("v_cvt_i32_f64 %0, -%1" : "=v"(nf) : "v"(f));
      const int ng = min(max(nf, -127), 128);
      const int v0 = mad24(ng, x0, hv0 + ((lane + s * 37) & 255));
      const int v1 = mad24(ng, x1, hv1 + ((lane * 3 + s * 11) & 255));
      z0 = min(max(z0 + (v0 >> 8), -128), 127);
      z1 = min(max(z1 + (v1 >> 8), -128), 127);
    }
  }
  out[blockIdx.x * 64 * NW + tid] = (uint32_t)(z0 * 131 + z1);
}

// The same for the form with ONE chain wave that holds a row of 512 coordinates (four strips
// per lane, two coordinates per register): per step one packed dot per strip, the DPP fold, the
// sum read from lane 63, the fp64 path of gamma, the update on packed 16-bit halves and one LDS
// store of the unclamped strips; the step's record (row values and rounding terms) comes from
// an LDS ring that nobody refills, read one step ahead; one barrier per window of 8 steps.
__global__ __launch_bounds__(64) void step_latency_lone_kernel(int64_t steps, double dscale, double aB,
                                                              double inv_s, uint32_t* out) {
  constexpr int UPL = 4;
  typedef short S2 __attribute__((ext_vector_type(2)));
  typedef int I4 __attribute__((ext_vector_type(4)));
  const int lane = threadIdx.x & 63;
  __shared__ __attribute__((aligned(16))) I4 s_rec[8][2][64];  // [step][values | rounding terms][lane]
  __shared__ __attribute__((aligned(16))) I4 s_log[8][64];
  for (int s = 0; s < 8; ++s) {
    I4 xv, cv;
#pragma unroll
    for (int u = 0; u < UPL; ++u) {
      const int a = ((lane * 13 + s * 5 + u) % 11) - 5, b = ((lane * 17 + s * 3 + u) % 13) - 6;
      xv[u] = (a & 0xFFFF) | (b << 16);
      cv[u] = ((lane * 29 + s * 37 + u) & 511) | (((lane * 31 + s * 11 + u) & 511) << 16);
    }
    s_rec[s][0][lane] = xv;
    s_rec[s][1][lane] = cv;
  }
  S2 zp[UPL];
#pragma unroll
  for (int u = 0; u < UPL; ++u) zp[u] = S2{(short)((lane * 7 + u) & 7), (short)(-((lane * 3 + u) & 3))};
  const double rho = 0.37;
  __syncthreads();
  for (int64_t t = 0; t < steps; t += 8) {
    I4 rx = s_rec[0][0][lane], rc = s_rec[0][1][lane];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      S2 xp[UPL], crp[UPL];
#pragma unroll
      for (int u = 0; u < UPL; ++u) {
        const int xe = rx[u], ce = rc[u];
        xp[u] = __builtin_bit_cast(S2, xe);
        crp[u] = __builtin_bit_cast(S2, ce);
      }
      if (s + 1 < 8) {
        rx = s_rec[s + 1][0][lane];
        rc = s_rec[s + 1][1][lane];
      }
      int p0 = 0, p1 = 0;
#pragma unroll
      for (int u = 0; u < UPL; u += 2) {
        p0 = __builtin_amdgcn_sdot2(xp[u], zp[u], p0, false);
        p1 = __builtin_amdgcn_sdot2(xp[u + 1], zp[u + 1], p1, false);
      }
      const int D = wave_sum_i32(p0 + p1);
      const double delta = __dmul_rn(dscale, (double)D);
      const double beta = __dmul_rn(aB, delta);
      const double f = floor(__dadd_rn(__dmul_rn(beta, inv_s), rho));
      int nf;
      asm("v_cvt_i32_f64 %0, -%1" : "=v"(nf) : "v"(f));
      const int ng = min(max(nf, -127), 128);
      const S2 ngp = S2{(short)ng, (short)ng};
      I4 vq;
#pragma unroll
      for (int u = 0; u < UPL; ++u) {
        S2 v = xp[u] * ngp + crp[u];
        v = (v >> (S2)(8)) + zp[u];  // the rounding term of the record carries the whole of -h~
        vq[u] = __builtin_bit_cast(int, v);
        zp[u] = __builtin_elementwise_min(__builtin_elementwise_max(v, (S2)(-128)), (S2)(127));
      }
      s_log[s][lane] = vq;
    }
    __syncthreads();
  }
  uint32_t acc = (uint32_t)s_log[7][lane][0];
#pragma unroll
  for (int u = 0; u < UPL; ++u) acc = acc * 131u + __builtin_bit_cast(uint32_t, zp[u]);
  out[blockIdx.x * 64 + threadIdx.x] = acc;
}

}  // namespace

int launch_debug_step_latency(int waves, int64_t steps, int blocks, uint32_t* out, hipStream_t s) {
  const double dscale = 1.0 / 512, aB = 0.3, inv_s = 8.0;
  const dim3 grid(blocks);
  switch (waves) {
    case 1: hipLaunchKernelGGL(step_latency_lone_kernel, grid, dim3(64), 0, s, steps, dscale, aB, inv_s, out); break;
    case 2: hipLaunchKernelGGL(step_latency_kernel<2>, grid, dim3(128), 0, s, steps, dscale, aB, inv_s, out); break;
    case 4: hipLaunchKernelGGL(step_latency_kernel<4>, grid, dim3(256), 0, s, steps, dscale, aB, inv_s, out); break;
    default: return HALP_ERR_INVALID;
  }
  return hip_ok(hipGetLastError());
}

}  // namespace halp
