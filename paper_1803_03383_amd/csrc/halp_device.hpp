// Device-side building blocks shared by the HALP kernels (gfx950, wave64):
// Philox4x32-10, the random-stream layout, wave reductions on DPP, and the two
// quantizers of Sec. 3 "Quantization" in the forms the library's contract fixes.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace halp {

constexpr int kWave = 64;

enum Purpose : uint32_t { kIdx = 0, kGamma = 1, kZround = 2, kReg = 3, kHround = 4, kOpt2 = 5 };

struct U4 {
  uint32_t x, y, z, w;
};

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies
// whose high halves are mixed with the neighbouring counter words and a Weyl
// sequence of round keys.
__device__ __forceinline__ U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c.x;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c.z;
    U4 n;
    n.x = (uint32_t)(p1 >> 32) ^ c.y ^ k0;
    n.y = (uint32_t)p1;
    n.z = (uint32_t)(p0 >> 32) ^ c.w ^ k1;
    n.w = (uint32_t)p0;
    c = n;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c;
}

// Block `blk` of the word stream of a purpose: counter (lo(blk), hi(blk), epoch, purpose).
__device__ __forceinline__ U4 stream_block(uint64_t seed, uint32_t purpose, uint32_t epoch,
                                           uint64_t blk) {
  return philox4x32_10(U4{(uint32_t)blk, (uint32_t)(blk >> 32), epoch, purpose}, (uint32_t)seed,
                       (uint32_t)(seed >> 32));
}

__device__ __forceinline__ uint32_t pick(const U4& v, uint32_t k) {
  return k == 0 ? v.x : (k == 1 ? v.y : (k == 2 ? v.z : v.w));
}

// Steps of an epoch.  Option I of Algorithms 1-3 runs all T; option II ends the epoch at the
// iterate after t steps, t uniform on {0, .., T-1} (word 0 of its own stream, multiply-shift).
__device__ __forceinline__ int64_t epoch_steps(uint64_t seed, uint32_t epoch, int64_t T, int option2) {
  if (!option2 || T <= 0) return T;
  const U4 r = stream_block(seed, kOpt2, epoch, 0);
  return (int64_t)(((uint64_t)r.x * (uint64_t)T) >> 32);
}

// Rounding bits of z: a row of z is cut into strips 16 rounding bits wide (16/b
// coordinates: two at b = 8, one at b = 16).  One block serves strip `strip` for the
// eight steps 8s .. 8s+7; step t reads the 16-bit field t % 8 (half f % 2 of word f / 2).
__device__ __forceinline__ U4 zround_block(uint64_t seed, uint32_t epoch, uint32_t strip,
                                           uint32_t s) {
  return philox4x32_10(U4{strip, s, epoch, (uint32_t)kZround}, (uint32_t)seed,
                       (uint32_t)(seed >> 32));
}

// the 16-bit field of step t (any t; only t % 8 matters) in a strip's block
__device__ __forceinline__ uint32_t zround_field(const U4& r, uint32_t t) {
  const uint32_t f = t & 7u;
  return (pick(r, f >> 1) >> (16u * (f & 1u))) & 0xFFFFu;
}

// ---- wave-wide sums --------------------------------------------------------
// Four DPP steps fold each row of 16 lanes (quad swaps, half-row mirror, row
// mirror); two row broadcasts (lane 15 of rows 0 and 2 into rows 1 and 3, then
// lane 31 into rows 2 and 3) bring the total to lane 63, which is read out.
// All 64 lanes must be active.

template <typename T>
__device__ __forceinline__ T dpp_quad_swap1(T v) {  // lanes 1,0,3,2
  return __builtin_bit_cast(
      T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));
}
template <typename T>
__device__ __forceinline__ T dpp_quad_swap2(T v) {  // lanes 2,3,0,1
  return __builtin_bit_cast(
      T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false));
}
template <typename T>
__device__ __forceinline__ T dpp_half_mirror(T v) {  // reverse within 8 lanes
  return __builtin_bit_cast(
      T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false));
}
template <typename T>
__device__ __forceinline__ T dpp_row_mirror(T v) {  // reverse within 16 lanes
  return __builtin_bit_cast(
      T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false));
}
template <typename T>
__device__ __forceinline__ T dpp_bcast15(T v) {  // rows 1, 3 get lane 15 of rows 0, 2; others 0
  return __builtin_bit_cast(
      T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false));
}
template <typename T>
__device__ __forceinline__ T dpp_bcast31(T v) {  // rows 2, 3 get lane 31; rows 0, 1 get 0
  return __builtin_bit_cast(
      T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false));
}

__device__ __forceinline__ int wave_sum_i32(int v) {
  v += dpp_quad_swap1(v);
  v += dpp_quad_swap2(v);
  v += dpp_half_mirror(v);
  v += dpp_row_mirror(v);
  v += dpp_bcast15(v);
  v += dpp_bcast31(v);
  return __builtin_amdgcn_readlane(v, 63);
}

// the same fold without the read-out: lane 63 holds the sum, the other lanes partial sums
__device__ __forceinline__ int wave_fold_i32(int v) {
  v += dpp_quad_swap1(v);
  v += dpp_quad_swap2(v);
  v += dpp_half_mirror(v);
  v += dpp_row_mirror(v);
  v += dpp_bcast15(v);
  v += dpp_bcast31(v);
  return v;
}

__device__ __forceinline__ float wave_sum_f32(float v) {
  v += dpp_quad_swap1(v);
  v += dpp_quad_swap2(v);
  v += dpp_half_mirror(v);
  v += dpp_row_mirror(v);
  v += dpp_bcast15(v);
  v += dpp_bcast31(v);
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

__device__ __forceinline__ float wave_fold_f32(float v) {  // lane 63 holds the sum
  v += dpp_quad_swap1(v);
  v += dpp_quad_swap2(v);
  v += dpp_half_mirror(v);
  v += dpp_row_mirror(v);
  v += dpp_bcast15(v);
  v += dpp_bcast31(v);
  return v;
}

__device__ __forceinline__ long long wave_sum_i64(long long v) {
  // exact 64-bit sum: move both halves with the same DPP pattern, add as a pair
  auto step = [](long long x, auto mv) {
    const int lo = mv((int)(uint32_t)x), hi = mv((int)(x >> 32));
    return x + (long long)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
  };
  v = step(v, [](int t) { return dpp_quad_swap1(t); });
  v = step(v, [](int t) { return dpp_quad_swap2(t); });
  v = step(v, [](int t) { return dpp_half_mirror(t); });
  v = step(v, [](int t) { return dpp_row_mirror(t); });
  v = step(v, [](int t) { return dpp_bcast15(t); });
  v = step(v, [](int t) { return dpp_bcast31(t); });
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, 63);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(v >> 32), 63);
  return (long long)(((uint64_t)hi << 32) | lo);
}

// exact 64-bit fold without the read-out: lane 63 holds the sum
__device__ __forceinline__ long long wave_fold_i64(long long v) {
  auto step = [](long long x, auto mv) {
    const int lo = mv((int)(uint32_t)x), hi = mv((int)(x >> 32));
    return x + (long long)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
  };
  v = step(v, [](int t) { return dpp_quad_swap1(t); });
  v = step(v, [](int t) { return dpp_quad_swap2(t); });
  v = step(v, [](int t) { return dpp_half_mirror(t); });
  v = step(v, [](int t) { return dpp_row_mirror(t); });
  v = step(v, [](int t) { return dpp_bcast15(t); });
  v = step(v, [](int t) { return dpp_bcast31(t); });
  return v;
}

// ---- exp of the inner loop's scalar path -----------------------------------------
// l'(phi + x^T z) - l'(phi) is rounded to the integer gamma (Algorithm 4), so the last bit of
// exp can decide an integer.  The library fixes exp as this sequence of correctly rounded
// double operations, which every conforming implementation reproduces bit for bit:
//   k = rint(x log2 e);  r = x - k ln2 (ln2 in two parts, fused multiply-adds);
//   e^r = 1 + (r + r^2 Q(r)),  Q = sum_{n=2..13} r^(n-2)/n!  joined pairwise by r, r^2, r^4;
//   exp(x) = e^r 2^k.   Within 1 ulp of exp; a short dependency chain, no table.
__device__ __forceinline__ double halp_exp(double x) {
  const double k = __builtin_rint(__dmul_rn(x, 0x1.71547652b82fep+0));
  double r = __fma_rn(-k, 0x1.62e42fefa39efp-1, x);
  r = __fma_rn(-k, 0x1.abc9e3b39803fp-56, r);
  const double r2 = __dmul_rn(r, r), r4 = __dmul_rn(r2, r2);
  const double a0 = __fma_rn(0x1.5555555555555p-3, r, 0x1.0000000000000p-1);
  const double a1 = __fma_rn(0x1.1111111111111p-7, r, 0x1.5555555555555p-5);
  const double a2 = __fma_rn(0x1.a01a01a01a01ap-13, r, 0x1.6c16c16c16c17p-10);
  const double a3 = __fma_rn(0x1.71de3a556c734p-19, r, 0x1.a01a01a01a01ap-16);
  const double a4 = __fma_rn(0x1.ae64567f544e4p-26, r, 0x1.27e4fb7789f5cp-22);
  const double a5 = __fma_rn(0x1.6124613a86d09p-33, r, 0x1.1eed8eff8d898p-29);
  const double b0 = __fma_rn(a1, r2, a0), b1 = __fma_rn(a3, r2, a2), b2 = __fma_rn(a5, r2, a4);
  const double q = __fma_rn(__fma_rn(b2, r4, b1), r4, b0);
  const double e = __dadd_rn(__fma_rn(r2, q, r), 1.0);
  double res = ldexp(e, (int)k);
  res = x > 0x1.62e42fefa39efp+9 ? __builtin_inf() : res;  // above log(DBL_MAX)
  res = x < -0x1.74910d52d3052p+9 ? 0.0 : res;             // below half the least subnormal
  return x != x ? x : res;
}

// ---- quantizers -------------------------------------------------------------

// Real -> integer lattice: clamp(floor(x * inv_delta + rho)), rho = r32 / 2^32.
// Multiplication and addition are rounded separately (no fused multiply-add).
__device__ __forceinline__ long long quantize_real(double x, double inv_delta, uint32_t r32,
                                                   double lo, double hi, bool* clamped) {
  const double rho = __dmul_rn((double)r32, 0x1p-32);
  const double q = __dmul_rn(x, inv_delta);
  double f = floor(__dadd_rn(q, rho));
  bool hit = false;
  if (f < lo) { f = lo; hit = true; }
  if (f > hi) { f = hi; hit = true; }
  if (clamped) *clamped = hit;
  return (long long)f;
}

}  // namespace halp
