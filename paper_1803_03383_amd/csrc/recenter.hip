// Bit centering (Sec. 4; the re-scale lines of Algorithm 4), the one-off data
// quantization into (delta_d, b), and two debug kernels that expose the random
// streams.
#include "halp_device.hpp"
#include "halp_internal.hpp"

namespace halp {
namespace {

struct RcArgs {
  const float* g;
  const float* w;  // LP-SVRG only
  int lp;          // 1: Algorithm 2 (fixed delta, z = round(w~ / delta)); 0: Algorithm 4
  double delta;
  void* h;
  void* z;
  double* scales;
  int n;  // K*d
  int b;
  const double* hyper;  // [R][2] alpha, mu of each chain
  double delta_d;
  uint64_t seed;
  uint32_t epoch;
};

// One workgroup per chain.  ||g~||^2 is accumulated by a single lane in index
// order in fp64 (every square of an fp32 value is exact in fp64), so the scales
// are the same bits whatever the launch shape; K*d is at most a few thousand
// and this runs once per epoch.
template <int BITS>
__global__ __launch_bounds__(256) void recenter_kernel(RcArgs a) {
  using ZT = typename std::conditional<BITS == 8, int8_t, int16_t>::type;
  using HT = typename std::conditional<BITS == 8, int16_t, int32_t>::type;
  const int chain = blockIdx.x;
  const int tid = threadIdx.x;
  const float* __restrict__ g = a.g + (int64_t)chain * a.n;
  HT* __restrict__ h = reinterpret_cast<HT*>(a.h) + (int64_t)chain * a.n;
  ZT* __restrict__ z = reinterpret_cast<ZT*>(a.z) + (int64_t)chain * a.n;
  double* sc = a.scales + (int64_t)chain * 8;

  constexpr int kChunk = 4096;
  __shared__ float stage[kChunk];
  __shared__ double s_inv_i;
  __shared__ int s_status;
  double ss = 0.0;
  for (int base = 0; base < a.n; base += kChunk) {
    const int m = min(kChunk, a.n - base);
    for (int k = tid; k < m; k += 256) stage[k] = g[base + k];
    __syncthreads();
    if (tid == 0) {
      for (int k = 0; k < m; ++k) {
        const double v = (double)stage[k];
        ss = __dadd_rn(ss, __dmul_rn(v, v));
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    const double nrm = __dsqrt_rn(ss);
    const double qmax = (double)((1 << (BITS - 1)) - 1);
    int status = 0;
    double delta_m = 0, delta_i = 0, delta_s = 0, inv_i = 0, inv_s = 0;
    if (!isfinite(nrm)) {
      status = -1;
    } else if (nrm == 0.0) {
      status = 1;
    } else {
      // Algorithm 4: s~ = ||g~|| / (mu (2^(b-1) - 1)); Algorithm 2: the given delta
      delta_m = a.lp ? a.delta : __ddiv_rn(nrm, __dmul_rn(a.hyper[2 * chain + 1], qmax));
      delta_i = __dmul_rn(delta_m, BITS == 8 ? 0x1p-8 : 0x1p-16);
      delta_s = __ddiv_rn(delta_i, a.delta_d);
      inv_i = __ddiv_rn(1.0, delta_i);
      inv_s = __ddiv_rn(1.0, delta_s);
      if (!(delta_i > 0) || !isfinite(inv_i) || !isfinite(inv_s)) {
        status = -1;
        delta_m = delta_i = delta_s = inv_i = inv_s = 0;
      }
    }
    sc[0] = delta_m; sc[1] = delta_i; sc[2] = delta_s; sc[3] = nrm;
    sc[4] = inv_i; sc[5] = inv_s; sc[7] = (double)status;
    s_inv_i = inv_i;
    s_status = status;
  }
  __syncthreads();
  const double inv_i = s_inv_i;
  const double alpha = a.hyper[2 * chain];
  const bool live = s_status == 0;
  const double hmax = BITS == 8 ? 32767.0 : 2147483647.0;
  const double hmin = BITS == 8 ? -32768.0 : -2147483648.0;
  const int nblk = (a.n + 3) / 4;
  for (int blk = tid; blk < nblk; blk += 256) {
    U4 r = U4{0, 0, 0, 0};
    if (live) r = stream_block(a.seed + (uint64_t)chain, kHround, a.epoch, (uint64_t)blk);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int k = 4 * blk + e;
      if (k < a.n) {
        long long q = 0;
        if (live)  // h~ = Q_(delta_i, 2b)(alpha g~)
          q = quantize_real(__dmul_rn(alpha, (double)g[k]), inv_i, pick(r, e), hmin, hmax, nullptr);
        h[k] = (HT)q;
        int z0 = 0;  // Algorithm 4: z_{k,0} = Q(0) = 0
        if (a.lp) {  // Algorithm 2: w_{k,0} = w~_k in (delta, b), nearest (ties to even)
          const double zq = rint(__ddiv_rn((double)a.w[(int64_t)chain * a.n + k], a.delta));
          z0 = (int)fmin(fmax(zq, (double)(-(1 << (BITS - 1)))), (double)((1 << (BITS - 1)) - 1));
        }
        z[k] = (ZT)z0;
      }
    }
  }
}

struct QdArgs {
  const float* X;
  void* Xq;
  int64_t rows, ldx, ldxq;
  int d;
  double delta_d;
  const float* fscale;  // [d] per-feature scales or null
};

// Four columns per thread (halp_bind guarantees rows whose strides and bases allow 16-byte
// loads and one packed store per thread).  A row takes tpr = 2^lg threads (the power of two
// at or above its column groups, 256 at most), a workgroup 256 / tpr rows per pass, and a
// thread keeps four rows in flight.  One scale for all columns: x / delta_d is taken as
// x * (1 / delta_d) wherever that cannot round differently -- further than 2^-24 from a
// half-integer, while the two quotients differ by less than 2^-35 below the clamp and both
// clamp above it -- and by the division otherwise.  Per-feature scales keep the division.
template <int BITS>
__device__ __forceinline__ int quantize_one(float x, double dd, double inv, bool fast, double qmax) {
  const double xd = (double)x;
  double q;
  if (fast) {
    q = __dmul_rn(xd, inv);
    const double fr = __dadd_rn(q, -floor(q));
    if (fabs(__dadd_rn(fr, -0.5)) < 0x1p-24) q = __ddiv_rn(xd, dd);
  } else {
    q = __ddiv_rn(xd, dd);
  }
  q = rint(q);  // ties to even
  q = fmin(fmax(q, -qmax), qmax);
  return (int)q;
}

template <int BITS>
__global__ __launch_bounds__(256) void quantize_data_kernel(QdArgs a, int lg) {
  typedef float F4 __attribute__((ext_vector_type(4)));
  const double qmax = (double)((1 << (BITS - 1)) - 1);
  const int groups = (int)(a.ldxq / 4);
  const bool fast = a.fscale == nullptr;
  const double inv = __ddiv_rn(1.0, a.delta_d);
  const int tpr = 1 << lg, rpb = 256 >> lg;
  const int g0 = (int)threadIdx.x & (tpr - 1);
  const int64_t rstep = (int64_t)gridDim.x * rpb;
  constexpr int kFlight = 4;
  for (int64_t row0 = (int64_t)blockIdx.x * rpb + ((int)threadIdx.x >> lg); row0 < a.rows;
       row0 += kFlight * rstep) {
    for (int g = g0; g < groups; g += tpr) {
      const int j = 4 * g;
      F4 xv[kFlight];
#pragma unroll
      for (int e = 0; e < kFlight; ++e) {
        const int64_t row = row0 + e * rstep;
        xv[e] = F4{0.f, 0.f, 0.f, 0.f};
        if (row < a.rows && j < a.d) xv[e] = __builtin_nontemporal_load(reinterpret_cast<const F4*>(a.X + row * a.ldx + j));
      }
#pragma unroll
      for (int e = 0; e < kFlight; ++e) {
        const int64_t row = row0 + e * rstep;
        if (row >= a.rows) break;
        int q[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int col = j + c;
          q[c] = 0;
          if (col < a.d) {
            const double dd = fast ? a.delta_d : __dmul_rn(a.delta_d, (double)a.fscale[col]);
            q[c] = quantize_one<BITS>(xv[e][c], dd, inv, fast, qmax);
          }
        }
        if (BITS == 8) {
          const uint32_t w = (uint32_t)(q[0] & 0xFF) | ((uint32_t)(q[1] & 0xFF) << 8) |
                             ((uint32_t)(q[2] & 0xFF) << 16) | ((uint32_t)(q[3] & 0xFF) << 24);
          *reinterpret_cast<uint32_t*>(reinterpret_cast<int8_t*>(a.Xq) + row * a.ldxq + j) = w;
        } else {
          uint2 w;
          w.x = (uint32_t)(q[0] & 0xFFFF) | ((uint32_t)(q[1] & 0xFFFF) << 16);
          w.y = (uint32_t)(q[2] & 0xFFFF) | ((uint32_t)(q[3] & 0xFFFF) << 16);
          *reinterpret_cast<uint2*>(reinterpret_cast<int16_t*>(a.Xq) + row * a.ldxq + j) = w;
        }
      }
    }
  }
}

__global__ void debug_words_kernel(uint64_t seed, uint32_t purpose, uint32_t epoch, uint64_t n0,
                                   int64_t count, uint32_t* out) {
  const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= count) return;
  const uint64_t n = n0 + (uint64_t)k;
  const U4 r = stream_block(seed, purpose, epoch, n >> 2);
  out[k] = pick(r, (uint32_t)(n & 3));
}

__global__ void debug_zround_kernel(uint64_t seed, uint32_t epoch, uint64_t t, int d, int b, int K,
                                    uint32_t* out) {
  const int cps = 16 / b;
  const int U = (d + cps - 1) / cps;
  const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= (int64_t)K * U) return;
  const int c = (int)(u / U), strip = (int)(u % U);
  const U4 r = zround_block(seed, epoch, (uint32_t)u, (uint32_t)(t >> 3));
  const uint32_t field = zround_field(r, (uint32_t)t);
  for (int e = 0; e < cps; ++e) {
    const int j = strip * cps + e;
    if (j < d) out[(int64_t)c * d + j] = (field >> (e * b)) & ((1u << b) - 1u);
  }
}

// Yardstick of the gradient pass: reads n16 16-byte words once (non-temporal, eight loads in
// flight per thread) and does nothing else; one partial sum per workgroup keeps the loads alive.
typedef uint32_t UV4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void debug_read_kernel(const UV4* __restrict__ p, int64_t n16,
                                                         uint32_t* out) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
  uint32_t acc = 0;
  for (; k + 7 * stride < n16; k += 8 * stride) {
    UV4 v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = __builtin_nontemporal_load(p + k + e * stride);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += v[e].x ^ v[e].y ^ v[e].z ^ v[e].w;
  }
  for (; k < n16; k += stride) {
    const UV4 v = __builtin_nontemporal_load(p + k);
    acc += v.x ^ v.y ^ v.z ^ v.w;
  }
  __shared__ uint32_t red[256];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = red[0];
}

}  // namespace

int launch_debug_read(const void* p, int64_t bytes, uint32_t* out, hipStream_t s) {
  hipLaunchKernelGGL(debug_read_kernel, dim3(kDebugReadBlocks), dim3(256), 0, s,
                     reinterpret_cast<const UV4*>(p), bytes / 16, out);
  return hip_ok(hipGetLastError());
}

int launch_recenter(const halp_handle& h, uint32_t epoch, hipStream_t s) {
  const halp_params& p = h.p;
  RcArgs a;
  a.g = h.buf.g; a.h = h.buf.h; a.z = h.buf.z; a.scales = h.buf.scales;
  a.n = p.K * p.d; a.b = p.b; a.hyper = h.hyper; a.delta_d = p.delta_d;
  a.seed = p.seed; a.epoch = epoch;
  a.w = h.buf.w; a.lp = p.algorithm == HALP_ALG_LPSVRG; a.delta = p.delta;
  if (p.b == 8) hipLaunchKernelGGL(recenter_kernel<8>, dim3(p.R), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(recenter_kernel<16>, dim3(p.R), dim3(256), 0, s, a);
  return hip_ok(hipGetLastError());
}

int launch_quantize_data(const halp_handle& h, hipStream_t s) {
  const halp_params& p = h.p;
  QdArgs a;
  a.X = h.buf.X; a.Xq = h.buf.Xq;
  a.rows = (p.share_data ? 1 : (int64_t)p.R) * p.N;
  a.ldx = h.buf.ldx; a.ldxq = h.buf.ldxq; a.d = p.d; a.delta_d = p.delta_d; a.fscale = h.fscale;
  // what the kernel's 16-byte loads and packed stores assume (halp_bind has checked it)
  const size_t xq_align = p.b == 8 ? 4 : 8;
  if (a.ldx % 4 != 0 || a.ldxq % 4 != 0 || reinterpret_cast<uintptr_t>(a.X) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(a.Xq) % xq_align != 0 || a.ldx < a.d)
    return HALP_ERR_ALIGN;
  const int64_t groups = a.ldxq / 4;
  int lg = 0;
  while (lg < 8 && (1 << lg) < groups) ++lg;  // threads per row: 2^lg >= groups, 256 at most
  const int rpb = 256 >> lg;
  int64_t blocks = (a.rows + 4 * rpb - 1) / (4 * rpb);
  if (blocks > 16384) blocks = 16384;
  if (blocks < 1) blocks = 1;
  if (p.b == 8) hipLaunchKernelGGL(quantize_data_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, s, a, lg);
  else hipLaunchKernelGGL(quantize_data_kernel<16>, dim3((unsigned)blocks), dim3(256), 0, s, a, lg);
  return hip_ok(hipGetLastError());
}

int launch_debug_stream_words(uint64_t seed, uint32_t purpose, uint32_t epoch, uint64_t n0,
                              int64_t count, uint32_t* out, hipStream_t s) {
  if (count == 0) return HALP_OK;
  hipLaunchKernelGGL(debug_words_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s,
                     seed, purpose, epoch, n0, count, out);
  return hip_ok(hipGetLastError());
}

int launch_debug_zround_bits(uint64_t seed, uint32_t epoch, uint64_t t, int32_t d, int32_t b,
                             int32_t K, uint32_t* out, hipStream_t s) {
  const int cps = 16 / b;
  const int64_t units = (int64_t)K * ((d + cps - 1) / cps);
  hipLaunchKernelGGL(debug_zround_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s,
                     seed, epoch, t, d, b, K, out);
  return hip_ok(hipGetLastError());
}

}  // namespace halp
