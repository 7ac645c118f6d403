// Full-precision pass of a HALP epoch (Algorithm 4, outer lines) for rows too wide for the
// kernels that keep a whole row (K = 1) or a whole tile of rows (softmax) on chip:
//   phi_i = x_i^T w~   and   g~ = (1/N) sum_i l_i'(phi_i) x_i + lambda w~.
//
// K = 1, 4096 < d <= 16384 (`fullgrad_k1_wide`): a row is cut across the waves of a workgroup,
// 1024 columns each; a wave keeps its part of w~, of the partial gradient and of the rows of
// two batches in registers.  Per batch the waves' partial margins meet in LDS (one barrier;
// the slots alternate between two sets), every wave adds them in wave order -- the same sum in
// every wave -- and applies the residual to its own columns: X still crosses HBM once.
//
// Softmax, d > 1024 or rows the pipelined kernel does not take: the margins need all columns of
// a row before the residuals exist, and 16 rows of such a width do not fit on chip, so the pass
// reads X twice: `softmax_wide_margins` (first product over column blocks of 512, softmax,
// residuals to a workspace), then `softmax_wide_gradient` (second product, one workgroup per
// column block and row split, G block in registers).  Both run on the matrix cores like the
// narrower kernels.  Scored against one read of X this form cannot pass 0.5 of the HBM peak.
#include "fullgrad_args.hpp"
#include "halp_device.hpp"

namespace halp {
namespace {

typedef float F4 __attribute__((ext_vector_type(4)));
typedef float F2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot4(const F4& a, const F4& b, float acc) {
  acc = __builtin_fmaf(a.x, b.x, acc);
  acc = __builtin_fmaf(a.y, b.y, acc);
  acc = __builtin_fmaf(a.z, b.z, acc);
  acc = __builtin_fmaf(a.w, b.w, acc);
  return acc;
}
__device__ __forceinline__ void axpy4(float s, const F4& x, F4& g) {
  g.x = __builtin_fmaf(s, x.x, g.x);
  g.y = __builtin_fmaf(s, x.y, g.y);
  g.z = __builtin_fmaf(s, x.z, g.z);
  g.w = __builtin_fmaf(s, x.w, g.w);
}

// chunk at column `col` of a row; columns >= d read as 0 (the row stride is a multiple of 4
// floats, so a whole F4 that starts below d lies inside the row)
__device__ __forceinline__ F4 load_chunk(const float* row, int col, int d) {
  F4 v = F4{0.f, 0.f, 0.f, 0.f};
  if (col < d) {
    v = __builtin_nontemporal_load(reinterpret_cast<const F4*>(row + col));
    if (col + 1 >= d) v.y = 0.f;
    if (col + 2 >= d) v.z = 0.f;
    if (col + 3 >= d) v.w = 0.f;
  }
  return v;
}

// ---- K = 1: squared and logistic, a row cut across the waves ---------------------------------
constexpr int kWideNV = 4;     // F4 chunks per lane: 1024 columns per wave
constexpr int kWideRB = 2;     // rows per batch
constexpr int kWideMaxW = 16;  // waves per workgroup at most: d <= 16384

template <int LOSS>
__global__ __launch_bounds__(64 * kWideMaxW) void fullgrad_k1_wide(FgArgs a) {
  constexpr int NV = kWideNV, RB = kWideRB;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int W = (int)(blockDim.x >> 6);
  const int chain = blockIdx.y;
  const float* __restrict__ X = a.X + (int64_t)chain * a.x_chain_stride;
  const float* __restrict__ y =
      reinterpret_cast<const float*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const float* __restrict__ w = a.w + (int64_t)chain * a.d;
  float* __restrict__ phi = a.phi + (int64_t)chain * a.N;
  const int d = a.d;
  const int64_t N = a.N, ldx = a.ldx;
  const int c0 = wave * 256 * NV;  // first column of this wave

  F4 wv[NV], gv[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int col = c0 + 4 * (lane + 64 * k);
    float t[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      t[e] = 0.f;
      if (col + e < d) t[e] = a.fscale ? __fdiv_rn(w[col + e], a.fscale[col + e]) : w[col + e];
    }
    wv[k] = F4{t[0], t[1], t[2], t[3]};
    gv[k] = F4{0.f, 0.f, 0.f, 0.f};
  }
  double loss_acc = 0.0;
  __shared__ float s_part[2][RB][kWideMaxW];  // partial margins: [set][row of the batch][wave]

  const int64_t nblk = (N + RB - 1) / RB;
  const int64_t stride = a.parts;
  int64_t bi = blockIdx.x;
  F4 xa[RB][NV], xb[RB][NV];

  auto load_batch = [&](F4(&xv)[RB][NV], int64_t blk) {
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const int64_t row = blk * RB + r;
      const float* rp = X + row * ldx;
#pragma unroll
      for (int k = 0; k < NV; ++k)
        xv[r][k] = row < N ? load_chunk(rp, c0 + 4 * (lane + 64 * k), d) : F4{0.f, 0.f, 0.f, 0.f};
    }
  };
  auto reduce_batch = [&](F4(&xv)[RB][NV], int64_t blk, int set) {
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      float p = 0.f;
#pragma unroll
      for (int k = 0; k < NV; ++k) p = dot4(xv[r][k], wv[k], p);
      p = wave_sum_f32(p);
      if (lane == 0) s_part[set][r][wave] = p;
    }
    __syncthreads();  // the slots of the other set were last read before the previous barrier
    float res[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      float m = 0.f;  // phi_i: the waves' parts in wave order, the same sum in every wave
      for (int w2 = 0; w2 < W; ++w2) m += s_part[set][r][w2];
      const int64_t row = blk * RB + r;
      const bool ok = row < N;
      const float yi = ok ? y[row] : 0.f;
      float rr, li;
      if (LOSS == HALP_LOSS_SQUARED) {
        rr = m - yi;
        li = 0.5f * rr * rr;
      } else {
        rr = -yi / (1.0f + expf(yi * m));
        const float s = -yi * m;
        li = fmaxf(s, 0.f) + log1pf(expf(-fabsf(s)));
      }
      res[r] = ok ? rr : 0.f;
      if (ok && wave == 0) {
        loss_acc += (double)li;
        if (lane == 0) phi[row] = m;
      }
    }
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
      for (int k = 0; k < NV; ++k) axpy4(res[r], xv[r][k], gv[k]);
  };

  // every wave of the workgroup takes the same trips through this loop (barriers inside)
  if (bi < nblk) load_batch(xa, bi);
  while (bi < nblk) {
    const int64_t b1 = bi + stride;
    if (b1 < nblk) load_batch(xb, b1);
    reduce_batch(xa, bi, 0);
    if (b1 >= nblk) break;
    const int64_t b2 = b1 + stride;
    if (b2 < nblk) load_batch(xa, b2);
    reduce_batch(xb, b1, 1);
    bi = b2;
  }

  // each wave owns its columns of the partial gradient; the loss lives in wave 0 (all its lanes
  // hold the same sum)
  float* pg = a.partial_g + ((int64_t)chain * a.parts + blockIdx.x) * (int64_t)d;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int col = c0 + 4 * (lane + 64 * k);
    if (col < d) pg[col] = gv[k].x;
    if (col + 1 < d) pg[col + 1] = gv[k].y;
    if (col + 2 < d) pg[col + 2] = gv[k].z;
    if (col + 3 < d) pg[col + 3] = gv[k].w;
  }
  if (wave == 0 && lane == 0) a.partial_loss[(int64_t)chain * max(a.parts, a.loss_parts) + blockIdx.x] = loss_acc;
}

// ---- softmax, wide rows: two passes over X on the matrix cores ------------------------------
constexpr int kRows = 16;          // rows per tile
constexpr int kCB = 512;           // columns per block: 128 per wave
constexpr int kLD = kCB + 8;       // LDS row stride (floats), 8 mod 64: see the narrower kernels
constexpr int kRtStride = 20;

template <typename T, typename F>
__device__ __forceinline__ T row_fold(T v, F op) {  // over each row of 16 lanes, into every lane
  v = op(v, dpp_quad_swap1(v));
  v = op(v, dpp_quad_swap2(v));
  v = op(v, dpp_half_mirror(v));
  v = op(v, dpp_row_mirror(v));
  return v;
}

// X[tile rows][cb .. cb + 511] into LDS, zero past d and past N: thread t takes float4 t % 128 of
// rows t / 128, t / 128 + 2, ..
__device__ __forceinline__ void stage_block(const float* X, int64_t ldx, int64_t N, int d, int64_t tile,
                                            int cb, float* s_x, int tid) {
  const int f = tid & 127, r0 = tid >> 7;
  const int col = cb + 4 * f;
  F4 v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t row = tile * kRows + r0 + 2 * i;
    v[i] = row < N ? load_chunk(X + row * ldx, col, d) : F4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) *reinterpret_cast<F4*>(s_x + (r0 + 2 * i) * kLD + 4 * f) = v[i];
}

// pass 1: margins, softmax, loss; residuals [N][16] to the workspace
__global__ __launch_bounds__(256) void softmax_wide_margins(FgArgs a) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int chain = blockIdx.y;
  const int d = a.d, K = a.K;
  const int64_t N = a.N, ldx = a.ldx;
  const float* __restrict__ X = a.X + (int64_t)chain * a.x_chain_stride;
  const int32_t* __restrict__ y =
      reinterpret_cast<const int32_t*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const float* __restrict__ w = a.w + (int64_t)chain * K * d;
  float* __restrict__ phi = a.phi + (int64_t)chain * N * K;
  float* __restrict__ resid = a.resid + (int64_t)chain * N * 16;
  __shared__ __attribute__((aligned(16))) float s_x[kRows * kLD];
  __shared__ __attribute__((aligned(16))) float s_pphi[4][kRows][16];
  __shared__ double s_loss[256];
  const int li = lane & 15, lq = lane >> 4;
  const int cw0 = wave * 128;
  double loss_acc = 0.0;
  const int64_t tiles = (N + kRows - 1) / kRows;
  for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    F4 pa = F4{0.f, 0.f, 0.f, 0.f}, pb = F4{0.f, 0.f, 0.f, 0.f};
    for (int cb = 0; cb < d; cb += kCB) {
      __syncthreads();  // the block before this one has been multiplied
      stage_block(X, ldx, N, d, tile, cb, s_x, tid);
      // W~ of this wave's 128 columns of the block as B operand: lane (j, q) holds
      // W~[j][cb + cw0 + 16 m + 4 q + e] for chunk m and e = 0..3
      float wreg[8][4];
#pragma unroll
      for (int m = 0; m < 8; ++m)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int col = cb + cw0 + 16 * m + 4 * lq + e;
          float v = w[(int64_t)min(li, K - 1) * d + min(col, d - 1)];
          if (a.fscale) v = __fdiv_rn(v, a.fscale[min(col, d - 1)]);
          wreg[m][e] = (li < K && col < d) ? v : 0.f;
        }
      __syncthreads();
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        const F4 x = *reinterpret_cast<const F4*>(s_x + li * kLD + cw0 + 16 * m + 4 * lq);
        pa = __builtin_amdgcn_mfma_f32_16x16x4f32(x.x, wreg[m][0], pa, 0, 0, 0);
        pb = __builtin_amdgcn_mfma_f32_16x16x4f32(x.y, wreg[m][1], pb, 0, 0, 0);
        pa = __builtin_amdgcn_mfma_f32_16x16x4f32(x.z, wreg[m][2], pa, 0, 0, 0);
        pb = __builtin_amdgcn_mfma_f32_16x16x4f32(x.w, wreg[m][3], pb, 0, 0, 0);
      }
    }
    // component r of lane (j, q) is row 4 q + r, class j
    s_pphi[wave][4 * lq + 0][li] = pa.x + pb.x;
    s_pphi[wave][4 * lq + 1][li] = pa.y + pb.y;
    s_pphi[wave][4 * lq + 2][li] = pa.z + pb.z;
    s_pphi[wave][4 * lq + 3][li] = pa.w + pb.w;
    __syncthreads();
    {  // softmax: thread (row tid / 16, class tid % 16)
      const int r = tid >> 4, c = tid & 15;
      const int64_t row = tile * kRows + r;
      const bool valid = c < K;
      const int ycur = y[min(row, N - 1)];
      const float logit = ((s_pphi[0][r][c] + s_pphi[1][r][c]) + s_pphi[2][r][c]) + s_pphi[3][r][c];
      const float mx = row_fold(valid ? logit : -INFINITY, [](float x, float y2) { return fmaxf(x, y2); });
      const float e = valid ? expf(logit - mx) : 0.f;
      const float se = row_fold(e, [](float x, float y2) { return x + y2; });
      if (row < N) {
        float rc = 0.f;
        if (valid) {
          rc = e / se - (c == ycur ? 1.0f : 0.f);
          phi[row * K + c] = logit;
          if (c == ycur) loss_acc += (double)(logf(se) + mx - logit);
        }
        resid[row * 16 + c] = rc;
      }
    }
  }
  s_loss[tid] = loss_acc;
  __syncthreads();
  if (tid == 0) {
    double l = 0.0;
    for (int t = 0; t < 256; ++t) l += s_loss[t];  // fixed order
    a.partial_loss[(int64_t)chain * max(a.parts, a.loss_parts) + blockIdx.x] = l;
  }
}

// pass 2: G[:, column block] += R^T X over this workgroup's tiles; workgroup (row split
// blockIdx.x, column block blockIdx.z) keeps its 16 x 512 block of G in registers
__global__ __launch_bounds__(256) void softmax_wide_gradient(FgArgs a) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int chain = blockIdx.y;
  const int d = a.d, K = a.K;
  const int64_t N = a.N, ldx = a.ldx;
  const float* __restrict__ X = a.X + (int64_t)chain * a.x_chain_stride;
  const float* __restrict__ resid = a.resid + (int64_t)chain * N * 16;
  __shared__ __attribute__((aligned(16))) float s_x[kRows * kLD];
  __shared__ __attribute__((aligned(16))) float s_rt[16 * kRtStride];  // residuals [class][row]
  const int li = lane & 15, lq = lane >> 4;
  const int cw0 = wave * 128;
  const int cb = blockIdx.z * kCB;
  // G[class 4 q + r][cb + cw0 + 32 g + 2 j + e] in component r of gacc[g][e] of lane (j, q)
  F4 gacc[4][2];
#pragma unroll
  for (int g = 0; g < 4; ++g) gacc[g][0] = gacc[g][1] = F4{0.f, 0.f, 0.f, 0.f};
  const int64_t tiles = (N + kRows - 1) / kRows;
  for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    __syncthreads();  // the tile before this one has been multiplied
    stage_block(X, ldx, N, d, tile, cb, s_x, tid);
    {  // residuals of the tile, transposed: thread (row tid / 16, class tid % 16)
      const int r = tid >> 4, c = tid & 15;
      const int64_t row = tile * kRows + r;
      s_rt[c * kRtStride + r] = row < N ? resid[row * 16 + c] : 0.f;
    }
    __syncthreads();
    const F4 rt = *reinterpret_cast<const F4*>(s_rt + li * kRtStride + 4 * lq);
    const float rtk[4] = {rt.x, rt.y, rt.z, rt.w};
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      F2 xb[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        xb[kk] = *reinterpret_cast<const F2*>(s_x + (4 * lq + kk) * kLD + cw0 + 32 * g + 2 * li);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        gacc[g][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(rtk[kk], xb[kk].x, gacc[g][0], 0, 0, 0);
        gacc[g][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(rtk[kk], xb[kk].y, gacc[g][1], 0, 0, 0);
      }
    }
  }
  float* pg = a.partial_g + ((int64_t)chain * a.parts + blockIdx.x) * (int64_t)K * d;
#pragma unroll
  for (int g = 0; g < 4; ++g)
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int col = cb + cw0 + 32 * g + 2 * li + e;
      if (col < d) {
        if (4 * lq + 0 < K) pg[(int64_t)(4 * lq + 0) * d + col] = gacc[g][e].x;
        if (4 * lq + 1 < K) pg[(int64_t)(4 * lq + 1) * d + col] = gacc[g][e].y;
        if (4 * lq + 2 < K) pg[(int64_t)(4 * lq + 2) * d + col] = gacc[g][e].z;
        if (4 * lq + 3 < K) pg[(int64_t)(4 * lq + 3) * d + col] = gacc[g][e].w;
      }
    }
}

}  // namespace

int fullgrad_k1_wide_max_d() { return 256 * kWideNV * kWideMaxW; }

int launch_fullgrad_k1_wide(const FgArgs& a, int loss, int R, hipStream_t s) {
  const int W = (a.d + 256 * kWideNV - 1) / (256 * kWideNV);
  if (W < 1 || W > kWideMaxW) return HALP_ERR_UNSUPPORTED;
  const dim3 grid(a.parts, R), block(64 * W);
  if (loss == HALP_LOSS_SQUARED) hipLaunchKernelGGL(fullgrad_k1_wide<HALP_LOSS_SQUARED>, grid, block, 0, s, a);
  else hipLaunchKernelGGL(fullgrad_k1_wide<HALP_LOSS_LOGISTIC>, grid, block, 0, s, a);
  return hip_ok(hipGetLastError());
}

int fullgrad_k1_wide_rows_per_batch() { return kWideRB; }

int launch_fullgrad_softmax_wide(const FgArgs& a, int R, hipStream_t s) {
  if (!a.resid) return HALP_ERR_UNSUPPORTED;
  static_assert(kCB == kSoftmaxWideBlock, "the launch shape is derived from this block width");
  hipLaunchKernelGGL(softmax_wide_margins, dim3(a.loss_parts, R), dim3(256), 0, s, a);
  if (hipGetLastError() != hipSuccess) return HALP_ERR_HIP;
  const int ncb = (a.d + kCB - 1) / kCB;
  hipLaunchKernelGGL(softmax_wide_gradient, dim3(a.parts, R, ncb), dim3(256), 0, s, a);
  return hip_ok(hipGetLastError());
}

}  // namespace halp
