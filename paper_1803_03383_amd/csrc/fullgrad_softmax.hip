// Full-precision pass of a HALP epoch for softmax regression (Algorithm 4, outer
// lines, K classes):
//   Phi = X W~^T                      [N x K]   margins
//   R   = softmax(Phi) - onehot(y)    [N x K]   residuals l'
//   G   = R^T X                       [K x d]   gradient sum (the 1/N and lambda W~ come later)
// Both products are dense contractions with one small dimension (K <= 16): they run on the
// matrix cores as v_mfma_f32_16x16x4_f32 with the classes padded to 16.
//
// A workgroup (4 waves) takes tiles of 16 rows.  The tile is fetched from HBM once, with
// row-contiguous 16-byte loads, into LDS, from where both products read it: as the A
// operand (rows x columns) of the first and as the B operand (rows x columns, rows being the
// contraction index) of the second.  The next tile's loads are in flight (into registers) while
// the current one is multiplied, and two workgroups share a CU so that one's products overlap
// the other's waits.  Each wave owns a quarter of the columns: its slice of W~ (B operand of the
// first product) and of G (accumulators of the second) stay in registers for the whole pass.
// The four partial margin tiles are summed in wave order through LDS, the softmax is taken
// by 256 threads (one per row and class; a row of 16 classes is a DPP row), and the
// residuals go back through LDS, transposed, as the A operand of the second product.
// Per-workgroup partial gradients and losses are summed by the common second-stage kernel.
#include "fullgrad_args.hpp"
#include "halp_device.hpp"

namespace halp {
namespace {

typedef float F4 __attribute__((ext_vector_type(4)));

constexpr int kRows = 16;    // rows per tile
constexpr int kRtStride = 20;  // floats between classes in the transposed residual tile

template <typename T, typename F>
__device__ __forceinline__ T row_fold(T v, F op) {  // over each row of 16 lanes, into every lane
  v = op(v, dpp_quad_swap1(v));
  v = op(v, dpp_quad_swap2(v));
  v = op(v, dpp_half_mirror(v));
  v = op(v, dpp_row_mirror(v));
  return v;
}

// NG: groups of 32 columns per wave; a wave covers CW = 32 NG columns, the workgroup 4 CW >= d.
// Two workgroups share a CU (one tile buffer each): while one multiplies, the other waits for
// memory, stages its tile or takes its softmax.
template <int NG>
__global__ __launch_bounds__(256, 2) void fullgrad_softmax_mfma(FgArgs a) {
  constexpr int CW = 32 * NG;
  constexpr int NT16 = 2 * NG;     // 16-column chunks per wave (first product), float4 slots per thread
  // LDS row stride (floats), 8 mod 64: the 8-byte reads of the second product (rows 4 apart
  // within a half-wave) are conflict-free, the 16-byte reads of the first meet in pairs
  constexpr int LDT = 4 * CW + 8;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int chain = blockIdx.y;
  const int d = a.d, K = a.K;
  const int64_t N = a.N, ldx = a.ldx;
  const float* __restrict__ X = a.X + (int64_t)chain * a.x_chain_stride;
  const int32_t* __restrict__ y =
      reinterpret_cast<const int32_t*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const float* __restrict__ w = a.w + (int64_t)chain * K * d;
  float* __restrict__ phi = a.phi + (int64_t)chain * N * K;

  extern __shared__ __attribute__((aligned(16))) float s_x[];            // [kRows][LDT]
  __shared__ __attribute__((aligned(16))) float s_pphi[4][kRows][16];    // partial margins per wave
  __shared__ __attribute__((aligned(16))) float s_rt[16 * kRtStride];    // residuals [class][row]
  __shared__ double s_loss[256];

  const int li = lane & 15;  // row (A) / class or column (B, C) index of this lane
  const int lq = lane >> 4;  // contraction index of this lane
  const int cw0 = wave * CW;

  // W~ slice as B operand of the first product: for column chunk m and e = 0..3, lane (j, q)
  // holds W~[j][cw0 + 16 m + 4 q + e]
  float wreg[NT16][4];
  // Every load is unconditional, from a clamped address, and all are issued before the first
  // is used (a load that is only needed under a condition would be waited for on its own).
#pragma unroll
  for (int m = 0; m < NT16; ++m)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      wreg[m][e] = w[(int64_t)min(li, K - 1) * d + min(cw0 + 16 * m + 4 * lq + e, d - 1)];
  if (a.fscale) {  // the buffer holds v = s w: one correctly rounded division per coordinate
#pragma unroll
    for (int m = 0; m < NT16; ++m)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        wreg[m][e] = __fdiv_rn(wreg[m][e], a.fscale[min(cw0 + 16 * m + 4 * lq + e, d - 1)]);
  }
#pragma unroll
  for (int m = 0; m < NT16; ++m)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      asm volatile("" : "+v"(wreg[m][e]));
      if (li >= K || cw0 + 16 * m + 4 * lq + e >= d) wreg[m][e] = 0.f;
    }
  // G[class 4 q + r][cw0 + 32 g + 2 j + e] in component r of gacc[g][e] of lane (j, q): a
  // lane's two accumulator tiles of a group take adjacent columns, so that one 8-byte LDS
  // read feeds both
  F4 gacc[NG][2];
#pragma unroll
  for (int g = 0; g < NG; ++g) gacc[g][0] = gacc[g][1] = F4{0.f, 0.f, 0.f, 0.f};
  double loss_acc = 0.0;

  // Tile fetch: thread t < CW takes float4 number t of each of the 16 rows (CW <= 256), so a
  // row is read by consecutive threads and the addresses need no per-load registers.  Loads
  // are unconditional from clamped addresses; a tile stays in registers while the previous
  // one is multiplied and is written to LDS when that is done.
  F4 xn[kRows];
  int yn = 0;  // label of row tid / 16 of the requested tile
  const int fcol = 4 * min(tid, CW - 1);
  const bool carrier = tid < CW && fcol < d;       // columns past d stay zero in LDS
  const int gcol = min(fcol, (int)ldx - 4);
  const bool whole_cols = (d & 3) == 0;
  for (int k = tid; k < kRows * LDT / 4; k += 256)
    reinterpret_cast<F4*>(s_x)[k] = F4{0.f, 0.f, 0.f, 0.f};
  auto request = [&](int64_t tile) {
    const float* tb = X + tile * kRows * ldx + gcol;
    const int last = (int)min((int64_t)kRows - 1, N - 1 - tile * kRows);  // rows past N read row N - 1
#pragma unroll
    for (int r = 0; r < kRows; ++r)
      xn[r] = __builtin_nontemporal_load(reinterpret_cast<const F4*>(tb + (int64_t)min(r, last) * ldx));
    yn = y[min(tile * kRows + (tid >> 4), N - 1)];
  };
  auto stage = [&](int64_t tile) {
    if (!carrier) return;
    if (whole_cols && (tile + 1) * kRows <= N) {  // nothing to mask
#pragma unroll
      for (int r = 0; r < kRows; ++r) *reinterpret_cast<F4*>(s_x + r * LDT + fcol) = xn[r];
    } else {
#pragma unroll
      for (int r = 0; r < kRows; ++r) {
        const bool in = tile * kRows + r < N;
        F4 v = xn[r];
        if (!in) v = F4{0.f, 0.f, 0.f, 0.f};
        if (fcol + 1 >= d) v.y = 0.f;
        if (fcol + 2 >= d) v.z = 0.f;
        if (fcol + 3 >= d) v.w = 0.f;
        *reinterpret_cast<F4*>(s_x + r * LDT + fcol) = v;
      }
    }
  };

  const int64_t tiles = (N + kRows - 1) / kRows;
  const int64_t step = a.parts;
  int64_t tile = blockIdx.x;
  if (tile < tiles) request(tile);
  __syncthreads();  // the zero fill is complete
  for (; tile < tiles; tile += step) {
    stage(tile);
    const int ycur = yn;
    __syncthreads();
    if (tile + step < tiles) request(tile + step);

    // ---- first product: partial margins of this wave's columns, [16 rows] x [16 classes]
    F4 pa = F4{0.f, 0.f, 0.f, 0.f}, pb = F4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m0 = 0; m0 < NT16; m0 += 4) {  // operand reads four chunks at a time
      F4 xa[4];
#pragma unroll
      for (int m = m0; m < m0 + 4 && m < NT16; ++m)
        xa[m - m0] = *reinterpret_cast<const F4*>(s_x + (size_t)li * LDT + cw0 + 16 * m + 4 * lq);
#pragma unroll
      for (int m = m0; m < m0 + 4 && m < NT16; ++m) {
        pa = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[m - m0].x, wreg[m][0], pa, 0, 0, 0);
        pb = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[m - m0].y, wreg[m][1], pb, 0, 0, 0);
        pa = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[m - m0].z, wreg[m][2], pa, 0, 0, 0);
        pb = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[m - m0].w, wreg[m][3], pb, 0, 0, 0);
      }
    }
    // component r of lane (j, q) is row 4 q + r, class j
    s_pphi[wave][4 * lq + 0][li] = pa.x + pb.x;
    s_pphi[wave][4 * lq + 1][li] = pa.y + pb.y;
    s_pphi[wave][4 * lq + 2][li] = pa.z + pb.z;
    s_pphi[wave][4 * lq + 3][li] = pa.w + pb.w;
    __syncthreads();

    // ---- softmax: thread (row tid / 16, class tid % 16)
    {
      const int r = tid >> 4, c = tid & 15;
      const int64_t row = tile * kRows + r;
      const bool valid = c < K;
      const float logit = ((s_pphi[0][r][c] + s_pphi[1][r][c]) + s_pphi[2][r][c]) + s_pphi[3][r][c];
      const float mx = row_fold(valid ? logit : -INFINITY, [](float x, float y) { return fmaxf(x, y); });
      const float e = valid ? expf(logit - mx) : 0.f;
      const float se = row_fold(e, [](float x, float y) { return x + y; });
      float rc = 0.f;
      if (row < N && valid) {
        rc = e / se - (c == ycur ? 1.0f : 0.f);
        phi[row * K + c] = logit;
        if (c == ycur) loss_acc += (double)(logf(se) + mx - logit);
      }
      s_rt[c * kRtStride + r] = rc;
    }
    __syncthreads();

    // ---- second product: G[:, this wave's columns] += R^T X; contraction index = row 4 q + kk
    {
      typedef float F2 __attribute__((ext_vector_type(2)));
      const F4 rt = *reinterpret_cast<const F4*>(s_rt + li * kRtStride + 4 * lq);
      const float rtk[4] = {rt.x, rt.y, rt.z, rt.w};
#pragma unroll
      for (int g0 = 0; g0 < NG; g0 += 2) {  // operand reads two groups at a time
        F2 xb[2][4];
#pragma unroll
        for (int g = g0; g < g0 + 2 && g < NG; ++g)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            xb[g - g0][kk] = *reinterpret_cast<const F2*>(s_x + (size_t)(4 * lq + kk) * LDT + cw0 + 32 * g + 2 * li);
#pragma unroll
        for (int g = g0; g < g0 + 2 && g < NG; ++g)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            gacc[g][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(rtk[kk], xb[g - g0][kk].x, gacc[g][0], 0, 0, 0);
            gacc[g][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(rtk[kk], xb[g - g0][kk].y, gacc[g][1], 0, 0, 0);
          }
      }
    }
    __syncthreads();  // the tile buffer is free for the next tile
  }

  // ---- partial gradient and loss of this workgroup
  float* pg = a.partial_g + ((int64_t)chain * a.parts + blockIdx.x) * (int64_t)K * d;
#pragma unroll
  for (int g = 0; g < NG; ++g)
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int col = cw0 + 32 * g + 2 * li + e;
      if (col < d) {
        if (4 * lq + 0 < K) pg[(int64_t)(4 * lq + 0) * d + col] = gacc[g][e].x;
        if (4 * lq + 1 < K) pg[(int64_t)(4 * lq + 1) * d + col] = gacc[g][e].y;
        if (4 * lq + 2 < K) pg[(int64_t)(4 * lq + 2) * d + col] = gacc[g][e].z;
        if (4 * lq + 3 < K) pg[(int64_t)(4 * lq + 3) * d + col] = gacc[g][e].w;
      }
    }
  s_loss[tid] = loss_acc;
  __syncthreads();
  if (tid == 0) {
    double l = 0.0;
    for (int t = 0; t < 256; ++t) l += s_loss[t];  // fixed order
    a.partial_loss[(int64_t)chain * a.parts + blockIdx.x] = l;
  }
}

template <int NG>
int launch_ng(const FgArgs& a, int R, hipStream_t s) {
  const size_t smem = (size_t)kRows * (4 * 32 * NG + 8) * sizeof(float);
  auto kern = fullgrad_softmax_mfma<NG>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
    return HALP_ERR_HIP;
  hipLaunchKernelGGL(kern, dim3(a.parts, R), dim3(256), smem, s, a);
  return hip_ok(hipGetLastError());
}

}  // namespace

// K <= 16 classes, d <= 1024 (a wave's quarter of the columns stays in registers)
int fullgrad_softmax_supported(const halp_params& p) {
  if (p.K < 2 || p.K > 16 || p.d > 1024) return HALP_ERR_UNSUPPORTED;
  return HALP_OK;
}

int launch_fullgrad_softmax(const FgArgs& a, int R, hipStream_t s) {
  const int ng = (a.d + 127) / 128;  // groups of 32 columns per wave
  if (ng <= 1) return launch_ng<1>(a, R, s);
  if (ng <= 2) return launch_ng<2>(a, R, s);
  if (ng <= 4) return launch_ng<4>(a, R, s);
  if (ng <= 7) return launch_ng<7>(a, R, s);
  if (ng <= 8) return launch_ng<8>(a, R, s);
  return HALP_ERR_UNSUPPORTED;
}

}  // namespace halp
