// Full-precision pass of a HALP epoch for softmax regression (Algorithm 4, outer
// lines, K classes):
//   Phi = X W~^T                      [N x K]   margins
//   R   = softmax(Phi) - onehot(y)    [N x K]   residuals l'
//   G   = R^T X                       [K x d]   gradient sum (the 1/N and lambda W~ come later)
// Both products are dense contractions with one small dimension (K <= 16): they run on the
// matrix cores with the classes padded to 16 -- as fp32 products (v_mfma_f32_16x16x4_f32), or,
// in the pipelined form further down on rows of whole float4s, with every fp32 operand split
// into two halves on the 16-bit path (fp32 accumulation, the accuracy of fp32 products).
//
// First form (rows of 801 .. 1024 coordinates): a workgroup (4 waves) takes tiles of 16 rows.  The tile is fetched from HBM once, with
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
#include <algorithm>
#include <type_traits>

#include "fullgrad_args.hpp"
#include "halp_device.hpp"

namespace halp {
namespace {

typedef float F4 __attribute__((ext_vector_type(4)));
typedef float F16 __attribute__((ext_vector_type(16)));
typedef _Float16 H8 __attribute__((ext_vector_type(8)));
typedef uint32_t U4v __attribute__((ext_vector_type(4)));

// Eight fp32 numbers as two vectors of halves with v = hi + lo up to 2^-22 |v|: hi is v rounded
// to a half, v - hi is exact in fp32, lo is that difference rounded to a half.  Two numbers so
// split multiply as hi hi' + hi lo' + lo hi' (+ lo lo') on the matrix cores' 16-bit path, which
// takes eight times the contraction depth of the fp32 one per instruction, to fp32 accuracy.
// The caller keeps |v| below 2^15; halves below the normal range lose nothing the fp32 sum
// would keep as long as the largest |v| is 2^-3 or more (the matrix cores take subnormal halves
// as they are).
__device__ __forceinline__ void split8(const float (&v)[8], H8& hi, H8& lo) {
  typedef float F2 __attribute__((ext_vector_type(2)));
  typedef _Float16 H2 __attribute__((ext_vector_type(2)));
  uint32_t hu[4], lu[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    hu[p] = __builtin_bit_cast(uint32_t, __builtin_convertvector(F2{v[2 * p], v[2 * p + 1]}, H2));
    float r0, r1;  // v - hi in one instruction each, the half taken from its packed place
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel_hi:[1,0,0]" : "=v"(r0) : "v"(hu[p]), "v"(v[2 * p]));
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r1) : "v"(hu[p]), "v"(v[2 * p + 1]));
    lu[p] = __builtin_bit_cast(uint32_t, __builtin_convertvector(F2{r0, r1}, H2));
  }
  hi = __builtin_bit_cast(H8, U4v{hu[0], hu[1], hu[2], hu[3]});
  lo = __builtin_bit_cast(H8, U4v{lu[0], lu[1], lu[2], lu[3]});
}

// 2^k with max 2^k in [2^13, 2^14), from the bits of max >= 0 (1 for max = 0), and its inverse
__device__ __forceinline__ void half_scale(uint32_t max_bits, float& s, float& inv) {
  const int e = (int)(max_bits >> 23) & 0xff;
  const int f = max_bits == 0 ? 127 : min(267 - e, 253);
  s = __builtin_bit_cast(float, (uint32_t)f << 23);
  inv = __builtin_bit_cast(float, (uint32_t)(254 - f) << 23);
}

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
    a.partial_loss[(int64_t)chain * max(a.parts, a.loss_parts) + blockIdx.x] = l;
  }
}

// ---- pipelined form (d <= 800): specialised waves, three tiles in LDS ---------------------
// One workgroup of eight waves per CU; waves 0-3 (one per SIMD) do the two products, three tile
// buffers of 16 rows in LDS.
//
// Serial form (rows of whole float4s, the 10-class shape): the matrix waves take a tile through
// margins -> softmax (wave w the rows 4w .. 4w+3) -> gradient sum, three barriers that wait for
// LDS traffic only; waves 4-7 do nothing but start tiles on their way from memory straight into
// LDS (global_load_lds, 1 KB per instruction, no registers and no LDS stores) and wait for them:
// tile k+2 is started during period k, a third of its loads beside each phase, into the buffer
// tile k-1 left, and has to be there when period k+1 ends.  With HALVES both products take their
// fp32 operands as pairs of halves (split8 above) on the 16-bit path of the matrix cores:
// 16x16x32 contractions for the margins, 32x32x16 over the tile's rows for the gradient sum,
// fp32 accumulators; without it they are fp32 products (16x16x4).
//
// Overlapped form (other rows, fp32 products): the work on a tile is spread over three periods, a
// period being two halves closed by a barrier each:
//                      half A                               half B
//   matrix waves       margins of tile k (first product)    gradient sum of tile k-1 (second product)
//   helper waves       stage tile k+1 through registers     softmax of tile k -> residuals of tile k
// (requested two tiles ahead, masked on the way into LDS).
//
// Columns are dealt to the matrix waves in groups of 32 (group g to wave g % 4): d = 784 = 24.5
// groups costs the half group only, not a padding of every wave's share.  The group count of a
// wave is a compile-time constant of its loop, so that all operand reads of a tile are issued
// before its first product.
// What bounded the fp32 products: a helper wave that shares a SIMD with a wave issuing them gets
// about one instruction through per product (~30 cycles each, whatever the instruction), and a
// tile's loads are accepted by the memory pipeline over ~1.4 us.
// The compiler may not move instructions across the borders of a phase: left to itself it
// spreads a phase's LDS traffic and address arithmetic into its neighbours, where they queue
// behind the other role's work (measured: 0.80 ms against 0.71 ms at N = 960000).
#define HALP_PHASE_BORDER() __builtin_amdgcn_sched_barrier(0)
constexpr int kPipeMaxD = 800;
constexpr int kPipeGroups = 7;   // groups of 32 columns per matrix wave: 4 x 7 x 32 = 896 >= 800
constexpr int kPipeSlots = 13;   // float4 slots per helper thread and tile: 16 x 200 / 256 = 12.5

// SERIAL: rows of whole float4s (the launch decides); HALVES: the serial form with both products
// on operands split into halves, which needs the largest |X| of the data (FgArgs::xabsmax)
template <bool SERIAL, bool HALVES>
__global__ __launch_bounds__(512) void fullgrad_softmax_pipe(FgArgs a, int LDT) {
  static_assert(SERIAL || !HALVES, "operands in halves exist in the serial form only");
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool matrix_wave = wave < 4;
  const int chain = blockIdx.y;
  const int d = a.d, K = a.K;
  const int64_t N = a.N, ldx = a.ldx;
  const float* __restrict__ X = a.X + (int64_t)chain * a.x_chain_stride;
  const int32_t* __restrict__ y =
      reinterpret_cast<const int32_t*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const float* __restrict__ w = a.w + (int64_t)chain * K * d;
  float* __restrict__ phi = a.phi + (int64_t)chain * N * K;

  // Tiles in dynamic LDS; the small arrays are objects of their own, so that a read of them is
  // known not to touch a tile that is still on its way from memory into LDS.
  extern __shared__ __attribute__((aligned(16))) float s_x[];                       // [3][kRows][LDT]
  __shared__ __attribute__((aligned(16))) float s_pphi[4 * kRows * 16];             // partial margins per matrix wave
  __shared__ __attribute__((aligned(16))) float s_rt[2 * 16 * kRtStride];           // residuals [2][class][row]
  __shared__ __attribute__((aligned(16))) _Float16 s_rp[2 * 16 * kRows];            // residuals in halves [piece][class][row]
  __shared__ uint32_t s_wmax;                                                       // bits of the largest |W~ / s|
  const int tile_floats = kRows * LDT;

  const int li = lane & 15, lq = lane >> 4;
  const int64_t tiles = (N + kRows - 1) / kRows;
  const int64_t step = a.parts;
  // local tile k is global tile blockIdx.x + k step, k = 0 .. n-1
  const int n = blockIdx.x < tiles ? (int)((tiles - blockIdx.x + step - 1) / step) : 0;
  auto tile_of = [&](int k) { return (int64_t)blockIdx.x + (int64_t)k * step; };

  // columns [d, LDT) of every buffer stay zero for the whole pass (staging writes below d only)
  for (int k = tid; k < 3 * kRows * (LDT - d); k += 512) {
    const int r = k / (LDT - d), c = k - r * (LDT - d);
    s_x[r * LDT + d + c] = 0.f;
  }
  // a matrix wave that narrow rows leave without columns never writes its partial margins
  for (int k = tid; k < 4 * kRows * 16; k += 512) s_pphi[k] = 0.f;
  if (tid == 0) s_wmax = 0u;
  __syncthreads();

  // ---------------------------------------------------------------- matrix waves: set-up
  const int ngr = matrix_wave ? max(0, ((d + 31) / 32 - wave + 3) / 4) : 0;  // groups wave, wave+4, ..
  float wreg[kPipeGroups][2][4];
  F4 gacc[kPipeGroups][2];
  // Rows of whole float4s take the serial form of a period (see below): the matrix waves also
  // take the softmax, of four rows each, so `ht` names a matrix thread there
  constexpr bool serial = SERIAL;
  // ---------------------------------------------------------------- helper waves: set-up
  const int ht = (serial && matrix_wave) ? tid : tid - 256;
  const int nf4 = (d + 3) / 4;
  double loss_acc = 0.0;
  if (matrix_wave) {
    // every load unconditional, from a clamped address, and all issued before the first is used
    auto wcol = [&](int i, int c2, int e) { return 32 * (wave + 4 * i) + 16 * c2 + 4 * lq + e; };
#pragma unroll
    for (int i = 0; i < kPipeGroups; ++i)
#pragma unroll
      for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          wreg[i][c2][e] = w[(int64_t)min(li, K - 1) * d + min(wcol(i, c2, e), d - 1)];
    if (a.fscale) {  // the buffer holds v = s w: one correctly rounded division per coordinate
#pragma unroll
      for (int i = 0; i < kPipeGroups; ++i)
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            wreg[i][c2][e] = __fdiv_rn(wreg[i][c2][e], a.fscale[min(wcol(i, c2, e), d - 1)]);
    }
#pragma unroll
    for (int i = 0; i < kPipeGroups; ++i)
#pragma unroll
      for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          asm volatile("" : "+v"(wreg[i][c2][e]));
          if (li >= K || wcol(i, c2, e) >= d) wreg[i][c2][e] = 0.f;
        }
#pragma unroll
    for (int i = 0; i < kPipeGroups; ++i) gacc[i][0] = gacc[i][1] = F4{0.f, 0.f, 0.f, 0.f};
    if constexpr (HALVES) {
      float m = 0.f;
#pragma unroll
      for (int i = 0; i < kPipeGroups; ++i)
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
          for (int e = 0; e < 4; ++e) m = fmaxf(m, fabsf(wreg[i][c2][e]));
      m = row_fold(m, [](float x, float y2) { return fmaxf(x, y2); });
      if (li == 0) atomicMax(&s_wmax, __builtin_bit_cast(uint32_t, m));
    }
  }
  __syncthreads();
  // Operands in halves are scaled by powers of two into the halves' range: W~ by sw (from its
  // largest magnitude, found above), the residuals by 2^13, X by sx -- but only where the data's
  // largest magnitude lies outside [2^-3, 2^15): inside, X is split as it is, and a tile costs
  // one multiplication per element less.
  float sx = 1.f, isx = 1.f, sw = 1.f, isw = 1.f;
  bool x_scaled = false;
  constexpr float kSr = 8192.f, kIsr = 1.f / 8192.f;
  H8 wh[kPipeGroups], wl[kPipeGroups];
  F16 gacc16[kPipeGroups];
  if constexpr (HALVES) {
    const uint32_t xm = *a.xabsmax;
    const int xe = (int)(xm >> 23);
    x_scaled = xm != 0u && (xe < 124 || xe > 141);
    if (x_scaled) half_scale(xm, sx, isx);
    half_scale(s_wmax, sw, isw);
    if (matrix_wave) {
#pragma unroll
      for (int i = 0; i < kPipeGroups; ++i) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = wreg[i][0][e] * sw;
          v[4 + e] = wreg[i][1][e] * sw;
        }
        split8(v, wh[i], wl[i]);
#pragma unroll
        for (int j = 0; j < 16; ++j) gacc16[i][j] = 0.f;
      }
    }
  }

  // matrix waves, first product: partial margins [16 rows] x [16 classes] of this wave's columns.
  // The group count is a compile-time constant (the loop over groups has no branches), so that
  // every operand read of a tile is issued ahead of the products that use it.
  auto margins = [&](auto ngr_c, int buf) {
    constexpr int NGR = decltype(ngr_c)::value;
    const float* xr = s_x + buf * tile_floats + li * LDT + 32 * wave + 4 * lq;
    F4 x0[NGR], x1[NGR];
#pragma unroll
    for (int i = 0; i < NGR; ++i) {
      x0[i] = *reinterpret_cast<const F4*>(xr + 128 * i);
      x1[i] = *reinterpret_cast<const F4*>(xr + 128 * i + 16);
    }
    __builtin_amdgcn_sched_barrier(0);  // all reads are in flight before the first product
    F4 pa = F4{0.f, 0.f, 0.f, 0.f}, pb = F4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NGR; ++i) {
      pa = __builtin_amdgcn_mfma_f32_16x16x4f32(x0[i].x, wreg[i][0][0], pa, 0, 0, 0);
      pb = __builtin_amdgcn_mfma_f32_16x16x4f32(x0[i].y, wreg[i][0][1], pb, 0, 0, 0);
      pa = __builtin_amdgcn_mfma_f32_16x16x4f32(x0[i].z, wreg[i][0][2], pa, 0, 0, 0);
      pb = __builtin_amdgcn_mfma_f32_16x16x4f32(x0[i].w, wreg[i][0][3], pb, 0, 0, 0);
      // the upper 16 columns of the row's last group may be padding only (d = 784: the wave
      // with the most groups): their products are zeros
      if (i + 1 < NGR || 32 * (wave + 4 * i) + 16 < d) {
        pa = __builtin_amdgcn_mfma_f32_16x16x4f32(x1[i].x, wreg[i][1][0], pa, 0, 0, 0);
        pb = __builtin_amdgcn_mfma_f32_16x16x4f32(x1[i].y, wreg[i][1][1], pb, 0, 0, 0);
        pa = __builtin_amdgcn_mfma_f32_16x16x4f32(x1[i].z, wreg[i][1][2], pa, 0, 0, 0);
        pb = __builtin_amdgcn_mfma_f32_16x16x4f32(x1[i].w, wreg[i][1][3], pb, 0, 0, 0);
      }
    }
    // component r of lane (j, q) is row 4 q + r, class j
    float* pp = s_pphi + wave * kRows * 16 + (4 * lq) * 16 + li;
    pp[0] = pa.x + pb.x;
    pp[16] = pa.y + pb.y;
    pp[32] = pa.z + pb.z;
    pp[48] = pa.w + pb.w;
  };
  // matrix waves, second product: G[:, this wave's columns] += R^T X, contraction over the rows
  auto gradient = [&](auto ngr_c, int buf, int par) {
    constexpr int NGR = decltype(ngr_c)::value;
    typedef float F2 __attribute__((ext_vector_type(2)));
    const float* xc = s_x + buf * tile_floats + (4 * lq) * LDT + 32 * wave + 2 * li;
    const F4 rt = *reinterpret_cast<const F4*>(s_rt + par * 16 * kRtStride + li * kRtStride + 4 * lq);
    F2 xb[NGR][4];
#pragma unroll
    for (int i = 0; i < NGR; ++i)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) xb[i][kk] = *reinterpret_cast<const F2*>(xc + kk * LDT + 128 * i);
    const float rtk[4] = {rt.x, rt.y, rt.z, rt.w};
    __builtin_amdgcn_sched_barrier(0);  // all reads are in flight before the first product
#pragma unroll
    for (int i = 0; i < NGR; ++i)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        gacc[i][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(rtk[kk], xb[i][kk].x, gacc[i][0], 0, 0, 0);
        gacc[i][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(rtk[kk], xb[i][kk].y, gacc[i][1], 0, 0, 0);
      }
  };
  // The same two products on operands in halves.  First product: a group of 32 columns is one
  // 16x16x32 contraction per pair of pieces; lane (row j, q) holds columns 4q .. 4q+3 and
  // 16+4q .. 16+4q+3 of the group on both sides.  lo lo' is left out: 2^-22 of the product.
  auto margins_h = [&](auto ngr_c, auto scaled_c, int buf) {
    constexpr int NGR = decltype(ngr_c)::value;
    constexpr bool SCALED = decltype(scaled_c)::value;
    const float* xr = s_x + buf * tile_floats + li * LDT + 32 * wave + 4 * lq;
    F4 x0[NGR], x1[NGR];
#pragma unroll
    for (int i = 0; i < NGR; ++i) {
      x0[i] = *reinterpret_cast<const F4*>(xr + 128 * i);
      x1[i] = *reinterpret_cast<const F4*>(xr + 128 * i + 16);
    }
    __builtin_amdgcn_sched_barrier(0);  // all reads are in flight before the first conversion
    F4 pa = F4{0.f, 0.f, 0.f, 0.f}, pb = F4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NGR; ++i) {
      float v[8] = {x0[i].x, x0[i].y, x0[i].z, x0[i].w, x1[i].x, x1[i].y, x1[i].z, x1[i].w};
      if constexpr (SCALED) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= sx;
      }
      H8 ah, al;
      split8(v, ah, al);
      pa = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, wh[i], pa, 0, 0, 0);
      pb = __builtin_amdgcn_mfma_f32_16x16x32_f16(al, wh[i], pb, 0, 0, 0);
      pb = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, wl[i], pb, 0, 0, 0);
    }
    // component r of lane (j, q) is row 4 q + r, class j
    float* pp = s_pphi + wave * kRows * 16 + (4 * lq) * 16 + li;
    pp[0] = ((pa.x + pb.x) * isx) * isw;
    pp[16] = ((pa.y + pb.y) * isx) * isw;
    pp[32] = ((pa.z + pb.z) * isx) * isw;
    pp[48] = ((pa.w + pb.w) * isx) * isw;
  };
  // Second product, G^T[column][class] += X^T R as 32x32x16 contractions over the tile's rows:
  // lane (m, h) holds column m of a group, rows 8h .. 8h+7, and of the residuals class m % 16,
  // piece m / 16, the same rows: the upper and the lower piece of R are 16 columns each of one
  // right operand, so two contractions (the pieces of X) give all four products of pieces.
  const int gm = lane & 31, gh = lane >> 5;
  auto gradient_h = [&](auto ngr_c, auto scaled_c, int buf) {
    constexpr int NGR = decltype(ngr_c)::value;
    constexpr bool SCALED = decltype(scaled_c)::value;
    const float* xc = s_x + buf * tile_floats + (8 * gh) * LDT + 32 * wave + gm;
    const H8 rb = *reinterpret_cast<const H8*>(s_rp + gm * kRows + 8 * gh);
    float xv[NGR][8];
#pragma unroll
    for (int i = 0; i < NGR; ++i)
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) xv[i][kk] = xc[kk * LDT + 128 * i];
    __builtin_amdgcn_sched_barrier(0);  // all reads are in flight before the first conversion
#pragma unroll
    for (int i = 0; i < NGR; ++i) {
      float v[8];
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) v[kk] = SCALED ? xv[i][kk] * sx : xv[i][kk];
      H8 ah, al;
      split8(v, ah, al);
      gacc16[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, rb, gacc16[i], 0, 0, 0);
      gacc16[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, rb, gacc16[i], 0, 0, 0);
    }
  };
  // helper waves: thread (row ht / 16, class ht % 16).  Every instruction here competes with
  // the matrix waves for the SIMD, so the transcendental steps are single hardware instructions
  // (2^x, log2, reciprocal: 1 ulp each, far inside the pass's 1e-5) and nothing branches.
  const int phi_off = (ht >> 4) * K + (ht & 15);
  auto softmax = [&](int64_t tile, int par, int ycur) {
    const int r = ht >> 4, c = ht & 15;
    const bool valid = c < K;
    const float* pp = s_pphi + r * 16 + c;
    const float logit = ((pp[0] + pp[kRows * 16]) + pp[2 * kRows * 16]) + pp[3 * kRows * 16];
    const float mx = row_fold(valid ? logit : -INFINITY, [](float x, float y2) { return fmaxf(x, y2); });
    const float e = valid ? __builtin_amdgcn_exp2f((logit - mx) * 1.4426950408889634f) : 0.f;
    const float se = row_fold(e, [](float x, float y2) { return x + y2; });
    const bool live = valid && tile * kRows + r < N;
    const bool mine = c == ycur;
    const float rc = live ? e * __builtin_amdgcn_rcpf(se) - (mine ? 1.0f : 0.f) : 0.f;
    if (live) (phi + tile * kRows * K)[phi_off] = logit;
    loss_acc += (live && mine) ? (double)(__builtin_amdgcn_logf(se) * 0.6931471805599453f + mx - logit) : 0.0;
    if constexpr (HALVES) {  // pieces [piece][class][row], scaled into the halves' range
      const float rs = rc * kSr;
      const _Float16 rh = (_Float16)rs;
      s_rp[c * kRows + r] = rh;
      s_rp[16 * kRows + c * kRows + r] = (_Float16)(rs - (float)rh);
    } else {
      s_rt[par * 16 * kRtStride + c * kRtStride + r] = rc;
    }
  };

  // Two loops, one per role, with the same barriers at the same places: the registers of the
  // two roles (W~ slice and gradient accumulators there, a tile in flight here) never live together.
  if (matrix_wave) {
    auto periods = [&](auto ngr_c) {
      int bprev = 1, bcur = 2, bnext = 0;  // buffers of tiles k - 1, k, k + 1 (tile k in buffer k mod 3)
      for (int k = -1; k <= n; ++k) {
        HALP_PHASE_BORDER();
        if (k >= 0 && k < n) margins(ngr_c, bcur);
        HALP_PHASE_BORDER();
        __syncthreads();
        HALP_PHASE_BORDER();
        if (k >= 1) gradient(ngr_c, bprev, (k - 1) & 1);
        HALP_PHASE_BORDER();
        __syncthreads();
        HALP_PHASE_BORDER();
        const int t = bprev; bprev = bcur; bcur = bnext; bnext = t;
      }
    };
    // Serial form (rows that travel by global_load_lds): margins, softmax and gradient sum of a
    // tile follow each other inside one period, all on the matrix waves (wave w takes the softmax
    // of rows 4w .. 4w+3).  The matrix pipe idles through the softmax and three barriers, but no
    // other wave competes with the matrix waves for their SIMDs, and a tile buffer is busy for
    // one period instead of two: with three buffers a tile has two periods to arrive.
    auto lds_barrier = [&]() {  // LDS traffic only: never waits for stores or loads in flight
      HALP_PHASE_BORDER();
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __builtin_amdgcn_s_barrier();
      HALP_PHASE_BORDER();
    };
    auto periods_serial = [&](auto ngr_c, auto scaled_c) {
      constexpr int NGR = decltype(ngr_c)::value;
      int y_cur = 0, y_nxt = n > 0 ? y[min(tile_of(0) * kRows + (ht >> 4), N - 1)] : 0;
      int buf = 0;
      lds_barrier();  // tile 0 has landed
      for (int k = 0; k < n; ++k) {
        y_cur = y_nxt;
        if (k + 1 < n) y_nxt = y[min(tile_of(k + 1) * kRows + (ht >> 4), N - 1)];
        if constexpr (NGR > 0) {
          if constexpr (HALVES) margins_h(ngr_c, scaled_c, buf);
          else margins(ngr_c, buf);
        }
        lds_barrier();
        softmax(tile_of(k), 0, y_cur);
        lds_barrier();
        if constexpr (NGR > 0) {
          if constexpr (HALVES) gradient_h(ngr_c, scaled_c, buf);
          else gradient(ngr_c, buf, 0);
        }
        lds_barrier();  // the buffer is free, the next tile has landed
        buf = buf == 2 ? 0 : buf + 1;
      }
    };
    if constexpr (serial) {
      auto by_groups = [&](auto scaled_c) {
        switch (ngr) {
          case 7: periods_serial(std::integral_constant<int, 7>{}, scaled_c); break;
          case 6: periods_serial(std::integral_constant<int, 6>{}, scaled_c); break;
          case 5: periods_serial(std::integral_constant<int, 5>{}, scaled_c); break;
          case 4: periods_serial(std::integral_constant<int, 4>{}, scaled_c); break;
          case 3: periods_serial(std::integral_constant<int, 3>{}, scaled_c); break;
          case 2: periods_serial(std::integral_constant<int, 2>{}, scaled_c); break;
          case 1: periods_serial(std::integral_constant<int, 1>{}, scaled_c); break;
          default: periods_serial(std::integral_constant<int, 0>{}, scaled_c); break;
        }
      };
      if constexpr (HALVES) {
        if (x_scaled) by_groups(std::true_type{});
        else by_groups(std::false_type{});
      } else {
        by_groups(std::false_type{});
      }
    } else
    switch (ngr) {  // same barriers in every case
      case 7: periods(std::integral_constant<int, 7>{}); break;
      case 6: periods(std::integral_constant<int, 6>{}); break;
      case 5: periods(std::integral_constant<int, 5>{}); break;
      case 4: periods(std::integral_constant<int, 4>{}); break;
      case 3: periods(std::integral_constant<int, 3>{}); break;
      case 2: periods(std::integral_constant<int, 2>{}); break;
      case 1: periods(std::integral_constant<int, 1>{}); break;
      default:  // narrow rows leave this wave without columns: it only keeps the barriers
        for (int k = -1; k <= n; ++k) {
          __syncthreads();
          __syncthreads();
        }
        break;
    }
    // partial gradient of this workgroup
    float* pg = a.partial_g + ((int64_t)chain * a.parts + blockIdx.x) * (int64_t)K * d;
    if constexpr (HALVES) {
      // component j of lane (m, h) is column 8 (j / 4) + 4 h + j % 4 of the group, class m % 16,
      // piece m / 16 of R: the two pieces are 16 lanes apart
#pragma unroll
      for (int i = 0; i < kPipeGroups; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const float v = gacc16[i][j];
          const float t = ((v + __shfl_xor(v, 16)) * kIsr) * isx;
          const int col = 32 * (wave + 4 * i) + 8 * (j >> 2) + 4 * gh + (j & 3);
          if (gm < K && col < d) pg[(int64_t)gm * d + col] = t;
        }
    } else
#pragma unroll
    for (int i = 0; i < kPipeGroups; ++i)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int col = 32 * (wave + 4 * i) + 2 * li + e;
        if (col < d) {
          if (4 * lq + 0 < K) pg[(int64_t)(4 * lq + 0) * d + col] = gacc[i][e].x;
          if (4 * lq + 1 < K) pg[(int64_t)(4 * lq + 1) * d + col] = gacc[i][e].y;
          if (4 * lq + 2 < K) pg[(int64_t)(4 * lq + 2) * d + col] = gacc[i][e].z;
          if (4 * lq + 3 < K) pg[(int64_t)(4 * lq + 3) * d + col] = gacc[i][e].w;
        }
      }
  } else {
    // A tile is 16 nf4 float4s, row after row; thread ht moves float4 number ht + 256 s for
    // s < NS (a wave reads 1 KB of consecutive addresses per instruction; slots past the tile
    // repeat its last float4: the same data to the same place).  Tile k + 1 is staged in period k
    // from register set (k + 1) mod 2, which then takes the request for tile k + 3: two tiles
    // are always on their way from memory.  Offsets are bytes from a base that is the same for
    // the whole wave, so a load or a store is one instruction.
    auto helper = [&](auto ns_c) {
      constexpr int NS = decltype(ns_c)::value;
      uint32_t gofs[NS], lofs[NS];
#pragma unroll
      for (int s2 = 0; s2 < NS; ++s2) {
        const int f = min(ht + 256 * s2, kRows * nf4 - 1);
        const int r = f / nf4, c4 = f - r * nf4;
        gofs[s2] = (uint32_t)(r * (int)ldx + 4 * c4) * 4u;
        lofs[s2] = (uint32_t)(r * LDT + 4 * c4) * 4u;
      }
      F4 xn[2][NS];
      int y_req[2] = {0, 0}, y_staged = 0, y_soft = 0;  // labels of row ht / 16: tiles requested / staged / in softmax
      const uint32_t row_bytes = (uint32_t)ldx * 4u, lds_row_bytes = (uint32_t)LDT * 4u;
      auto request = [&](auto set_c, int64_t tile) {
        constexpr int S = decltype(set_c)::value;
        const char* tb = reinterpret_cast<const char*>(X + tile * kRows * ldx);
        const int rows_in = (int)min((int64_t)kRows, N - tile * kRows);
        if (rows_in == kRows) {
#pragma unroll
          for (int s2 = 0; s2 < NS; ++s2)
            xn[S][s2] = __builtin_nontemporal_load(reinterpret_cast<const F4*>(tb + gofs[s2]));
        } else {  // the last tile: rows past N read row N - 1 (zeroed when staged)
#pragma unroll
          for (int s2 = 0; s2 < NS; ++s2) {
            const int r = (int)(lofs[s2] / lds_row_bytes);
            const uint32_t back = r >= rows_in ? (uint32_t)(r - (rows_in - 1)) * row_bytes : 0u;
            xn[S][s2] = __builtin_nontemporal_load(reinterpret_cast<const F4*>(tb + (gofs[s2] - back)));
          }
        }
        y_req[S] = y[min(tile * kRows + (ht >> 4), N - 1)];
      };
      auto stage = [&](auto set_c, int buf, int64_t tile) {
        constexpr int S = decltype(set_c)::value;
        char* dst = reinterpret_cast<char*>(s_x + buf * tile_floats);
        const int rows_in = (int)min((int64_t)kRows, N - tile * kRows);
        if ((d & 3) == 0 && rows_in == kRows) {
#pragma unroll
          for (int s2 = 0; s2 < NS; ++s2) *reinterpret_cast<F4*>(dst + lofs[s2]) = xn[S][s2];
        } else {
#pragma unroll
          for (int s2 = 0; s2 < NS; ++s2) {
            const int r = (int)(lofs[s2] / lds_row_bytes);
            const int c0 = (int)(lofs[s2] - (uint32_t)r * lds_row_bytes) / 4;
            F4 v = xn[S][s2];
            if (r >= rows_in) v = F4{0.f, 0.f, 0.f, 0.f};
            if (c0 + 1 >= d) v.y = 0.f;
            if (c0 + 2 >= d) v.z = 0.f;
            if (c0 + 3 >= d) v.w = 0.f;
            *reinterpret_cast<F4*>(dst + lofs[s2]) = v;
          }
        }
      };
      // Requests are unconditional (past this workgroup's last tile they re-read the matrix's last
      // tile and are never staged), so that the number of loads in flight is the same in every
      // period and a wait for the older set does not have to wait for the younger one as well.
      auto clamped = [&](int k) { return min(tile_of(k), tiles - 1); };
      request(std::integral_constant<int, 0>{}, clamped(0));
      request(std::integral_constant<int, 1>{}, clamped(1));
      int bnext = 0;
      auto period = [&](auto set_c, int k) {
        y_soft = y_staged;
        if (k + 1 < n) {
          stage(set_c, bnext, tile_of(k + 1));
          y_staged = y_req[decltype(set_c)::value];
        }
        request(set_c, clamped(k + 3));
        __syncthreads();
        if (k >= 0 && k < n) softmax(tile_of(k), k & 1, y_soft);
        __syncthreads();
        bnext = bnext == 2 ? 0 : bnext + 1;
      };
      for (int k = -1; k <= n; k += 2) {
        period(std::integral_constant<int, 0>{}, k);
        if (k + 1 <= n) period(std::integral_constant<int, 1>{}, k + 1);
      }
    };
    // Rows that are whole float4s go from memory straight into LDS (no registers, no stores
    // from this wave): a padded tile is cut into blocks of 64 float4 slots = 1 KB of LDS; helper
    // wave hw moves blocks hw, hw + 4, ..; a lane's slot names the float4 of the matrix it holds
    // (a slot in a row's padding repeats the row's last float4, so the padding holds finite
    // numbers; the padding meets zeros of W~ in the first product and columns that are never
    // stored in the second).  One tile is on its way while the two before it are multiplied; it has
    // landed when the period's closing barrier (which waits for it) is passed.
    auto helper_dma = [&]() {
      const int row_f4 = LDT / 4, total = kRows * row_f4;
      const int nblocks = (total + 63) / 64;
      const int hw = wave - 4;
      const uint32_t row_bytes = (uint32_t)ldx * 4u;
      uint32_t gofs[kPipeSlots];
#pragma unroll
      for (int s2 = 0; s2 < kPipeSlots; ++s2) {
        const int q = min(64 * (hw + 4 * s2) + lane, total - 1);
        const int r = q / row_f4, c4 = min(q - r * row_f4, nf4 - 1);
        gofs[s2] = (uint32_t)(r * (int)ldx + 4 * c4) * 4u;
      }
      typedef __attribute__((address_space(1))) const void* GPtr;
      typedef __attribute__((address_space(3))) void* LPtr;
      const int nbw = max(0, (nblocks - hw + 3) / 4);  // blocks of this wave
      // lanes of this wave's last block that lie inside the tile (64: all)
      const int last_lanes = nbw > 0 ? min(64, total - 64 * (hw + 4 * (nbw - 1))) : 0;
      // the block count is a compile-time constant: a whole tile takes one m0 update and one load
      // per block, with nothing else in between
      auto run = [&](auto nbw_c) {
        constexpr int NBW = decltype(nbw_c)::value;
        // blocks [LO, HI) of this wave's share of a tile
        auto dma_part = [&](auto lo_c, auto hi_c, int buf, int64_t tile) {
          constexpr int LO = decltype(lo_c)::value, HI = decltype(hi_c)::value;
          const char* tb = reinterpret_cast<const char*>(X + tile * kRows * ldx);
          char* lb = reinterpret_cast<char*>(s_x + buf * tile_floats) + 1024 * hw;
          const int rows_in = (int)min((int64_t)kRows, N - tile * kRows);
          if (rows_in == kRows) {
#pragma unroll
            for (int s2 = LO; s2 < HI; ++s2)
              if (s2 + 1 < NBW || lane < last_lanes)
                __builtin_amdgcn_global_load_lds((GPtr)(tb + gofs[s2]), (LPtr)(lb + 4096 * s2), 16, 0, 2);
          } else {  // the last tile: rows past N repeat row N - 1 (their residuals are 0)
#pragma unroll
            for (int s2 = LO; s2 < HI; ++s2) {
              uint32_t go = gofs[s2];
              const int r = (int)(go / row_bytes);
              if (r >= rows_in) go -= (uint32_t)(r - (rows_in - 1)) * row_bytes;
              if (s2 + 1 < NBW || lane < last_lanes)
                __builtin_amdgcn_global_load_lds((GPtr)(tb + go), (LPtr)(lb + 4096 * s2), 16, 0, 2);
            }
          }
        };
        typedef std::integral_constant<int, 0> C0;
        typedef std::integral_constant<int, (NBW + 2) / 3> C1;
        typedef std::integral_constant<int, (2 * NBW + 2) / 3> C2;
        typedef std::integral_constant<int, NBW> C3;
        auto dma = [&](int buf, int64_t tile) { dma_part(C0{}, C3{}, buf, tile); };
        // s_waitcnt for "at most NBW loads in flight" (the youngest tile), every other counter left alone
        constexpr int kLeaveOne = (NBW & 0xF) | (0x7 << 4) | (0xF << 8) | ((NBW >> 4) << 14);
        auto bare_barrier = [&]() {  // never waits for the tiles in flight
          HALP_PHASE_BORDER();
          __builtin_amdgcn_s_waitcnt(0xc07f);
          __builtin_amdgcn_s_barrier();
          HALP_PHASE_BORDER();
        };
        auto landed = [&](bool younger_in_flight) {  // every tile but the youngest has arrived
          HALP_PHASE_BORDER();
          if (younger_in_flight) __builtin_amdgcn_s_waitcnt(kLeaveOne);
          else __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
          HALP_PHASE_BORDER();
        };
        // tile k in buffer k mod 3; tile k + 2 is started at the top of period k, into the buffer
        // that tile k - 1 left at the end of period k - 1, and has to be there when period k + 1 ends
        if (n > 0) dma(0, tile_of(0));
        if (n > 1) dma(1, tile_of(1));
        landed(n > 1);
        bare_barrier();
        int b2 = 2;
        for (int k = 0; k < n; ++k) {
          // the next tile but one is started in three parts, one beside each phase of the matrix
          // waves: no barrier then waits for a whole tile's loads to be issued
          if (k + 2 < n) dma_part(C0{}, C1{}, b2, tile_of(k + 2));
          bare_barrier();
          if (k + 2 < n) dma_part(C1{}, C2{}, b2, tile_of(k + 2));
          bare_barrier();
          if (k + 2 < n) dma_part(C2{}, C3{}, b2, tile_of(k + 2));
          landed(k + 2 < n);
          bare_barrier();
          b2 = b2 == 2 ? 0 : b2 + 1;
        }
      };
      switch (nbw) {
        case 13: run(std::integral_constant<int, 13>{}); break;
        case 12: run(std::integral_constant<int, 12>{}); break;
        case 11: run(std::integral_constant<int, 11>{}); break;
        case 10: run(std::integral_constant<int, 10>{}); break;
        case 9: run(std::integral_constant<int, 9>{}); break;
        case 8: run(std::integral_constant<int, 8>{}); break;
        case 7: run(std::integral_constant<int, 7>{}); break;
        case 6: run(std::integral_constant<int, 6>{}); break;
        case 5: run(std::integral_constant<int, 5>{}); break;
        case 4: run(std::integral_constant<int, 4>{}); break;
        case 3: run(std::integral_constant<int, 3>{}); break;
        case 2: run(std::integral_constant<int, 2>{}); break;
        case 1: run(std::integral_constant<int, 1>{}); break;
        default: run(std::integral_constant<int, 0>{}); break;
      }
    };
    const int nslots = (kRows * nf4 + 255) / 256;
    if constexpr (serial) helper_dma();
    else if (nslots <= 2) helper(std::integral_constant<int, 2>{});
    else if (nslots <= 7) helper(std::integral_constant<int, 7>{});
    else helper(std::integral_constant<int, kPipeSlots>{});
  }
  // every read of the margins' LDS lies before the loop's last barrier: it carries the loss terms now
  double* s_loss = reinterpret_cast<double*>(s_pphi);  // 256 doubles in the 4 KB of the margins
  if (serial ? matrix_wave : !matrix_wave) s_loss[ht] = loss_acc;
  __syncthreads();
  if (tid == 256) {
    double l = 0.0;
    for (int t = 0; t < 256; ++t) l += s_loss[t];  // fixed order
    a.partial_loss[(int64_t)chain * max(a.parts, a.loss_parts) + blockIdx.x] = l;
  }
}

#undef HALP_PHASE_BORDER

int launch_pipe(const FgArgs& a, int R, hipStream_t s) {
  const int LDT = (a.d + 31) / 32 * 32 + 8;  // 8 mod 16: the 8-byte reads of the second product
                                             // (rows 4 apart per half-wave) do not collide
  const size_t smem = (size_t)3 * kRows * LDT * sizeof(float);  // 155136 bytes at most; 6.6 KB more are static
  const bool serial = (a.d & 3) == 0;
  auto kern = !serial ? fullgrad_softmax_pipe<false, false>
                      : (a.xabsmax ? fullgrad_softmax_pipe<true, true> : fullgrad_softmax_pipe<true, false>);
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
    return HALP_ERR_HIP;
  hipLaunchKernelGGL(kern, dim3(a.parts, R), dim3(512), smem, s, a, LDT);
  return hip_ok(hipGetLastError());
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

// K <= 16 classes; d <= 1024 in one pass (a wave's quarter of the columns stays in registers),
// wider rows in two
int fullgrad_softmax_supported(const halp_params& p) {
  if (p.K < 2 || p.K > 16) return HALP_ERR_UNSUPPORTED;
  return HALP_OK;
}

bool fullgrad_softmax_one_pass(int d) { return d <= 1024; }

bool fullgrad_softmax_pipelined(int d) { return d <= kPipeMaxD; }

bool fullgrad_softmax_wants_absmax(int d) { return fullgrad_softmax_pipelined(d) && (d & 3) == 0; }

namespace {
constexpr int kAbsmaxBlocks = 2048;
__global__ __launch_bounds__(256) void absmax_zero(uint32_t* out) { *out = 0u; }
// largest |X[r][c]|, rows of whole float4s: bit patterns of non-negative floats order like the numbers
__global__ __launch_bounds__(256) void absmax_kernel(const float* __restrict__ X, int64_t rows, int nf4,
                                                     int64_t ldx, uint32_t* out) {
  float m = 0.f;
  const int64_t total = rows * nf4;
  for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < total; k += (int64_t)gridDim.x * 256) {
    const int64_t r = k / nf4;
    const int c4 = (int)(k - r * nf4);
    const F4 v = *reinterpret_cast<const F4*>(X + r * ldx + 4 * c4);
    m = fmaxf(fmaxf(m, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
  }
  uint32_t b = __builtin_bit_cast(uint32_t, m);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) b = max(b, (uint32_t)__shfl_xor((int)b, o));
  if ((threadIdx.x & 63) == 0) atomicMax(out, b);
}
}  // namespace

int launch_absmax(const float* X, int64_t rows, int d, int64_t ldx, uint32_t* out, hipStream_t s) {
  if ((d & 3) != 0) return HALP_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(absmax_zero, dim3(1), dim3(1), 0, s, out);
  const int64_t total = rows * (d / 4);
  const int blocks = (int)std::min<int64_t>(kAbsmaxBlocks, (total + 255) / 256);
  if (blocks > 0)
    hipLaunchKernelGGL(absmax_kernel, dim3(blocks), dim3(256), 0, s, X, rows, d / 4, ldx, out);
  return hip_ok(hipGetLastError());
}

int launch_fullgrad_softmax(const FgArgs& a, int R, hipStream_t s) {
  if (!fullgrad_softmax_one_pass(a.d)) return launch_fullgrad_softmax_wide(a, R, s);
  if (fullgrad_softmax_pipelined(a.d)) return launch_pipe(a, R, s);
  const int ng = (a.d + 127) / 128;  // groups of 32 columns per wave
  if (ng <= 1) return launch_ng<1>(a, R, s);
  if (ng <= 2) return launch_ng<2>(a, R, s);
  if (ng <= 4) return launch_ng<4>(a, R, s);
  if (ng <= 7) return launch_ng<7>(a, R, s);
  if (ng <= 8) return launch_ng<8>(a, R, s);
  return HALP_ERR_UNSUPPORTED;
}

}  // namespace halp
