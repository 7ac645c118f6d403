// Full-precision pass of a HALP epoch (Algorithm 4, outer lines):
//   phi_i = x_i^T w~   and   g~ = (1/N) sum_i l_i'(phi_i) x_i + lambda w~,
// fused so that every example row crosses HBM once.
//
// One wave owns a row at a time.  A lane holds NV F4 column chunks of the
// row (columns 4*(lane + 64 k)), the same chunks of w~ and of its partial
// gradient, all in registers.  The margin is a lane-local dot product folded
// across the wave with DPP; the residual l'(phi) is then a wave-uniform scalar
// and the gradient update is a broadcast multiply-add.  Rows are fetched one
// batch ahead of the batch being reduced so that loads stay in flight while the
// wave computes.  Waves of a workgroup fold their partial gradients through
// LDS; a second small kernel adds the per-workgroup partials in a fixed order
// (fp64), so the result does not depend on scheduling.
#include <mutex>

#include "halp_device.hpp"
#include "fullgrad_args.hpp"
#include "halp_internal.hpp"

namespace halp {
namespace {

typedef float F4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ F4 make_f4(float a, float b, float c, float d) { return F4{a, b, c, d}; }


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

// Coordinate j of the model the data belong to: with per-feature scales the buffer holds
// v_j = s_j w_j (one correctly rounded division, once per workgroup).
__device__ __forceinline__ float model_coord(const FgArgs& a, const float* w, int j) {
  return a.fscale ? __fdiv_rn(w[j], a.fscale[j]) : w[j];
}

// Loads the chunk at column `col` of a row; columns >= d read as 0.  The row
// stride is a multiple of 4 floats, so a whole F4 is always inside the row.
template <bool EXACT>
__device__ __forceinline__ F4 load_chunk(const float* row, int col, int d) {
  if (EXACT) return __builtin_nontemporal_load(reinterpret_cast<const F4*>(row + col));
  F4 v = make_f4(0.f, 0.f, 0.f, 0.f);
  if (col < d) {
    v = __builtin_nontemporal_load(reinterpret_cast<const F4*>(row + col));
    if (col + 1 >= d) v.y = 0.f;
    if (col + 2 >= d) v.z = 0.f;
    if (col + 3 >= d) v.w = 0.f;
  }
  return v;
}

// ---- K = 1: squared and logistic ---------------------------------------------
// NV chunks per lane, RB rows per batch, two batches in registers.
template <int NV, int RB, int LOSS, bool EXACT>
__global__ __launch_bounds__(256) void fullgrad_k1(FgArgs a) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int chain = blockIdx.y;
  const float* __restrict__ X = a.X + (int64_t)chain * a.x_chain_stride;
  const float* __restrict__ y =
      reinterpret_cast<const float*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const float* __restrict__ w = a.w + (int64_t)chain * a.d;
  float* __restrict__ phi = a.phi + (int64_t)chain * a.N;
  const int d = a.d;
  const int64_t N = a.N, ldx = a.ldx;

  F4 wv[NV], gv[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int col = 4 * (lane + 64 * k);
    wv[k] = make_f4(0.f, 0.f, 0.f, 0.f);
    if (col < d) wv[k].x = model_coord(a, w, col);
    if (col + 1 < d) wv[k].y = model_coord(a, w, col + 1);
    if (col + 2 < d) wv[k].z = model_coord(a, w, col + 2);
    if (col + 3 < d) wv[k].w = model_coord(a, w, col + 3);
    gv[k] = make_f4(0.f, 0.f, 0.f, 0.f);
  }
  double loss_acc = 0.0;

  const int64_t nblk = (N + RB - 1) / RB;
  const int64_t stride = (int64_t)a.parts * 4;
  int64_t bi = (int64_t)blockIdx.x * 4 + wave;

  F4 xa[RB][NV], xb[RB][NV];

  auto load_batch = [&](F4(&xv)[RB][NV], int64_t blk) {
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const int64_t row = blk * RB + r;
      const float* rp = X + row * ldx;
      if (row < N) {
#pragma unroll
        for (int k = 0; k < NV; ++k) xv[r][k] = load_chunk<EXACT>(rp, 4 * (lane + 64 * k), d);
      } else {
#pragma unroll
        for (int k = 0; k < NV; ++k) xv[r][k] = make_f4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };

  auto reduce_batch = [&](F4(&xv)[RB][NV], int64_t blk) {
    float res[RB];
    float mine = 0.f;
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      float p = 0.f;
#pragma unroll
      for (int k = 0; k < NV; ++k) p = dot4(xv[r][k], wv[k], p);
      const float m = wave_sum_f32(p);  // phi_i
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
      if (ok) loss_acc += (double)li;
      if (lane == r) mine = m;
    }
    if (lane < RB && blk * RB + lane < N) phi[blk * RB + lane] = mine;
#pragma unroll
    for (int r = 0; r < RB; ++r) {
#pragma unroll
      for (int k = 0; k < NV; ++k) axpy4(res[r], xv[r][k], gv[k]);
    }
  };

  if (bi < nblk) load_batch(xa, bi);
  while (bi < nblk) {
    const int64_t b1 = bi + stride;
    if (b1 < nblk) load_batch(xb, b1);
    reduce_batch(xa, bi);
    if (b1 >= nblk) break;
    const int64_t b2 = b1 + stride;
    if (b2 < nblk) load_batch(xa, b2);
    reduce_batch(xb, b1);
    bi = b2;
  }

  // fold the four waves' partial gradients in wave order through LDS
  __shared__ F4 fold[64 * NV];
  __shared__ double fold_loss[4];
  if (lane == 0) fold_loss[wave] = loss_acc;
  for (int s = 1; s < 4; ++s) {
    if (wave == s) {
#pragma unroll
      for (int k = 0; k < NV; ++k) fold[lane + 64 * k] = gv[k];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int k = 0; k < NV; ++k) {
        const F4 o = fold[lane + 64 * k];
        gv[k].x += o.x; gv[k].y += o.y; gv[k].z += o.z; gv[k].w += o.w;
      }
    }
    __syncthreads();
  }
  if (wave == 0) {
    float* pg = a.partial_g + ((int64_t)chain * a.parts + blockIdx.x) * (int64_t)d;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int col = 4 * (lane + 64 * k);
      if (col < d) pg[col] = gv[k].x;
      if (col + 1 < d) pg[col + 1] = gv[k].y;
      if (col + 2 < d) pg[col + 2] = gv[k].z;
      if (col + 3 < d) pg[col + 3] = gv[k].w;
    }
    if (lane == 0)
      a.partial_loss[(int64_t)chain * max(a.parts, a.loss_parts) + blockIdx.x] =
          ((fold_loss[0] + fold_loss[1]) + fold_loss[2]) + fold_loss[3];
  }
}

// ---- K = 1, narrow rows (d <= 128) ----------------------------------------------
// A row of up to 4 G floats is held by G lanes (G = 4, 8, 16, 32), so a wave works on 64 / G
// consecutive rows at once -- one coalesced load of 1 KB at d = 4 G -- instead of leaving most
// of its lanes idle.  The margin is folded inside the G lanes only.  RB such row groups make
// a batch; batches are double-buffered as above.
template <typename T>
__device__ __forceinline__ T group_sum(T v, int G) {
  v += dpp_quad_swap1(v);
  v += dpp_quad_swap2(v);
  if (G >= 8) v += dpp_half_mirror(v);
  if (G >= 16) v += dpp_row_mirror(v);
  if (G >= 32) v += __shfl_xor(v, 16);
  return v;
}

template <int G, int RB, int LOSS>
__global__ __launch_bounds__(256) void fullgrad_k1_narrow(FgArgs a) {
  constexpr int RW = 64 / G;       // rows per wave and group
  constexpr int BR = RB * RW;      // rows per batch
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sub = lane % G, rsel = lane / G;
  const int chain = blockIdx.y;
  const float* __restrict__ X = a.X + (int64_t)chain * a.x_chain_stride;
  const float* __restrict__ y =
      reinterpret_cast<const float*>(a.y) + (int64_t)chain * a.y_chain_stride;
  const float* __restrict__ w = a.w + (int64_t)chain * a.d;
  float* __restrict__ phi = a.phi + (int64_t)chain * a.N;
  const int d = a.d;
  const int64_t N = a.N, ldx = a.ldx;
  const int col = 4 * sub;

  F4 wv = make_f4(0.f, 0.f, 0.f, 0.f), gv = make_f4(0.f, 0.f, 0.f, 0.f);
  if (col < d) wv.x = model_coord(a, w, col);
  if (col + 1 < d) wv.y = model_coord(a, w, col + 1);
  if (col + 2 < d) wv.z = model_coord(a, w, col + 2);
  if (col + 3 < d) wv.w = model_coord(a, w, col + 3);
  double loss_acc = 0.0;

  const int64_t nblk = (N + BR - 1) / BR;
  const int64_t stride = (int64_t)a.parts * 4;
  int64_t bi = (int64_t)blockIdx.x * 4 + wave;

  F4 xa[RB], xb[RB];
  auto load_batch = [&](F4(&xv)[RB], int64_t blk) {
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const int64_t row = blk * BR + r * RW + rsel;
      xv[r] = make_f4(0.f, 0.f, 0.f, 0.f);
      if (row < N) xv[r] = load_chunk<false>(X + row * ldx, col, d);
    }
  };
  auto reduce_batch = [&](F4(&xv)[RB], int64_t blk) {
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const float m = group_sum(dot4(xv[r], wv, 0.f), G);  // phi_i, in all G lanes of the row
      const int64_t row = blk * BR + r * RW + rsel;
      const bool ok = row < N;
      const float yi = ok ? y[row] : 0.f;
      float rr, li;
      if (LOSS == HALP_LOSS_SQUARED) {
        rr = m - yi;
        li = 0.5f * rr * rr;
      } else {
        rr = -yi / (1.0f + expf(yi * m));
        const float sgn = -yi * m;
        li = fmaxf(sgn, 0.f) + log1pf(expf(-fabsf(sgn)));
      }
      if (ok && sub == 0) {
        phi[row] = m;
        loss_acc += (double)li;
      }
      axpy4(ok ? rr : 0.f, xv[r], gv);
    }
  };

  if (bi < nblk) load_batch(xa, bi);
  while (bi < nblk) {
    const int64_t b1 = bi + stride;
    if (b1 < nblk) load_batch(xb, b1);
    reduce_batch(xa, bi);
    if (b1 >= nblk) break;
    const int64_t b2 = b1 + stride;
    if (b2 < nblk) load_batch(xa, b2);
    reduce_batch(xb, b1);
    bi = b2;
  }

  // the wave's row groups hold partial gradients of the same columns: add them, group 0 ends
  // up with the wave's sum (a fixed order), likewise the loss
#pragma unroll
  for (int off = 32; off >= G; off >>= 1) {
    gv.x += __shfl_xor(gv.x, off); gv.y += __shfl_xor(gv.y, off);
    gv.z += __shfl_xor(gv.z, off); gv.w += __shfl_xor(gv.w, off);
    loss_acc += __shfl_xor(loss_acc, off);
  }
  __shared__ F4 fold[4][G];
  __shared__ double fold_loss[4];
  if (lane < G) fold[wave][lane] = gv;
  if (lane == 0) fold_loss[wave] = loss_acc;
  __syncthreads();
  if (wave == 0 && lane < G) {
#pragma unroll
    for (int sw = 1; sw < 4; ++sw) {
      const F4 o = fold[sw][lane];
      gv.x += o.x; gv.y += o.y; gv.z += o.z; gv.w += o.w;
    }
    float* pg = a.partial_g + ((int64_t)chain * a.parts + blockIdx.x) * (int64_t)d;
    if (col < d) pg[col] = gv.x;
    if (col + 1 < d) pg[col + 1] = gv.y;
    if (col + 2 < d) pg[col + 2] = gv.z;
    if (col + 3 < d) pg[col + 3] = gv.w;
    if (lane == 0)
      a.partial_loss[(int64_t)chain * max(a.parts, a.loss_parts) + blockIdx.x] =
          ((fold_loss[0] + fold_loss[1]) + fold_loss[2]) + fold_loss[3];
  }
}

// ---- second stage: fixed-order sum of the per-workgroup partials --------------
struct RedArgs {
  const float* partial_g;
  const double* partial_loss;
  int loss_parts;       // partial losses per chain (a row of partial_loss has parts_stride entries)
  int loss_stride;
  const float* w;
  const float* fscale;  // [d] or null: the gradient is handed on as d f / d v_j = g_j / s_j
  float* g;
  double* scales;
  int64_t N;
  int n;  // K*d
  int d;
  int parts;
  double lambda;
};

// A workgroup sums 32 entries: thread (entry tid % 32, group tid / 32) adds every GROUPS-th
// partial in index order, the group sums are then added in group order: a fixed order, with a
// thread's few loads all in flight at once (the pass is as long as its longest chain of waits).
// GROUPS = 32 where a chain has many partials, 8 where it has few (a chain of the headline
// workload has two).
template <int kReduceGroups>
__global__ __launch_bounds__(32 * kReduceGroups) void fullgrad_reduce(RedArgs a) {
  const int chain = blockIdx.y;
  const int e = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int k = blockIdx.x * 32 + e;
  const float* pg = a.partial_g + (int64_t)chain * a.parts * a.n;
  const float* w = a.w + (int64_t)chain * a.n;
  __shared__ double gsum[kReduceGroups][32];
  double s = 0.0;
  if (k < a.n) {
#pragma unroll 8
    for (int p = grp; p < a.parts; p += kReduceGroups) s += (double)pg[(int64_t)p * a.n + k];
  }
  gsum[grp][e] = s;
  __syncthreads();
  if (grp == 0 && k < a.n) {
    double t = gsum[0][e];
#pragma unroll
    for (int q = 1; q < kReduceGroups; ++q) t += gsum[q][e];
    double gk = t / (double)a.N + a.lambda * (double)w[k];
    if (a.fscale) gk = gk / (double)a.fscale[k % a.d];
    a.g[(int64_t)chain * a.n + k] = (float)gk;
  }
  if (blockIdx.x == 0) {  // f(w~): data term plus lambda/2 ||w~||^2
    constexpr int NT = 32 * kReduceGroups;
    __shared__ double red[NT], redl[NT];
    double w2 = 0.0, l = 0.0;  // thread t takes entries t, t + NT, ..; then a tree: a fixed order
    for (int j = threadIdx.x; j < a.n; j += NT) w2 += (double)w[j] * (double)w[j];
    for (int p = threadIdx.x; p < a.loss_parts; p += NT) l += a.partial_loss[(int64_t)chain * a.loss_stride + p];
    red[threadIdx.x] = w2;
    redl[threadIdx.x] = l;
    __syncthreads();
    for (int h = NT / 2; h > 0; h >>= 1) {
      if ((int)threadIdx.x < h) {
        red[threadIdx.x] += red[threadIdx.x + h];
        redl[threadIdx.x] += redl[threadIdx.x + h];
      }
      __syncthreads();
    }
    if (threadIdx.x == 0)
      a.scales[(int64_t)chain * 8 + 6] = redl[0] / (double)a.N + 0.5 * a.lambda * red[0];
  }
}

// ---- dispatch ------------------------------------------------------------------
int nv_for(int d) {
  const int chunks = (d + 255) / 256;  // F4 chunks per lane
  int nv = 1;
  while (nv < chunks) nv *= 2;
  return nv;
}

template <int NV, int RB>
int launch_k1(const FgArgs& a, int loss, bool exact, dim3 grid, hipStream_t s) {
  if (loss == HALP_LOSS_SQUARED) {
    if (exact) hipLaunchKernelGGL((fullgrad_k1<NV, RB, HALP_LOSS_SQUARED, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((fullgrad_k1<NV, RB, HALP_LOSS_SQUARED, false>), grid, dim3(256), 0, s, a);
  } else {
    if (exact) hipLaunchKernelGGL((fullgrad_k1<NV, RB, HALP_LOSS_LOGISTIC, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((fullgrad_k1<NV, RB, HALP_LOSS_LOGISTIC, false>), grid, dim3(256), 0, s, a);
  }
  return hip_ok(hipGetLastError());
}

}  // namespace

// K = 1: a row per wave up to d = 4096, a row across a workgroup's waves up to 16384
int fullgrad_supported(const halp_params& p) {
  if (p.loss == HALP_LOSS_SOFTMAX) return fullgrad_softmax_supported(p);
  return p.d <= fullgrad_k1_wide_max_d() ? HALP_OK : HALP_ERR_UNSUPPORTED;
}

// narrow rows: lanes per row (0 = the row-per-wave kernel) and rows per batch
constexpr int kNarrowGroups = 8;
static int narrow_lanes(int d) {
  if (d > 128) return 0;
  int g = 4;
  while (4 * g < d) g *= 2;
  return g;
}
static int rows_per_batch(int d) {
  if (d > 4096) return fullgrad_k1_wide_rows_per_batch();
  const int g = narrow_lanes(d);
  if (g) return kNarrowGroups * (64 / g);
  const int nv = nv_for(d);
  return nv >= 16 ? 1 : 16 / nv;
}

template <int G>
int launch_narrow(const FgArgs& a, int loss, dim3 grid, hipStream_t s) {
  if (loss == HALP_LOSS_SQUARED)
    hipLaunchKernelGGL((fullgrad_k1_narrow<G, kNarrowGroups, HALP_LOSS_SQUARED>), grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((fullgrad_k1_narrow<G, kNarrowGroups, HALP_LOSS_LOGISTIC>), grid, dim3(256), 0, s, a);
  return hip_ok(hipGetLastError());
}

// workgroups per chain when the caller has not fixed the count: two per CU over all chains
static int fullgrad_auto_parts(const halp_params& p, int num_cus) {
  if (p.loss == HALP_LOSS_SOFTMAX) {  // tiles of 16 rows; one (pipelined form) or two workgroups per CU
    const int64_t tiles = (p.N + 15) / 16;
    int64_t parts;
    if (!fullgrad_softmax_one_pass(p.d)) {  // second pass: a workgroup per row split and column block
      const int ncb = (p.d + kSoftmaxWideBlock - 1) / kSoftmaxWideBlock;
      parts = (2 * (int64_t)num_cus + (int64_t)ncb * p.R - 1) / ((int64_t)ncb * p.R);
    } else {
      const int per_cu = fullgrad_softmax_pipelined(p.d) ? 1 : 2;
      parts = (per_cu * (int64_t)num_cus + p.R - 1) / p.R;
    }
    if (parts > tiles) parts = tiles;
    return (int)(parts < 1 ? 1 : parts);
  }
  const int rb = rows_per_batch(p.d);
  const int64_t nblk = (p.N + rb - 1) / rb;
  const bool wide = p.d > 4096;  // a workgroup of up to 16 waves per CU
  int64_t parts = ((wide ? 1 : 2) * (int64_t)num_cus + p.R - 1) / p.R;  // two workgroups per CU
  const int64_t most = wide ? nblk : (nblk + 3) / 4;                     // one batch per wave at least
  if (parts > most) parts = most;
  if (parts < 1) parts = 1;
  return (int)parts;
}

// workgroups that write a partial loss: the first pass of the two-pass softmax form has its own
// count (two per CU); everywhere else every workgroup of the one kernel writes one
static int fullgrad_auto_loss_parts(const halp_params& p, int num_cus, int parts) {
  if (p.loss != HALP_LOSS_SOFTMAX || fullgrad_softmax_one_pass(p.d)) return parts;
  const int64_t tiles = (p.N + 15) / 16;
  int64_t lp = (2 * (int64_t)num_cus + p.R - 1) / p.R;
  if (lp > tiles) lp = tiles;
  return (int)(lp < 1 ? 1 : lp);
}

int fullgrad_parts(const halp_handle& h) {
  if (h.fullgrad_blocks > 0) return h.fullgrad_blocks;
  return fullgrad_auto_parts(h.p, h.num_cus);
}

bool fullgrad_needs_resid(const halp_params& p) {
  return p.loss == HALP_LOSS_SOFTMAX && !fullgrad_softmax_one_pass(p.d);
}

int fullgrad_loss_parts(const halp_handle& h) {
  if (h.fullgrad_blocks > 0) return h.fullgrad_blocks;
  return fullgrad_auto_loss_parts(h.p, h.num_cus, fullgrad_parts(h));
}

// What a gradient pass needs beyond the parameters: the caller's buffers and a workspace of
// per-workgroup partial sums ([R][parts][K d] floats, [R][parts] doubles).
struct FgPlan {
  const halp_params* p;
  const halp_buffers* buf;
  const float* fscale;
  float* partial_g;
  double* partial_loss;
  int parts;
  int loss_parts;  // entries per chain of partial_loss in use (its rows are max(parts, loss_parts) long)
  float* resid;    // [R][N][16] for the two-pass softmax form, else unused
  const uint32_t* xabsmax = nullptr;  // softmax: bits of the largest |X|, or null (fp32 products)
};

static int launch_full_gradient_plan(const FgPlan& f, hipStream_t s) {
  const halp_params& p = *f.p;
  const halp_buffers& buf = *f.buf;
  int rc = fullgrad_supported(p);
  if (rc != HALP_OK) return rc;
  FgArgs a;
  a.X = buf.X; a.y = buf.y; a.w = buf.w; a.phi = buf.phi;
  a.partial_g = f.partial_g; a.partial_loss = f.partial_loss;
  a.N = p.N; a.ldx = buf.ldx;
  a.x_chain_stride = p.share_data ? 0 : p.N * buf.ldx;
  a.y_chain_stride = p.share_data ? 0 : p.N;
  a.d = p.d; a.K = p.K; a.parts = f.parts; a.fscale = f.fscale;
  a.loss_parts = f.loss_parts; a.resid = f.resid; a.xabsmax = f.xabsmax;
  const dim3 grid(f.parts, p.R);
  const int nv = nv_for(p.d);
  if (p.loss == HALP_LOSS_SOFTMAX) {
    rc = launch_fullgrad_softmax(a, p.R, s);
  } else if (p.d > 4096) {
    rc = launch_fullgrad_k1_wide(a, p.loss, p.R, s);
  } else if (const int g = narrow_lanes(p.d)) {
    switch (g) {
      case 4: rc = launch_narrow<4>(a, p.loss, grid, s); break;
      case 8: rc = launch_narrow<8>(a, p.loss, grid, s); break;
      case 16: rc = launch_narrow<16>(a, p.loss, grid, s); break;
      default: rc = launch_narrow<32>(a, p.loss, grid, s); break;
    }
  } else {
    const bool exact = p.d == 256 * nv;
    switch (nv) {
      case 1: rc = launch_k1<1, 16>(a, p.loss, exact, grid, s); break;
      case 2: rc = launch_k1<2, 8>(a, p.loss, exact, grid, s); break;
      case 4: rc = launch_k1<4, 4>(a, p.loss, exact, grid, s); break;
      case 8: rc = launch_k1<8, 2>(a, p.loss, exact, grid, s); break;
      default: rc = launch_k1<16, 1>(a, p.loss, exact, grid, s); break;
    }
  }
  if (rc != HALP_OK) return rc;
  RedArgs r;
  r.partial_g = f.partial_g; r.partial_loss = f.partial_loss; r.w = buf.w; r.g = buf.g;
  r.scales = buf.scales; r.N = p.N; r.n = p.K * p.d; r.parts = f.parts; r.lambda = p.lambda;
  r.fscale = f.fscale; r.d = p.d;
  r.loss_parts = f.loss_parts; r.loss_stride = f.parts > f.loss_parts ? f.parts : f.loss_parts;
  if (f.parts > 64)
    hipLaunchKernelGGL(fullgrad_reduce<32>, dim3((r.n + 31) / 32, p.R), dim3(32 * 32), 0, s, r);
  else
    hipLaunchKernelGGL(fullgrad_reduce<8>, dim3((r.n + 31) / 32, p.R), dim3(32 * 8), 0, s, r);
  return hip_ok(hipGetLastError());
}

int launch_full_gradient(const halp_handle& h, hipStream_t s) {
  const bool halves = h.xabsmax && h.xabsmax_fresh && !h.gradient_fp32;
  const FgPlan f{&h.p, &h.buf, h.fscale, h.partial_g, h.partial_loss, h.parts, h.loss_parts, h.resid,
                 halves ? h.xabsmax : nullptr};
  return launch_full_gradient_plan(f, s);
}

int prepare_full_gradient(halp_handle& h, hipStream_t s) {
  if (!h.xabsmax || h.xabsmax_fresh || h.gradient_fp32 || !h.buf.X) return HALP_OK;
  // chains with data of their own lie one after the other: N rows each
  const int64_t rows = h.p.share_data ? h.p.N : h.p.N * (int64_t)h.p.R;
  const int rc = launch_absmax(h.buf.X, rows, h.p.d, h.buf.ldx, h.xabsmax, s);
  if (rc == HALP_OK) h.xabsmax_fresh = true;
  return rc;
}

// ---- allocation-free form -------------------------------------------------------
// The workspace of per-workgroup partial sums lives in a file-scope device array instead of
// memory from hipMalloc.  Every GPU holds its own copy of the array at its own address; the
// name below is only a host-side stand-in for it, so the address is looked up once per device
// and that pointer is what the kernels get.  Every launch overwrites the part of the array it
// uses (each workgroup stores its whole partial, zero or not), so nothing has to be cleared;
// two calls in flight on one GPU at once would share the array and race.
static __device__ __align__(256) unsigned char scratch[HALP_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
struct DeviceScratch {
  unsigned char* ptr = nullptr;
  int cus = 0;
};
std::mutex g_scratch_mu;
DeviceScratch g_scratch[kMaxDevices];

// address of this device's copy of `scratch` and its CU count, looked up on first use
int device_scratch(DeviceScratch* out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return HALP_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return HALP_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  DeviceScratch& e = g_scratch[dev];
  if (!e.ptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return HALP_ERR_HIP;
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
      (void)hipGetLastError();
      return HALP_ERR_HIP;
    }
    e.cus = cus > 0 ? cus : 256;
    e.ptr = static_cast<unsigned char*>(ptr);
  }
  *out = e;
  return HALP_OK;
}
}  // namespace

int launch_full_gradient_static(const halp_params& p, const halp_buffers& buf, hipStream_t s) {
  int rc = fullgrad_supported(p);
  if (rc != HALP_OK) return rc;
  // the two-pass softmax form keeps N x 16 residuals between its passes: not in the fixed array
  if (p.loss == HALP_LOSS_SOFTMAX && !fullgrad_softmax_one_pass(p.d)) return HALP_ERR_UNSUPPORTED;
  // bytes one workgroup's partial takes per chain: K d floats and a double
  const size_t n = (size_t)p.K * (size_t)p.d;
  const size_t per_part = (size_t)p.R * (n * sizeof(float) + sizeof(double));
  const size_t budget = (size_t)HALP_STATIC_SCRATCH_BYTES - 256;  // the doubles start 256-aligned
  if (per_part > budget) return HALP_ERR_TOO_LARGE;
  DeviceScratch ds;
  if ((rc = device_scratch(&ds)) != HALP_OK) return rc;
  int64_t parts = fullgrad_auto_parts(p, ds.cus);
  if ((size_t)parts > budget / per_part) parts = (int64_t)(budget / per_part);
  const size_t g_bytes = ((size_t)p.R * (size_t)parts * n * sizeof(float) + 255) / 256 * 256;
  float* partial_g = reinterpret_cast<float*>(ds.ptr);
  double* partial_loss = reinterpret_cast<double*>(ds.ptr + g_bytes);
  const FgPlan f{&p, &buf, nullptr, partial_g, partial_loss, (int)parts, (int)parts, nullptr};
  return launch_full_gradient_plan(f, s);
}

}  // namespace halp
