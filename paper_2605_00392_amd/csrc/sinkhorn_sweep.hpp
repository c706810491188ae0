// Sinkhorn (Appendix C) for images whose kernel matrix is too large for one
// workgroup's registers (more than 512 kept or 64 pruned tokens: tiled pages,
// other OCR models' 1000-4500 tokens).  The matrix K = exp((S - shift)/eps)
// stays in memory (packed M x R, fp64) and every iteration streams it ONCE:
//
//   k_sweep_rows   workgroup = 16 rows of one image, all columns, in registers
//                  (thread t holds columns t, t + 512, ...).  Row sums with the
//                  current y give x for the 16 rows (u-update); with the strip
//                  still in registers, the strip's share of every column sum
//                  sum_i K_ij x_i is formed and written out.
//   k_sweep_cols   adds the strips' shares per column and takes y (v-update).
//
// The dustbin row, column and corner all equal kz = exp((z - shift)/eps) and are
// handled in closed form: with sx = sum_i x_i, sy = sum_j y_j,
//   x_i = 1 / (sum_j K_ij y_j + kz y_d),   x_d = R / (kz (sy + y_d)),
//   y_j = 1 / (sum_i K_ij x_i + kz x_d),   y_d = M / (kz (sx + x_d)).
// Sums over strips and blocks are taken in index order, so results do not depend
// on scheduling.  Scalars that one launch writes and the same launch's other
// workgroups still read (sy, y_d) are double-buffered by iteration parity.
#pragma once
#include "common.hpp"
#include "sinkhorn_team.hpp"
#include "sinkhorn_wave.hpp"

namespace rtp {

constexpr int kSweepRows = 16;          // rows per workgroup of k_sweep_rows
constexpr int kSweepThreads = 512;
constexpr int kSweepChunks = 4;         // columns per thread
constexpr int kSweepMaxR = kSweepThreads * kSweepChunks;
static_assert(kSweepMaxR == kSweepMaxPruned, "shape limit");
constexpr int kSweepCols = 64;          // columns per workgroup of k_sweep_cols
constexpr int kSweepColGroups = 4;      // waves of that workgroup, each with a share of the strips
constexpr int kSweepColThreads = 64 * kSweepColGroups;

struct SweepArgs {
  const int32_t* offsets;
  const int32_t* keep;
  const long long* plan_offsets;
  const int32_t* work;    // work lists (k_classify)
  int B;
  DevParams p;
  const double* kmat;
  long long plan_cap;
  double* x;        // [total] x of kept rank i of image b at offsets[b] + i
  double* y;        // [total] y of pruned rank j at offsets[b] + j
  double* colpart;  // strips' column shares: image b, strip s, column j at strip_base(b) + s r + j
  double* xpart;    // [total] strip sums of x at offsets[b] + strip
  double* ysum;     // [2][total] block sums of y at offsets[b] + block, by parity
  double* ydust;    // [2][B] by parity
  float* bestv;     // per strip and column: largest plan entry and its row (indexing of colpart)
  int32_t* besti;
  long long total;
  float* plan_out;     // may be null
  int32_t* pair_out;   // may be null
};

// Where image b's per-strip arrays start: ceil(m/16) r <= m r / 16 + r entries
// fit between consecutive bases because n = m + r > 15 r / 16 + 1.
__device__ __forceinline__ long long strip_base(long long plan_offset, int lo) { return plan_offset / kSweepRows + lo; }

struct SweepImage {
  int b, lo, m, r;
  long long po;
};
__device__ __forceinline__ bool sweep_image(const SweepArgs& A, int idx, SweepImage& I) {
  if (idx >= A.work[kVariantSweep]) return false;
  I.b = A.work[kWorkLists + kVariantSweep * A.B + idx];
  I.lo = A.offsets[I.b];
  const int n = A.offsets[I.b + 1] - I.lo;
  I.m = min(max(A.keep[I.b], 0), n);
  I.r = n - I.m;
  if (I.r <= 0 || I.m <= 0 || I.r > kSweepMaxR) return false;
  I.po = A.plan_offsets[I.b];
  return plan_fits(I.po, I.m, I.r, A.plan_cap);
}

// u = v = 0: x = exp(shift/eps) (so that x K y = exp(S/eps)), y = 1.
__global__ __launch_bounds__(kSweepColThreads) void k_sweep_init(SweepArgs A, const int32_t* __restrict__ status) {
  if (status[0]) return;
  SweepImage I;
  if (!sweep_image(A, blockIdx.y, I)) return;
  const int tid = threadIdx.x;
  const double x_init = exp(A.p.shift / A.p.eps);
  for (int i = blockIdx.x * kSweepColThreads + tid; i < I.m; i += gridDim.x * kSweepColThreads) {
    A.x[I.lo + i] = x_init;
    if (A.pair_out) A.pair_out[I.lo + i] = i;
  }
  const int j0 = blockIdx.x * kSweepCols;
  if (j0 < I.r) {
    if (tid < kSweepCols && j0 + tid < I.r) A.y[I.lo + j0 + tid] = 1.0;
    if (tid == 0) A.ysum[I.lo + blockIdx.x] = static_cast<double>(min(kSweepCols, I.r - j0));
  }
  if (blockIdx.x == 0 && tid == 0) A.ydust[I.b] = 1.0;
}

// FINAL = false: one u-update and the strips' column shares.  `parity` is that
// of the values to read (the previous iteration's).
// FINAL = true: plan entries of the strip and, per column, its largest entry.
// KT: storage type of the kernel matrix (float when A.p.k32).
template <bool FINAL, typename KT>
__global__ __launch_bounds__(kSweepThreads) void k_sweep_rows(SweepArgs A, int parity,
                                                             const int32_t* __restrict__ status) {
  if (status[0]) return;
  SweepImage I;
  if (!sweep_image(A, blockIdx.y, I)) return;
  const int i0 = blockIdx.x * kSweepRows;
  if (i0 >= I.m) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int m = I.m, r = I.r;
  const KT* __restrict__ Kg = reinterpret_cast<const KT*>(A.kmat + I.po);
  const double kz = exp((A.p.z - A.p.shift) / A.p.eps);

  // The strip stays in registers in its storage type.  Every load is issued
  // unconditionally from a clamped address (all of them in flight at once) and
  // out-of-range entries are zeroed afterwards.
  KT K[kSweepRows][kSweepChunks];
  double yv[kSweepChunks];
#pragma unroll
  for (int c = 0; c < kSweepChunks; ++c) {
    const int j = min(tid + kSweepThreads * c, r - 1);
#pragma unroll
    for (int a = 0; a < kSweepRows; ++a)
      K[a][c] = Kg[static_cast<long long>(min(i0 + a, m - 1)) * r + j];
  }
#pragma unroll
  for (int c = 0; c < kSweepChunks; ++c) {
    const int j = tid + kSweepThreads * c;
    yv[c] = j < r ? A.y[I.lo + j] : 0.0;
#pragma unroll
    for (int a = 0; a < kSweepRows; ++a)
      if (!(i0 + a < m && j < r)) K[a][c] = KT(0);
  }
  __shared__ double red[kSweepThreads / 64][kSweepRows];
  __shared__ double xs[kSweepRows];
  if (!FINAL) {
    double s[kSweepRows];
#pragma unroll
    for (int a = 0; a < kSweepRows; ++a) {
      double acc = 0.0;
#pragma unroll
      for (int c = 0; c < kSweepChunks; ++c) acc = fma(static_cast<double>(K[a][c]), yv[c], acc);
      s[a] = acc;
    }
    const double mine = reduce_scatter<kSweepRows>(s, lane);     // row wave_column(lane) of this wave
    if ((lane & 3) == 0) red[wave][wave_column<kSweepRows>(lane)] = mine;
    __syncthreads();
    if (tid < kSweepRows) {
      double t = 0.0;
#pragma unroll
      for (int w = 0; w < kSweepThreads / 64; ++w) t += red[w][tid];
      const double xa = (i0 + tid < m) ? rcp64(t + kz * A.ydust[parity * A.B + I.b]) : 0.0;
      xs[tid] = xa;
      if (i0 + tid < m) A.x[I.lo + i0 + tid] = xa;
    }
    __syncthreads();
    double xa[kSweepRows];
#pragma unroll
    for (int a = 0; a < kSweepRows; ++a) xa[a] = xs[a];
    if (tid == 0) {
      double t = 0.0;
#pragma unroll
      for (int a = 0; a < kSweepRows; ++a) t += xa[a];
      A.xpart[I.lo + blockIdx.x] = t;
    }
    double* out = A.colpart + strip_base(I.po, I.lo) + static_cast<long long>(blockIdx.x) * r;
#pragma unroll
    for (int c = 0; c < kSweepChunks; ++c) {
      const int j = tid + kSweepThreads * c;
      double acc = 0.0;
#pragma unroll
      for (int a = 0; a < kSweepRows; ++a) acc = fma(static_cast<double>(K[a][c]), xa[a], acc);
      if (j < r) out[j] = acc;
    }
  } else {
    if (tid < kSweepRows) xs[tid] = (i0 + tid < m) ? A.x[I.lo + i0 + tid] : 0.0;
    __syncthreads();
    float* P = A.plan_out ? A.plan_out + I.po : nullptr;
    const long long sb = strip_base(I.po, I.lo) + static_cast<long long>(blockIdx.x) * r;
#pragma unroll
    for (int c = 0; c < kSweepChunks; ++c) {
      const int j = tid + kSweepThreads * c;
      float bv = -1.f;
      int bi = 0x7fffffff;
#pragma unroll
      for (int a = 0; a < kSweepRows; ++a) {
        if (i0 + a < m && j < r) {
          const float v = static_cast<float>(xs[a] * static_cast<double>(K[a][c]) * yv[c]);
          if (P) P[static_cast<long long>(i0 + a) * r + j] = v;
          if (v > bv) { bv = v; bi = i0 + a; }
        }
      }
      if (j < r && A.pair_out) { A.bestv[sb + j] = bv; A.besti[sb + j] = bi; }
    }
  }
}

// Workgroup = 64 columns x 4 waves; wave g takes the strips s = g, g + 4, ...
// FINAL = false: the v-update from the strips' shares; reads scalars of
// `parity`, writes those of parity ^ 1.
// FINAL = true: the pairing - largest plan entry of each column over all strips
// (the lowest row wins ties) against the dustbin row's entry.
template <bool FINAL>
__global__ __launch_bounds__(kSweepColThreads) void k_sweep_cols(SweepArgs A, int parity, int first,
                                                                const int32_t* __restrict__ status) {
  if (status[0]) return;
  SweepImage I;
  if (!sweep_image(A, blockIdx.y, I)) return;
  const int j0 = blockIdx.x * kSweepCols;
  if (j0 >= I.r) return;
  const int tid = threadIdx.x, lane = tid & 63, g = tid >> 6, j = j0 + lane;
  const int m = I.m, r = I.r;
  const int nstrips = (m + kSweepRows - 1) / kSweepRows, nblocks = (r + kSweepCols - 1) / kSweepCols;
  const double kz = exp((A.p.z - A.p.shift) / A.p.eps);
  __shared__ double red[kSweepColThreads / 64];
  __shared__ double part[kSweepColGroups][kSweepCols];
  __shared__ float pv[kSweepColGroups][kSweepCols];
  __shared__ int pi[kSweepColGroups][kSweepCols];
  // x_d of the iteration just swept: from the previous iteration's sy and y_d
  double x_dust;
  if (first) {
    x_dust = exp(A.p.shift / A.p.eps);                // no iteration yet (T = 0 pairing only)
  } else {
    double sy = A.ydust[parity * A.B + I.b];
    for (int k = 0; k < nblocks; ++k) sy += A.ysum[parity * A.total + I.lo + k];
    x_dust = static_cast<double>(r) * rcp64(kz * sy);
  }
  const long long sb = strip_base(I.po, I.lo);
  if (!FINAL) {
    double sx = 0.0;
    for (int s = tid; s < nstrips; s += kSweepColThreads) sx += A.xpart[I.lo + s];
    sx = block_sum<kSweepColThreads>(sx, red);
    double t0 = 0.0, t1 = 0.0;
    if (j < r) {
      const double* cp = A.colpart + sb + j;
      int s = g;
      for (; s + kSweepColGroups < nstrips; s += 2 * kSweepColGroups) {
        t0 += cp[static_cast<long long>(s) * r];
        t1 += cp[static_cast<long long>(s + kSweepColGroups) * r];
      }
      if (s < nstrips) t0 += cp[static_cast<long long>(s) * r];
    }
    part[g][lane] = t0 + t1;
    __syncthreads();
    double yj = 0.0;
    if (g == 0 && j < r) {
      double t = part[0][lane];
#pragma unroll
      for (int k = 1; k < kSweepColGroups; ++k) t += part[k][lane];
      yj = rcp64(t + kz * x_dust);
      A.y[I.lo + j] = yj;
    }
    const double ys = block_sum<kSweepColThreads>(yj, red);
    if (tid == 0) {
      A.ysum[(parity ^ 1) * A.total + I.lo + blockIdx.x] = ys;
      if (blockIdx.x == 0) A.ydust[(parity ^ 1) * A.B + I.b] = static_cast<double>(m) * rcp64(kz * (sx + x_dust));
    }
  } else {
    if (!A.pair_out) return;
    float bv = -1.f;
    int bi = 0x7fffffff;
    if (j < r) {
      for (int s = g; s < nstrips; s += kSweepColGroups) {
        const float v = A.bestv[sb + static_cast<long long>(s) * r + j];
        if (v > bv) { bv = v; bi = A.besti[sb + static_cast<long long>(s) * r + j]; }
      }
    }
    pv[g][lane] = bv;
    pi[g][lane] = bi;
    __syncthreads();
    if (g == 0 && j < r) {
#pragma unroll
      for (int k = 1; k < kSweepColGroups; ++k) {
        const float ov = pv[k][lane];
        const int oi = pi[k][lane];
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
      }
      const float dust = static_cast<float>(x_dust * kz * A.y[I.lo + j]);
      A.pair_out[I.lo + m + j] = dust > bv ? -1 : bi;
    }
  }
}

}  // namespace rtp
