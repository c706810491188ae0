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
  void* colpart;    // strips' column shares (stored like the kernel matrix: fp32 when p.k32, else fp64):
                    // image b, strip s, column j at strip_base(b) + s r + j
  double* xpart;    // [total] strip sums of x at offsets[b] + strip
  double* ysum;     // [2][total] block sums of y at offsets[b] + block, by parity
  double* ydust;    // [2][B] by parity
  float* bestv;     // per strip and column: largest plan entry and its row (indexing of colpart)
  int32_t* besti;
  long long total;
  float* plan_out;     // may be null
  int32_t* pair_out;   // may be null
  int stream_16ths;    // >= 0: that many of every 16 strips are read with streaming loads, whatever the
                       // list builder worked out (a switch for tests); < 0: its figure
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
// FINAL = true: plan entries of the strips and, per column, their largest entry.
//
// The 512 threads form RG row groups of CG column threads (CG RG = 512); a row
// group owns one 16-row strip.  With the fp32 layout (VEC = 4: padded, aligned
// rows) thread ct holds the four columns 4 ct .. 4 ct + 3, read 16 bytes at a
// time: 64 column threads cover 256 columns, 512 cover 2048, and narrower images
// put more strips into a workgroup.  With fp64 storage (VEC = 1) thread ct holds
// columns ct, ct + CG, ... (CH of them).
template <bool FINAL, typename KT, int CG, int RG, int CH, int VEC>
__device__ __forceinline__ void sweep_rows_body(const SweepArgs& A, const SweepImage& I, int parity) {
  static_assert(CG * RG == kSweepThreads && CG % 64 == 0, "workgroup shape");
  static_assert(VEC == 1 || (VEC == 4 && sizeof(KT) == 4 && CH == 1), "vector loads: fp32 layout only");
  constexpr int kGroupWaves = CG / 64;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int rg = tid / CG, ct = tid - rg * CG;
  const int m = I.m, r = I.r;
  const int nstrips = (m + kSweepRows - 1) / kSweepRows;
  if (static_cast<int>(blockIdx.x) * RG >= nstrips) return;
  const int strip = blockIdx.x * RG + rg;              // may be past the last strip: then all rows are masked
  const int i0 = strip * kSweepRows;
  const double kz = exp((A.p.z - A.p.shift) / A.p.eps);
  const double y_dust = FINAL ? 0.0 : A.ydust[parity * A.B + I.b];   // early: not on the critical path

  // The strip stays in registers in its storage type.  Every load is issued
  // unconditionally from a clamped address (all of them in flight at once) and
  // out-of-range entries are zeroed afterwards.
  KT K[kSweepRows][CH * VEC];
  double yv[CH * VEC];
  // this strip's share of what the memory-side cache cannot keep is read with streaming loads
  const bool stream = (strip & 15) < (A.stream_16ths >= 0 ? A.stream_16ths : A.work[kWorkLists * (1 + A.B) + kWorkStreamWord]);
  auto column = [&](int cv) { return VEC == 4 ? 4 * ct + cv : ct + CG * cv; };   // of register slot cv
  if (VEC == 4) {
    const int pitch = k32_pitch(r);
    const float* __restrict__ Kg = k32_base(A.kmat, I.po);
    const int j4 = min(4 * ct, pitch - 4);             // a whole aligned group inside the padded row
#pragma unroll
    for (int a = 0; a < kSweepRows; ++a) {
      const float4* src = reinterpret_cast<const float4*>(Kg + static_cast<long long>(min(i0 + a, m - 1)) * pitch + j4);
      const float4 v = stream ? load_stream(src) : *src;
      K[a][0] = static_cast<KT>(v.x);
      K[a][1 % (CH * VEC)] = static_cast<KT>(v.y);
      K[a][2 % (CH * VEC)] = static_cast<KT>(v.z);
      K[a][3 % (CH * VEC)] = static_cast<KT>(v.w);
    }
  } else {
    // fp32 storage of an image with fewer than eight columns comes here too: its
    // rows are unpadded but start at the aligned base like every fp32 image
    const KT* __restrict__ Kg = sizeof(KT) == 4 ? reinterpret_cast<const KT*>(k32_base(A.kmat, I.po))
                                                : reinterpret_cast<const KT*>(A.kmat + I.po);
    const int pitch = sizeof(KT) == 4 ? k32_pitch(r) : r;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int j = min(ct + CG * c, r - 1);
#pragma unroll
      for (int a = 0; a < kSweepRows; ++a)
      {
        const KT* src = Kg + static_cast<long long>(min(i0 + a, m - 1)) * pitch + j;
        K[a][c] = stream ? __builtin_nontemporal_load(src) : *src;
      }
    }
  }
#pragma unroll
  for (int cv = 0; cv < CH * VEC; ++cv) {
    const int j = column(cv);
    yv[cv] = j < r ? A.y[I.lo + j] : 0.0;
#pragma unroll
    for (int a = 0; a < kSweepRows; ++a)
      if (!(i0 + a < m && j < r)) K[a][cv] = KT(0);
  }
  __shared__ double red[kSweepThreads / 64][kSweepRows];
  __shared__ double xs[RG][kSweepRows];
  if (!FINAL) {
    double s[kSweepRows];
#pragma unroll
    for (int a = 0; a < kSweepRows; ++a) {
      double acc = 0.0;
#pragma unroll
      for (int cv = 0; cv < CH * VEC; ++cv) acc = fma(static_cast<double>(K[a][cv]), yv[cv], acc);
      s[a] = acc;
    }
    const double mine = reduce_scatter<kSweepRows>(s, lane);     // row wave_column(lane) of this wave
    if ((lane & 3) == 0) red[wave][wave_column<kSweepRows>(lane)] = mine;
    __syncthreads();
    if (tid < kSweepRows * RG) {
      const int g = tid / kSweepRows, a = tid - g * kSweepRows;
      const int i = (blockIdx.x * RG + g) * kSweepRows + a;
      double t = 0.0;
#pragma unroll
      for (int w = 0; w < kGroupWaves; ++w) t += red[g * kGroupWaves + w][a];
      const double xa = i < m ? rcp64(t + kz * y_dust) : 0.0;
      xs[g][a] = xa;
      if (i < m) A.x[I.lo + i] = xa;
    }
    __syncthreads();
    if (strip >= nstrips) return;
    // the strip's x are read from LDS row by row (every lane the same address)
    // rather than held: registers decide how many workgroups share a CU
    double share[CH * VEC], xsum = 0.0;
#pragma unroll
    for (int cv = 0; cv < CH * VEC; ++cv) share[cv] = 0.0;
    // widen the entries again here rather than keep their fp64 copies of the row
    // sums alive (twice the registers)
#pragma unroll
    for (int a = 0; a < kSweepRows; ++a)
#pragma unroll
      for (int cv = 0; cv < CH * VEC; ++cv) forget_origin(K[a][cv]);
#pragma unroll
    for (int a = 0; a < kSweepRows; ++a) {
      const double xa = xs[rg][a];
      xsum += xa;
#pragma unroll
      for (int cv = 0; cv < CH * VEC; ++cv) share[cv] = fma(static_cast<double>(K[a][cv]), xa, share[cv]);
    }
    if (ct == 0) A.xpart[I.lo + strip] = xsum;
    // a share rounded to fp32 is off by 6e-8 of itself, so a column sum by at most
    // that much: the same size as the rounding of the fp32 kernel matrix
    KT* out = static_cast<KT*>(A.colpart) + strip_base(I.po, I.lo) + static_cast<long long>(strip) * r;
#pragma unroll
    for (int cv = 0; cv < CH * VEC; ++cv) {
      const int j = column(cv);
      if (j < r) out[j] = static_cast<KT>(share[cv]);
    }
  } else {
    if (tid < kSweepRows * RG) {
      const int g = tid / kSweepRows, a = tid - g * kSweepRows;
      const int i = (blockIdx.x * RG + g) * kSweepRows + a;
      xs[g][a] = i < m ? A.x[I.lo + i] : 0.0;
    }
    __syncthreads();
    if (strip >= nstrips) return;
    float* P = A.plan_out ? A.plan_out + I.po : nullptr;
    const long long sb = strip_base(I.po, I.lo) + static_cast<long long>(strip) * r;
#pragma unroll
    for (int cv = 0; cv < CH * VEC; ++cv) {
      const int j = column(cv);
      float bv = -1.f;
      int bi = 0x7fffffff;
#pragma unroll
      for (int a = 0; a < kSweepRows; ++a) {
        if (i0 + a < m && j < r) {
          const float v = static_cast<float>(xs[rg][a] * static_cast<double>(K[a][cv]) * yv[cv]);
          if (P) P[static_cast<long long>(i0 + a) * r + j] = v;
          if (v > bv) { bv = v; bi = i0 + a; }
        }
      }
      if (j < r && A.pair_out) { A.bestv[sb + j] = bv; A.besti[sb + j] = bi; }
    }
  }
}

// One kernel for all widths (separate kernels for narrow and wide images, each
// with its own register budget, were measured: the extra launch over a mostly
// idle grid costs what the higher occupancy gains).  CH: columns per thread of
// the wide shape, the smallest that covers the batch's largest possible pruned
// set.  The 16-byte loads are used for the widest images only: measured, the
// registers they take slow every narrower shape down.
template <bool FINAL, typename KT, int CH>
__global__ __launch_bounds__(kSweepThreads) void k_sweep_rows(SweepArgs A, int parity,
                                                             const int32_t* __restrict__ status) {
  if (status[0]) return;
  SweepImage I;
  if (!sweep_image(A, blockIdx.y, I)) return;
  if (I.r <= 128) sweep_rows_body<FINAL, KT, 128, 4, 1, 1>(A, I, parity);
  else if (I.r <= 256) sweep_rows_body<FINAL, KT, 256, 2, 1, 1>(A, I, parity);
  else if (sizeof(KT) == 4 && CH == 4 && I.r > kSweepThreads * 2)
    sweep_rows_body<FINAL, float, 512, 1, 1, 4>(A, I, parity);   // widest images: 16-byte loads pay
  else if (I.r <= kSweepThreads * CH) sweep_rows_body<FINAL, KT, 512, 1, CH, 1>(A, I, parity);
}

// Workgroup = 64 columns x 4 waves; wave g takes the strips s = g, g + 4, ...
// FINAL = false: the v-update from the strips' shares; reads scalars of
// `parity`, writes those of parity ^ 1.
// FINAL = true: the pairing - largest plan entry of each column over all strips
// (the lowest row wins ties) against the dustbin row's entry.
template <bool FINAL, typename ST>
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
    // at most 32 block sums: one per lane, added by the wave (every wave of
    // every workgroup forms the same total in the same order)
    const double mine = lane < nblocks ? A.ysum[parity * A.total + I.lo + lane] : 0.0;
    const double sy = wave_sum_dpp(mine) + A.ydust[parity * A.B + I.b];
    x_dust = static_cast<double>(r) * rcp64(kz * sy);
  }
  const long long sb = strip_base(I.po, I.lo);
  if (!FINAL) {
    double sx = 0.0;
    if (blockIdx.x == 0) {                              // only this workgroup writes y_d
      for (int s = tid; s < nstrips; s += kSweepColThreads) sx += A.xpart[I.lo + s];
      sx = block_sum<kSweepColThreads>(sx, red);
    }
    // this wave's strips g, g + 4, ...: eight loads in flight, eight running sums
    double t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) t[u] = 0.0;
    if (j < r) {
      const ST* cp = static_cast<const ST*>(A.colpart) + sb + j;
      int s = g;
      for (; s + 7 * kSweepColGroups < nstrips; s += 8 * kSweepColGroups) {
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] += static_cast<double>(cp[static_cast<long long>(s + u * kSweepColGroups) * r]);
      }
      for (; s < nstrips; s += kSweepColGroups) t[0] += static_cast<double>(cp[static_cast<long long>(s) * r]);
    }
    part[g][lane] = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
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
