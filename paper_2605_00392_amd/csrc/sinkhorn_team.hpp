// Register-resident Sinkhorn (Appendix C) for images whose kept x pruned kernel
// matrix fits the vector registers of a small team of waves.
//
// A team of W waves (T = 64 W threads) is laid out as TR row slots x TC column
// slots, TC = 2^LOG_TC <= 64 so that the column slots of one row slot are
// adjacent lanes of one wave.  Thread (rslot, cslot) holds
//     K[a][c] = K_{rslot + TR a, cslot + TC c},  a < RPT, c < CPT
// in fp64 registers for the whole iteration, so an image needs
// M <= TR RPT and R <= TC CPT.  Per iteration:
//   u-update  row sums are local over c, then summed over the TC column slots
//             with lane shuffles;
//   v-update  column sums are local over a, then summed over the row slots:
//             lane shuffles inside a wave, LDS across the team's waves (two
//             barriers per iteration).
// The dustbin row, column and corner all equal kz = exp((z - shift)/eps) and are
// handled in closed form (they add kz * y_dust to a row sum, kz * x_dust to a
// column sum, and need sum_i x_i and sum_j y_j).
//
// A one-wave team (W = 1) never executes a workgroup barrier, so several of them
// can share a workgroup, one image per wave.
#pragma once
#include "common.hpp"

namespace rtp {

// 1 / d from the hardware estimate and one Newton step.  Measured on gfx950 over
// 2^20 arguments: v_rcp_f64 is off by at most 4.6e-8 relative, one step brings
// that to 2.2e-15 - rounding level for the Sinkhorn scalings it is used for.
__device__ __forceinline__ double rcp64(double d) {
  const double r = __builtin_amdgcn_rcp(d);
  return fma(fma(-d, r, 1.0), r, r);
}

// Where the iteration loop may end.  One iteration maps (x, y) to (x', y') by
// x' = f(y), y' = g(x'), in a fixed order of operations, so it is a function of
// the state's bits.  `moved` says whether the x just computed in iteration `it`
// (0-based) differs anywhere from the previous x.  If it does not, and the previous
// x itself came out of an update (it >= 1, so that the current y is g of it), the y
// about to be computed repeats too, and so does every later iterate: this iteration
// is the last that needs running, and the state after it equals, bit for bit, the
// state after all the iterations asked for.  (Iterates that alternate between two
// states were looked for as well and do not occur: pages that do not settle wander.)
__device__ __forceinline__ int settled_stop(int stop_at, int it, bool moved) {
  return (it >= 1 && !moved) ? min(stop_at, it + 1) : stop_at;
}

// 1 / d to the last bit or two: a second Newton step on top of rcp64's.  The shapes
// that stop once their iterates repeat (settled_stop) use it: with the one-step value,
// off by up to ten units in the last place, the iterates of one page in seven wander
// among neighbouring values without ever repeating; with this one 97 % of 1024
// benchmark pages settle, after 35 iterations on average.
__device__ __forceinline__ double rcp64_tight(double d) {
  const double r = rcp64(d);
  return fma(fma(-d, r, 1.0), r, r);
}

template <int W_, int LOG_TC_, int RPT_, int CPT_>
struct TeamShape {
  static constexpr int W = W_, LOG_TC = LOG_TC_, RPT = RPT_, CPT = CPT_;
  static constexpr int T = 64 * W, TC = 1 << LOG_TC, TR = T / TC;
  static constexpr int kMaxM = TR * RPT, kMaxR = TC * CPT;
  static constexpr int kBlock = T < 256 ? 256 : T;
  static constexpr int kTeamsPerBlock = kBlock / T;
  __host__ __device__ static constexpr bool fits(int m, int r) { return m <= kMaxM && r <= kMaxR; }
};

// The shapes compiled in, tried in this order; an image that fits none is left
// to the general kernel (variant kGeneralVariant).
using TeamB = TeamShape<8, 2, 4, 10>;    // M <= 512,  R <= 40
using TeamC = TeamShape<8, 3, 8, 8>;     // M <= 512,  R <= 64
// Team C's columns with six rows per lane and the kernel matrix held as fp32
// (when its range allows): half the registers, so that two workgroups share a
// compute unit and one's waits are filled by the other (k_sinkhorn_c32).
using TeamC32 = TeamShape<8, 3, 6, 8>;   // M <= 384,  R <= 64
// Tall images (tiled pages with a few pruned tokens): the kernel matrix is held
// as fp32 values, which the same range condition as for the sweep kernels allows,
// and widened at each use; all sums and both scaling vectors stay fp64.
using TeamTall = TeamShape<8, 3, 19, 8>;  // M <= 1216, R <= 64
// The same rows with fewer column registers, for images whose pruned set leaves the
// upper column slots empty (the iteration is bound by instruction issue).
using TeamTall48 = TeamShape<8, 3, 19, 6>;  // R <= 48
using TeamTall32 = TeamShape<8, 3, 19, 4>;  // R <= 32
// Heavily pruned images of up to 512 tokens (65 to 224 pruned), likewise held as
// fp32; between them the three cover every such image with M + R <= 512.
using TeamWideA = TeamShape<8, 4, 14, 8>;   // M <= 448, R <= 128
using TeamWideB = TeamShape<8, 5, 24, 6>;   // M <= 384, R <= 192
using TeamWideC = TeamShape<8, 5, 20, 7>;   // M <= 320, R <= 224
// A strip of a larger image in the multi-workgroup kernel (sinkhorn_cluster.hpp) when it has
// more than 128 pruned tokens: a wave per row slot, the 64 lanes across the columns.
using TeamStripWide = TeamShape<8, 6, 18, 9>;   // 144 rows x 576 columns per workgroup
using TeamStripWider = TeamShape<8, 6, 10, 15>;  // 80 rows x 960 columns per workgroup
// The one- and two-wave kernels (sinkhorn_wave.hpp): kRows augmented rows per
// lane, kCols augmented columns.
struct WaveShape {
  static constexpr int kWaves = 1, kRows = 7, kCols = 8;
  static constexpr int kMaxRows = 64 * kWaves * kRows;
  __host__ __device__ static constexpr bool fits(int m, int r) { return m + 1 <= kMaxRows && r + 1 <= kCols; }
};
struct PairShape {
  static constexpr int kWaves = 2, kRows = 4, kCols = 16;
  static constexpr int kMaxRows = 64 * kWaves * kRows;
  __host__ __device__ static constexpr bool fits(int m, int r) { return m + 1 <= kMaxRows && r + 1 <= kCols; }
};
struct TallShape {   // a whole workgroup on one image
  static constexpr int kWaves = 8, kRows = 3, kCols = 16;
  static constexpr int kMaxRows = 64 * kWaves * kRows;
  __host__ __device__ static constexpr bool fits(int m, int r) { return m + 1 <= kMaxRows && r + 1 <= kCols; }
};
constexpr int kSinkhornBlockWaves = 8;   // waves of a k_sinkhorn_regs workgroup
// The two-copy kernels (sinkhorn_dual.hpp) take M + 1 <= 512 and R + 1 <= 32
// or R + 1 <= 48.
constexpr int kDualRows = 512, kDualCols = 32;
constexpr int kVariantA = 0, kVariantDual = 1, kVariantDual48 = 2, kVariantB = 3, kVariantC = 4,
              kVariantPair = 5, kVariantSweep = 6, kVariantTall = 7, kVariantTeamTall = 8, kVariantWideA = 9,
              kVariantWideB = 10, kVariantWideC = 11, kVariantC32 = 12, kVariantCluster = 13, kGeneralVariant = 14;
// The work lists k_classify builds: one per register-resident shape above, and
// one of the images whose scores and merge go to the tiled matrix-core kernels.
constexpr int kListTiled = 14, kListMid = 15, kWorkLists = 16;
// after the lists: synchronisation words of the multi-workgroup Sinkhorn kernel (arrival counters
// of its cluster slots, a give-up word), zeroed by whoever builds the lists, and one word for the
// sweep kernels: how many of every 16 strips they read with streaming loads (kWorkStreamWord)
constexpr int kWorkSyncWords = 66, kWorkStreamWord = 65;
// The sweep kernels read every kernel matrix once per iteration.  The memory-side cache
// (256 MB) keeps a working set that fits and keeps nothing of one that does not (it is read
// round and round), so of a larger set only this much is read with ordinary loads and the rest
// with streaming ones, which leave no lines behind.  16 pages of 4512 tokens (308 MB): 7.5 ->
// 6.6 ms for 100 iterations at 25 to 37 % streamed, 7.9 ms with everything streamed.
constexpr long long kSweepResidentBytes = 200ll * 1000 * 1000;
// What a call launches besides the 512-row register shapes, as the kernels
// receive it (`mode`).  kModeLarge: the batch may hold images with more than 512
// tokens, so the tall shapes' kernel and the sweep kernels run.  kModeF32: the
// kernel matrix's range fits fp32 (the shapes that hold it as fp32 may be used).
// kModeCluster: the device has compute units enough for the multi-workgroup kernel that keeps
// taller matrices on chip (sinkhorn_cluster.hpp).
// kModeSweep: the launches of the streaming multi-workgroup kernels (sinkhorn_sweep.hpp) are issued.
constexpr int kModeLarge = 1, kModeF32 = 2, kModeCluster = 4, kModeSweep = 8;
// bits 8-12 of `mode`: workgroups per cluster slot of the multi-workgroup kernel in this launch
// (1 to 16); an image that would need more is not that kernel's
constexpr int kModeGroupsShift = 8;
__host__ __device__ inline int mode_cluster_groups(int mode) { return (mode >> kModeGroupsShift) & 31; }
// (that kernel's shapes: up to eight workgroups of 224 or 448 rows with at most 128 pruned tokens,
// up to eight of 144 rows with at most 576, up to sixteen of 80 rows with at most 960)
constexpr int kClusterRows = 8 * 448, kClusterCols = 128;
constexpr int kClusterHalfRows = 8 * 224;
constexpr int kClusterWideRows = 8 * 144, kClusterWideCols = 576;
constexpr int kClusterWiderRows = 16 * 80, kClusterWiderCols = 960;
// which of them an image takes (0 .. 3; -1: none).  With at most 128 pruned tokens the strips are
// 224 rows high while eight of them cover the image (half the arithmetic per workgroup and
// iteration for the same exchange), else 448.
__host__ __device__ inline int cluster_shape(int m, int r) {
  if (m <= kClusterHalfRows && r <= kClusterCols) return 0;
  if (m <= kClusterRows && r <= kClusterCols) return 3;
  if (m <= kClusterWideRows && r <= kClusterWideCols) return 1;
  if (m <= kClusterWiderRows && r <= kClusterWiderCols) return 2;
  return -1;
}
__host__ __device__ inline bool cluster_fits(int m, int r) { return cluster_shape(m, r) >= 0; }
// workgroups the kernel spreads such an image over
__host__ __device__ inline int cluster_groups(int m, int r) {
  const int shape = cluster_shape(m, r);
  return shape == 0 ? (m + 223) / 224 : shape == 3 ? (m + 447) / 448 : shape == 1 ? (m + 143) / 144 : (m + 79) / 80;
}
// The multi-workgroup sweep kernels (sinkhorn_sweep.hpp) take up to this many
// pruned tokens.
constexpr int kSweepMaxPruned = 2048;

// Which Sinkhorn kernel serves an image; every kernel evaluates this and takes
// only its own images, so each image is processed exactly once.
__host__ __device__ inline int sinkhorn_variant(int m, int r, int mode) {
  if (WaveShape::fits(m, r)) return kVariantA;
  if (PairShape::fits(m, r)) return kVariantPair;
  if (m + 1 <= kDualRows && r + 1 <= kDualCols) return kVariantDual;
  if ((mode & kModeLarge) && TallShape::fits(m, r)) return kVariantTall;
  if ((mode & kModeLarge) && (mode & kModeF32) && TeamTall::fits(m, r)) return kVariantTeamTall;
  // rows beyond the shapes above with at most 128 pruned tokens, or up to 1152 rows with at most
  // 576: a cluster of workgroups that keeps the matrix on chip
  if ((mode & kModeLarge) && (mode & kModeF32) && (mode & kModeCluster) && cluster_fits(m, r) &&
      cluster_groups(m, r) <= mode_cluster_groups(mode))
    return kVariantCluster;
  // when the sweep kernels run anyway (their launches are paid for) they also
  // take the images of the slowest register shapes, which otherwise set the
  // duration of the register-resident launch
  if ((mode & kModeSweep) && r <= kSweepMaxPruned) return kVariantSweep;
  if (m + 1 <= kDualRows && r + 1 <= 48) return kVariantDual48;
  if (TeamB::fits(m, r)) return kVariantB;
  if ((mode & kModeF32) && TeamC32::fits(m, r)) return kVariantC32;
  if (TeamC::fits(m, r)) return kVariantC;
  if (mode & kModeF32) {
    if (TeamWideA::fits(m, r)) return kVariantWideA;
    if (TeamWideB::fits(m, r)) return kVariantWideB;
    if (TeamWideC::fits(m, r)) return kVariantWideC;
  }
  return kGeneralVariant;
}

// How an image's kernel matrix K = exp((S - shift)/eps) lies in its slot of the
// workspace (plan_offsets[b], m r doubles); the score kernels write it and the
// Sinkhorn kernel that serves the image reads it, both deciding by this function.
//   kKernelRowsF64  row-major fp64, entry (i, j) at i r + j.
//   kKernelRowsF32  the images of the shapes that hold the matrix as fp32 anyway (the fp32
//                   team shapes, the multi-workgroup kernel) and, when the range allows
//                   (p.k32), the sweep kernels': fp32, rows padded (k32_pitch).  A relative
//                   rounding of 6e-8 on K is an absolute perturbation of eps * 6e-8 on the
//                   score S, below the scores' own error; it halves the bytes the score
//                   pass writes and the Sinkhorn pass reads (every iteration, for the sweep).
//   kKernelColsF64  the one-, two- and eight-wave shapes, whose lanes own rows:
//                   column-major fp64, entry (i, j) at j m + i, so that the 64 lanes of
//                   a load read 64 consecutive entries (row-major, they read 64 cache
//                   lines: the loads alone took 15 to 25 us of a workgroup's time).
constexpr int kKernelRowsF64 = 0, kKernelRowsF32 = 1, kKernelColsF64 = 2;
__device__ __forceinline__ int kernel_layout(const DevParams& p, int m, int r) {
  const int v = sinkhorn_variant(m, r, p.mode);
  if (v == kVariantSweep) return p.k32 ? kKernelRowsF32 : kKernelRowsF64;
  // (these are only chosen under kModeF32)
  if (v == kVariantTeamTall || v == kVariantWideA || v == kVariantWideB || v == kVariantWideC || v == kVariantC32 ||
      v == kVariantCluster)
    return kKernelRowsF32;
  return (v == kVariantA || v == kVariantPair || v == kVariantTall) ? kKernelColsF64 : kKernelRowsF64;
}
__device__ __forceinline__ bool kernel_is_f32(const DevParams& p, int m, int r) {
  return kernel_layout(p, m, r) == kKernelRowsF32;
}
// fp32 layout of image b's kernel matrix: rows padded to a multiple of four
// entries (when there are at least eight columns) and the first row on a 16-byte
// boundary, so that a lane can read four entries of a row at once.  It fits the
// image's fp64 slot of m r doubles: one double of alignment plus m (r + 3) / 2.
__host__ __device__ inline int k32_pitch(int r) { return r >= 8 ? (r + 3) & ~3 : r; }
__device__ __forceinline__ float* k32_base(const double* kmat, long long po) {
  return reinterpret_cast<float*>(const_cast<double*>(kmat) + ((po + 1) & ~1LL));
}
__device__ __forceinline__ void store_kernel(double* __restrict__ kmat, long long po, int i, int j, int m, int r,
                                             double v, int layout) {
  if (layout == kKernelRowsF32) k32_base(kmat, po)[static_cast<long long>(i) * k32_pitch(r) + j] = static_cast<float>(v);
  else if (layout == kKernelColsF64) kmat[po + static_cast<long long>(j) * m + i] = v;
  else kmat[po + static_cast<long long>(i) * r + j] = v;
}

// What every register-resident Sinkhorn body needs.
struct SinkhornArgs {
  const int32_t* offsets;
  const int32_t* keep;
  const long long* plan_offsets;
  DevParams p;
  const double* kmat;
  long long plan_cap;
  float* plan_out;     // may be null
  int32_t* pair_out;   // may be null
};

// One image on one team.  `tw` is the wave's index inside the team, `lane` the
// lane; every wave of the team calls this with the same `b`.
template <typename S, typename KT = double>
__device__ __forceinline__ void sinkhorn_team_image(const SinkhornArgs& A, int b, int tw, int lane) {
  constexpr int W = S::W, TC = S::TC, TR = S::TR, RPT = S::RPT, CPT = S::CPT, T = S::T;
  constexpr int LOG_TC = S::LOG_TC;
  const DevParams& p = A.p;
  const int32_t* __restrict__ offsets = A.offsets;
  const long long* __restrict__ plan_offsets = A.plan_offsets;
  const double* __restrict__ kmat = A.kmat;
  float* __restrict__ plan_out = A.plan_out;
  int32_t* __restrict__ pair_out = A.pair_out;
  const int tt = tw * 64 + lane;                    // thread index inside the team
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  if (n <= 0) return;
  const int m = min(max(A.keep[b], 0), n), r = n - m;
  if (!S::fits(m, r)) return;                       // uniform over the team
  if (pair_out)
    for (int i = tt; i < m; i += T) pair_out[lo + i] = i;
  if (r <= 0 || m <= 0) return;
  if (!plan_fits(plan_offsets[b], m, r, A.plan_cap)) return;
  const long long po = plan_offsets[b];
  // KT = float: the registers hold rounded entries, widened again at each use
  // (the compiler must not keep the widened copies, hence `forget_origin`); the score
  // pass has stored them rounded already (kKernelRowsF32)
  constexpr bool kNarrow = std::is_same<KT, float>::value;
  const KT* Kg;
  int pitch;
  if constexpr (kNarrow) { Kg = k32_base(kmat, po); pitch = k32_pitch(r); }
  else { Kg = kmat + po; pitch = r; }

  const int cslot = tt & (TC - 1);
  const int rslot = tt >> LOG_TC;

  KT K[RPT][CPT];
  // Loads are unconditional (from a clamped position), so that a thread's loads
  // overlap instead of each waiting inside its own branch; they go four rows at
  // a time, and with KT = float each group is narrowed before the next is
  // requested, so that the loads in flight need no more registers than the matrix.
#pragma unroll
  for (int a0 = 0; a0 < RPT; a0 += 4) {
    KT v[4][CPT];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = min(rslot + TR * (a0 + u), m - 1);
#pragma unroll
      for (int c = 0; c < CPT; ++c)
        if (a0 + u < RPT) v[u][c] = Kg[static_cast<long long>(i) * pitch + min(cslot + TC * c, r - 1)];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < CPT; ++c)
        if (a0 + u < RPT) {
          KT k = (rslot + TR * (a0 + u) < m && cslot + TC * c < r) ? v[u][c] : KT(0);
          if constexpr (kNarrow) forget_origin(k);
          K[a0 + u][c] = k;
        }
  }

  const double kz = exp((p.z - p.shift) / p.eps);
  double x[RPT], y[CPT];
  const double x_init = exp(p.shift / p.eps);      // T = 0 leaves u = 0
#pragma unroll
  for (int a = 0; a < RPT; ++a) x[a] = (rslot + TR * a < m) ? x_init : 0.0;
#pragma unroll
  for (int c = 0; c < CPT; ++c) y[c] = (cslot + TC * c < r) ? 1.0 : 0.0;
  double x_dust = x_init, y_dust = 1.0;
  double sum_y = static_cast<double>(r) + 1.0;

  __shared__ double xw[W > 1 ? W : 1][TC][CPT + 1];
  __shared__ double xtot[TC][CPT + 1];

  // KT = float: the latest x, one value per row, kept here for the plan
  __shared__ double xs[kNarrow ? TR : 1][kNarrow ? RPT : 1];
  if constexpr (kNarrow) {
    if (cslot == 0) {
#pragma unroll
      for (int a = 0; a < RPT; ++a) xs[rslot][a] = x[a];   // what T = 0 leaves
    }
  }

  for (int it = 0; it < p.iters; ++it) {
    double t[CPT + 1];
    const double row_dust = kz * y_dust;
    if constexpr (kNarrow) {
      // one pass over the rows: a row is widened once, summed against y, and as
      // soon as its x is known added into the column sums, so that neither the
      // widened entries nor the x of other rows stay in registers
#pragma unroll
      for (int c = 0; c <= CPT; ++c) t[c] = 0.0;
#pragma unroll
      for (int a = 0; a < RPT; ++a) {
        if (TR * a >= m) {                   // no row of this pass exists (the same for every thread)
          xs[rslot][a] = 0.0;
          continue;
        }
        double kd[CPT];
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
          forget_origin(K[a][c]);
          kd[c] = static_cast<double>(K[a][c]);
        }
        double acc = 0.0;
#pragma unroll
        for (int c = 0; c < CPT; ++c) acc = fma(kd[c], y[c], acc);
        acc = group_sum<LOG_TC>(acc);
        const double xa = (rslot + TR * a < m) ? rcp64(acc + row_dust) : 0.0;
#pragma unroll
        for (int c = 0; c < CPT; ++c) t[c] = fma(kd[c], xa, t[c]);
        t[CPT] += xa;
        xs[rslot][a] = xa;   // the lanes of a row slot write the same value; no branch in this loop
        // rows are independent, and left alone the scheduler would widen all of
        // them at once
        if (a % 2 == 1) __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      // ---- u-update ----
      double s[RPT];
#pragma unroll
      for (int a = 0; a < RPT; ++a) {
        double acc = 0.0;
#pragma unroll
        for (int c = 0; c < CPT; ++c) acc = fma(static_cast<double>(K[a][c]), y[c], acc);
        s[a] = acc;
      }
#pragma unroll
      for (int a = 0; a < RPT; ++a) s[a] = group_sum<LOG_TC>(s[a]);
#pragma unroll
      for (int a = 0; a < RPT; ++a) x[a] = (rslot + TR * a < m) ? rcp64(s[a] + row_dust) : 0.0;

      // ---- v-update ----
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        double acc = 0.0;
#pragma unroll
        for (int a = 0; a < RPT; ++a) acc = fma(static_cast<double>(K[a][c]), x[a], acc);
        t[c] = acc;
      }
      double acc = 0.0;
#pragma unroll
      for (int a = 0; a < RPT; ++a) acc += x[a];
      t[CPT] = acc;
    }
    x_dust = static_cast<double>(r) * rcp64(kz * sum_y);
    constexpr bool kScatter = W > 1 && LOG_TC == 3 && CPT <= 8;
    if constexpr (kScatter) {
      // Eight column slots x eight row slots per wave, up to eight column sums per
      // lane (taken as eight): the sums over the row slots (lane bits 3-5) are a
      // reduce-scatter - each exchange hands half of the values to the partner,
      // 4 + 2 + 1 additions instead of 3 per value - which leaves the wave's total of
      // column cslot + 8 (4 b5 + 2 b4 + b3) in this lane, where it goes to LDS directly.
      auto tv = [&](int c) { return c < CPT ? t[c < CPT ? c : 0] : 0.0; };
      double h[4], q[2];
#pragma unroll
      for (int c = 0; c < 4; ++c) h[c] = halve32(tv(c), tv(c + 4));
#pragma unroll
      for (int c = 0; c < 2; ++c) q[c] = halve16(h[c], h[c + 2]);
      const bool b3 = (lane & 8) != 0;
      const double keep = b3 ? q[1] : q[0], send = b3 ? q[0] : q[1];
      const double mine = keep + dpp_move<0x128>(send);              // lane ^ 8
      const int c_own = 4 * (lane >> 5) + 2 * ((lane >> 4) & 1) + (b3 ? 1 : 0);
      if (c_own < CPT) xw[tw][cslot][c_own] = mine;
      t[CPT] = cross_sum<LOG_TC>(t[CPT]);
      if (lane < TC) xw[tw][lane][CPT] = t[CPT];
      __syncthreads();
    } else {
#pragma unroll
      for (int c = 0; c <= CPT; ++c) t[c] = cross_sum<LOG_TC>(t[c]);
    }
    if (W > 1) {
      // wave totals -> LDS; one thread per (column slot, value) adds the W
      // partials; everybody reads back its CPT + 1 totals
      if constexpr (!kScatter) {
        if (lane < TC) {
#pragma unroll
          for (int c = 0; c <= CPT; ++c) xw[tw][lane][c] = t[c];
        }
        __syncthreads();
      }
      // (the thread that adds a column's partials also takes the reciprocal: once per
      // workgroup instead of once per row slot)
      const double col_dust_w = kz * x_dust;
      if (tt < TC * (CPT + 1)) {
        const int cs = tt / (CPT + 1), c = tt - cs * (CPT + 1);
        double acc = 0.0;
#pragma unroll
        for (int w = 0; w < W; ++w) acc += xw[w][cs][c];
        if (c < CPT) acc = (cs + TC * c < r) ? rcp64(acc + col_dust_w) : 0.0;
        xtot[cs][c] = acc;
      }
      __syncthreads();
#pragma unroll
      for (int c = 0; c <= CPT; ++c) t[c] = xtot[cslot][c];
    }
    const double col_dust = kz * x_dust;
    double ly = 0.0;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      if constexpr (W > 1) y[c] = t[c];
      else y[c] = (cslot + TC * c < r) ? rcp64(t[c] + col_dust) : 0.0;
      ly += y[c];
    }
    y_dust = static_cast<double>(m) * rcp64(kz * (t[CPT] + x_dust));
    ly = group_sum<LOG_TC>(ly);
    sum_y = ly + y_dust;
  }

  // ---- plan and pairing ----
  if constexpr (kNarrow) {   // written by this row slot's first lane, a lane of this wave
#pragma unroll
    for (int a = 0; a < RPT; ++a) x[a] = xs[rslot][a];
  }
  float bv[CPT];
  int bi[CPT];
#pragma unroll
  for (int c = 0; c < CPT; ++c) { bv[c] = -1.f; bi[c] = 0x7fffffff; }
  float* P = plan_out ? plan_out + po : nullptr;
  // the entries' offsets are recomputed from slots the compiler cannot relate to
  // the ones the loads used: otherwise it keeps all RPT CPT offsets in registers
  // across the iteration loop
  int rslot_p = rslot, cslot_p = cslot;
  forget_origin(rslot_p);
  forget_origin(cslot_p);
#pragma unroll
  for (int a = 0; a < RPT; ++a) {
    const int i = rslot_p + TR * a;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int j = cslot_p + TC * c;
      if (i < m && j < r) {
        const float v = static_cast<float>(x[a] * static_cast<double>(K[a][c]) * y[c]);
        if (P) P[static_cast<long long>(i) * r + j] = v;
        if (v > bv[c]) { bv[c] = v; bi[c] = i; }
      }
    }
  }
  if (!pair_out) return;
#pragma unroll
  for (int mask = TC; mask < kWave; mask <<= 1)
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const float ov = __shfl_xor(bv[c], mask, kWave);
      const int oi = __shfl_xor(bi[c], mask, kWave);
      if (ov > bv[c] || (ov == bv[c] && oi < bi[c])) { bv[c] = ov; bi[c] = oi; }
    }
  if (W > 1) {
    __shared__ float pv[W > 1 ? W : 1][TC][CPT];
    __shared__ int pi[W > 1 ? W : 1][TC][CPT];
    if (lane < TC) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) { pv[tw][lane][c] = bv[c]; pi[tw][lane][c] = bi[c]; }
    }
    __syncthreads();
    if (tt < TC) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
#pragma unroll
        for (int w = 1; w < W; ++w) {
          const float ov = pv[w][tt][c];
          const int oi = pi[w][tt][c];
          if (ov > bv[c] || (ov == bv[c] && oi < bi[c])) { bv[c] = ov; bi[c] = oi; }
        }
      }
    }
  }
  if (tt < TC) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int j = cslot + TC * c;
      if (j < r) {
        const float dust = static_cast<float>(x_dust * kz * y[c]);
        pair_out[lo + m + j] = dust > bv[c] ? -1 : bi[c];
      }
    }
  }
}

}  // namespace rtp
