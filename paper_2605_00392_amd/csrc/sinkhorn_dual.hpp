// Sinkhorn (Appendix C) with the kernel matrix held twice in registers, once
// per sweep direction, so that neither sweep needs a cross-lane reduction.
//
// Workgroup = 8 waves = 512 threads, one image with M + 1 <= 512 and
// R + 1 <= 32.  The dustbin row and column are ordinary entries here: the
// augmented kernel Kb is (M+1) x (R+1) with Kb = kz = exp((z - shift)/eps) on
// the last row and column, row marginals a = [1_M, R], column marginals
// b = [1_R, M].
//
//   row copy     thread t owns row t of Kb (32 doubles): the u-update
//                x_t = a_t / sum_j Kb_tj y_j is thread-local; y is read from
//                LDS as a broadcast.
//   column copy  lane = 32 h + j of wave w owns column j of the 32-row chunk
//                q = 2 w + h (32 doubles): the v-update's partial column sums
//                sum_{i in chunk} Kb_ij x_i are thread-local; x is read from
//                LDS (each half-wave reads one address at a time).  The 16
//                partials of a column go through LDS; every wave adds them up
//                for itself, so y needs no third barrier.
//
// Two workgroup barriers per iteration, no lane shuffles.
#pragma once
#include "common.hpp"
#include "sinkhorn_team.hpp"
#include "sinkhorn_wave.hpp"

namespace rtp {

constexpr int kDualThreads = 512;  // = kDualRows: one augmented row per thread
static_assert(kDualThreads == 64 * kSinkhornBlockWaves, "workgroup shape");
constexpr int kDualChunks = 16;    // 32-row chunks of the column copy

// One image on the whole 512-thread workgroup.
__device__ __forceinline__ void sinkhorn_dual_image(const SinkhornArgs& A, int b) {
  const DevParams& p = A.p;
  const int32_t* __restrict__ offsets = A.offsets;
  const long long* __restrict__ plan_offsets = A.plan_offsets;
  const double* __restrict__ kmat = A.kmat;
  float* __restrict__ plan_out = A.plan_out;
  int32_t* __restrict__ pair_out = A.pair_out;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  if (n <= 0) return;
  const int m = min(max(A.keep[b], 0), n), r = n - m;
  if (!(m + 1 <= kDualRows && r + 1 <= kDualCols)) return;
  if (pair_out)
    for (int i = tid; i < m; i += kDualThreads) pair_out[lo + i] = i;
  if (r <= 0 || m <= 0) return;
  if (!plan_fits(plan_offsets[b], m, r, A.plan_cap)) return;
  const long long po = plan_offsets[b];
  const double* Kg = kmat + po;
  const double kz = exp((p.z - p.shift) / p.eps);

  __shared__ double xs[kDualRows];
  __shared__ double part[kDualChunks][kDualCols];
  __shared__ double ys[kDualThreads / 64][kDualCols];
  __shared__ float pv[kDualChunks][kDualCols];
  __shared__ int pi[kDualChunks][kDualCols];

  // row copy: row `tid` of the augmented kernel
  // (loads are unconditional, from clamped positions, so that all of a thread's
  // loads are in flight together; the dustbin row and column hold kz, everything
  // outside the augmented matrix 0)
  double Kr[kDualCols];
  {
    const double* row = Kg + static_cast<long long>(min(tid, m - 1)) * r;
#pragma unroll
    for (int c = 0; c < kDualCols; ++c) {
      const double v = row[min(c, r - 1)];
      Kr[c] = (tid < m && c < r) ? v : ((tid <= m && c <= r) ? kz : 0.0);
    }
  }
  // column copy: column j of rows 32 q .. 32 q + 31
  const int j = lane & 31, q = 2 * wave + (lane >> 5);
  double Kc[32];
  {
    const double* col = Kg + min(j, r - 1);
#pragma unroll
    for (int a = 0; a < 32; ++a) {
      const int i = 32 * q + a;
      const double v = col[static_cast<long long>(min(i, m - 1)) * r];
      Kc[a] = (i < m && j < r) ? v : ((i <= m && j <= r) ? kz : 0.0);
    }
  }
  const double a_row = tid < m ? 1.0 : static_cast<double>(r);   // row marginal of row tid
  const double b_col = j < r ? 1.0 : static_cast<double>(m);     // column marginal of column j

  double x = (tid <= m) ? exp(p.shift / p.eps) : 0.0;   // T = 0 leaves u = 0
  double y = (j <= r) ? 1.0 : 0.0;
  xs[tid] = x;
  if (lane < 32) ys[wave][lane] = y;
  __syncthreads();

  // (the loop ends as soon as the iterates repeat: see settled_stop)
  __shared__ int moved[kDualThreads / 64];
  int stop_at = p.iters;
  for (int it = 0; it < stop_at; ++it) {
    // ---- u-update (row copy) ----
    {
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int c = 0; c < kDualCols; c += 2) {
        s0 = fma(Kr[c], ys[wave][c], s0);
        s1 = fma(Kr[c + 1], ys[wave][c + 1], s1);
      }
      const double xn = (tid <= m) ? a_row * rcp64_tight(s0 + s1) : 0.0;
      const int bits = __builtin_amdgcn_ballot_w64(__double_as_longlong(xn) != __double_as_longlong(x)) != 0 ? 1 : 0;
      x = xn;
      xs[tid] = x;
      if (lane == 0) moved[wave] = bits;   // (rewritten only after the next barrier but one)
    }
    __syncthreads();
    {
      int moved_bits = 0;
#pragma unroll
      for (int w = 0; w < kDualThreads / 64; ++w) moved_bits |= moved[w];
      stop_at = settled_stop(stop_at, it, moved_bits != 0);   // the same in every thread
    }
    // ---- v-update (column copy) ----
    {
      const double* xq = xs + 32 * q;
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int a = 0; a < 32; a += 2) {
        s0 = fma(Kc[a], xq[a], s0);
        s1 = fma(Kc[a + 1], xq[a + 1], s1);
      }
      part[q][j] = s0 + s1;
    }
    __syncthreads();
    {
      double t = 0.0;
#pragma unroll
      for (int c = 0; c < kDualChunks; ++c) t += part[c][j];
      y = (j <= r) ? b_col * rcp64_tight(t) : 0.0;
      if (lane < 32) ys[wave][lane] = y;   // read back by this wave only
    }
  }
  __syncthreads();

  // ---- plan: row t of P = x_t K_tj y_j ----
  if (plan_out && tid < m) {
    float* P = plan_out + po + static_cast<long long>(tid) * r;
#pragma unroll
    for (int c = 0; c < kDualCols; ++c)
      if (c < r) P[c] = static_cast<float>(x * Kr[c] * ys[wave][c]);
  }
  if (!pair_out) return;
  // ---- pairing: arg-max over rows 0..M of column j (row M is the dustbin) ----
  {
    const double* xq = xs + 32 * q;
    float bv = -1.f;
    int bi = 0x7fffffff;
#pragma unroll
    for (int a = 0; a < 32; ++a) {
      const int i = 32 * q + a;
      const float v = static_cast<float>(xq[a] * Kc[a] * y);
      if (i <= m && v > bv) { bv = v; bi = i; }
    }
    pv[q][j] = bv;
    pi[q][j] = bi;
  }
  __syncthreads();
  if (tid < r) {
    float bv = pv[0][tid];
    int bi = pi[0][tid];
#pragma unroll
    for (int c = 1; c < kDualChunks; ++c) {
      const float ov = pv[c][tid];
      const int oi = pi[c][tid];
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    pair_out[lo + m + tid] = (bi >= m) ? -1 : bi;
  }
}

// The same two-copy scheme for up to 47 pruned tokens (R + 1 <= 48).  The row
// copy is fp64 (48 doubles per thread); in the column copy lane = column and
// wave = a chunk of CR rows, so it serves M + 1 <= 8 CR rows:
//   CR = 52, fp64  M + 1 <= 416 (every 400-token page);
//   CR = 64, fp32  M + 1 <= 512: the column copy only feeds the v-update's sums,
//                  and a relative rounding of 6e-8 per entry averages out to a
//                  few 1e-9 on a column sum, far inside the 1e-6 near-tie band.
// The plan and the pairing are formed from the fp64 row copy in both cases.
constexpr int kDual48Cols = 48;

template <int CR, typename KcT>
__device__ __forceinline__ void sinkhorn_dual48_image(const SinkhornArgs& A, int b) {
  const DevParams& p = A.p;
  const int32_t* __restrict__ offsets = A.offsets;
  const long long* __restrict__ plan_offsets = A.plan_offsets;
  const double* __restrict__ kmat = A.kmat;
  float* __restrict__ plan_out = A.plan_out;
  int32_t* __restrict__ pair_out = A.pair_out;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  if (n <= 0) return;
  const int m = min(max(A.keep[b], 0), n), r = n - m;
  if (!(m + 1 <= 8 * CR && r + 1 <= kDual48Cols)) return;
  if (pair_out)
    for (int i = tid; i < m; i += kDualThreads) pair_out[lo + i] = i;
  if (r <= 0 || m <= 0) return;
  if (!plan_fits(plan_offsets[b], m, r, A.plan_cap)) return;
  const long long po = plan_offsets[b];
  const double* Kg = kmat + po;
  const double kz = exp((p.z - p.shift) / p.eps);
  constexpr int NW = kDualThreads / 64;

  __shared__ double xs[kDualRows];
  __shared__ double part[NW][64];
  __shared__ double ys[NW][64];
  __shared__ float pv[NW][kDual48Cols];
  __shared__ int pi[NW][kDual48Cols];

  // Both copies are loaded unconditionally from clamped positions (all loads of a
  // thread in flight together) and patched afterwards: the dustbin row and column
  // hold kz, everything outside the augmented matrix 0.
  double Kr[kDual48Cols];
  {
    const double* row = Kg + static_cast<long long>(min(tid, m - 1)) * r;
#pragma unroll
    for (int c = 0; c < kDual48Cols; ++c) {
      const double v = row[min(c, r - 1)];
      Kr[c] = (tid < m && c < r) ? v : ((tid <= m && c <= r) ? kz : 0.0);
    }
  }
  __builtin_amdgcn_sched_barrier(0);   // the second copy's loads after the first's have landed: registers
  KcT Kc[CR];
  {
    const double* col = Kg + min(lane, r - 1);
#pragma unroll
    for (int a = 0; a < CR; ++a) {
      const int i = CR * wave + a;
      const double v = col[static_cast<long long>(min(i, m - 1)) * r];
      Kc[a] = static_cast<KcT>((i < m && lane < r) ? v : ((i <= m && lane <= r) ? kz : 0.0));
    }
  }
  const double a_row = tid < m ? 1.0 : static_cast<double>(r);
  const double b_col = lane < r ? 1.0 : static_cast<double>(m);

  double x = (tid <= m) ? exp(p.shift / p.eps) : 0.0;
  double y = (lane <= r) ? 1.0 : 0.0;
  xs[tid] = x;
  ys[wave][lane] = y;
  __syncthreads();

  __shared__ int moved[NW];                // (the loop ends as soon as the iterates repeat: see settled_stop)
  int stop_at = p.iters;
  for (int it = 0; it < stop_at; ++it) {
    {
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int c = 0; c < kDual48Cols; c += 2) {
        s0 = fma(Kr[c], ys[wave][c], s0);
        s1 = fma(Kr[c + 1], ys[wave][c + 1], s1);
      }
      const double xn = (tid <= m) ? a_row * rcp64_tight(s0 + s1) : 0.0;
      const int bits = __builtin_amdgcn_ballot_w64(__double_as_longlong(xn) != __double_as_longlong(x)) != 0 ? 1 : 0;
      x = xn;
      xs[tid] = x;
      if (lane == 0) moved[wave] = bits;
    }
    __syncthreads();
    {
      int moved_bits = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) moved_bits |= moved[w];
      stop_at = settled_stop(stop_at, it, moved_bits != 0);
    }
    {
      const double* xq = xs + CR * wave;
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int a = 0; a < CR; a += 2) {
        s0 = fma(static_cast<double>(Kc[a]), xq[a], s0);
        s1 = fma(static_cast<double>(Kc[a + 1]), xq[a + 1], s1);
      }
      part[wave][lane] = s0 + s1;
    }
    __syncthreads();
    {
      double t = 0.0;
#pragma unroll
      for (int c = 0; c < NW; ++c) t += part[c][lane];
      y = (lane <= r) ? b_col * rcp64_tight(t) : 0.0;
      ys[wave][lane] = y;                  // read back by this wave only
    }
  }
  __syncthreads();

  // plan row t of P = x_t K_tj y_j from the row copy
  if (plan_out && tid < m) {
    float* P = plan_out + po + static_cast<long long>(tid) * r;
#pragma unroll
    for (int c = 0; c < kDual48Cols; ++c)
      if (c < r) P[c] = static_cast<float>(x * Kr[c] * ys[wave][c]);
  }
  if (!pair_out) return;
  // per column, the wave's best (value, row): the dustbin is row m
  if constexpr (std::is_same<KcT, double>::value) {
    // the fp64 column copy gives the same products as the row copy: lane = column
    const double* xq = xs + CR * wave;
    float bv = -1.f;
    int bi = 0x7fffffff;
#pragma unroll
    for (int a = 0; a < CR; ++a) {
      const int i = CR * wave + a;
      const float v = static_cast<float>(xq[a] * Kc[a] * y);
      if (i <= m && v > bv) { bv = v; bi = i; }
    }
    if (lane < kDual48Cols) { pv[wave][lane] = bv; pi[wave][lane] = bi; }
  } else {
    // the fp32 column copy is not exact: entries come from the row copy, one
    // column at a time, and the wave's lanes (rows) are compared by shuffles
    for (int c = 0; c < r; ++c) {
      float v = -1.f;
      int idx = 0x7fffffff;
      if (tid <= m) {
        double kc = 0.0;
#pragma unroll
        for (int cc = 0; cc < kDual48Cols; ++cc) kc = (cc == c) ? Kr[cc] : kc;   // static register indexing
        v = static_cast<float>(x * kc * ys[wave][c]);
        idx = tid;
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, kWave);
        const int oi = __shfl_xor(idx, o, kWave);
        if (ov > v || (ov == v && oi < idx)) { v = ov; idx = oi; }
      }
      if (lane == 0) { pv[wave][c] = v; pi[wave][c] = idx; }
    }
  }
  __syncthreads();
  if (tid < r) {
    float bv = pv[0][tid];
    int bi = pi[0][tid];
#pragma unroll
    for (int c = 1; c < NW; ++c) {
      const float ov = pv[c][tid];
      const int oi = pi[c][tid];
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    pair_out[lo + m + tid] = (bi >= m) ? -1 : bi;
  }
}

// Work lists for the register-resident kernels: `work` holds kWorkLists counts
// (one per shape, indexed by variant id) followed by as many lists of B image
// indices each.  One workgroup; list order follows image order.
constexpr int kClassifyLdsBytes = kWorkLists * 256 * 4;   // LDS classify_images works in
__device__ __forceinline__ void classify_images(const int32_t* __restrict__ offsets,
                                                const int32_t* __restrict__ keep, int B,
                                                int32_t* __restrict__ work, int mode, void* lds) {
  constexpr int NV = kWorkLists;
  int (*cnt)[256] = static_cast<int (*)[256]>(lds);   // [NV][256]
  const int tid = threadIdx.x;
  const int span = (B + 255) / 256;
  const int b0 = min(B, tid * span), b1 = min(B, b0 + span);
  int c[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) c[v] = 0;
  __shared__ unsigned long long sweep_cells;      // entries of the sweep kernels' matrices, padding included
  if (tid == 0) sweep_cells = 0;
  __syncthreads();
  unsigned long long cells = 0;
  for (int b = b0; b < b1; ++b) {
    const int n = offsets[b + 1] - offsets[b];
    const int m = min(max(keep[b], 0), max(n, 0));
    const int v = sinkhorn_variant(m, n - m, mode);
    if (n > 0 && v < kGeneralVariant) {
#pragma unroll
      for (int u = 0; u < NV; ++u) c[u] += (u == v);
    }
    if (n > 0 && v == kVariantSweep) cells += static_cast<unsigned long long>(m) * k32_pitch(n - m);
    if (n > 0 && n - m > kTiledMinPruned) c[kListTiled] += 1;
    if (n > 0 && merge_is_mid(n - m)) c[kListMid] += 1;
  }
#pragma unroll
  for (int v = 0; v < NV; ++v) cnt[v][tid] = c[v];
  if (cells) atomicAdd(&sweep_cells, cells);
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    int add[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) add[v] = tid >= o ? cnt[v][tid - o] : 0;
    __syncthreads();
#pragma unroll
    for (int v = 0; v < NV; ++v) cnt[v][tid] += add[v];
    __syncthreads();
  }
  int at[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) at[v] = cnt[v][tid] - c[v];
  for (int b = b0; b < b1; ++b) {
    const int n = offsets[b + 1] - offsets[b];
    const int m = min(max(keep[b], 0), max(n, 0));
    const int v = sinkhorn_variant(m, n - m, mode);
    if (n > 0 && v < kGeneralVariant) {
#pragma unroll
      for (int u = 0; u < NV; ++u)
        if (u == v) work[NV + u * B + at[u]++] = b;
    }
    if (n > 0 && n - m > kTiledMinPruned) work[NV + kListTiled * B + at[kListTiled]++] = b;
    if (n > 0 && merge_is_mid(n - m)) work[NV + kListMid * B + at[kListMid]++] = b;
  }
  if (tid == 255) {
#pragma unroll
    for (int v = 0; v < NV; ++v) work[v] = cnt[v][255];
  }
  // the cluster kernel's arrival counters and give-up word start at zero
  if (tid < kWorkStreamWord) work[NV * (1 + B) + tid] = 0;
  if (tid == kWorkStreamWord) {
    // (the matrices are fp32 when the range allows and the sweep kernels run, else fp64)
    const double bytes = static_cast<double>(sweep_cells) * (((mode & kModeF32) && (mode & kModeSweep)) ? 4.0 : 8.0);
    const double over = bytes > static_cast<double>(kSweepResidentBytes)
                            ? 1.0 - static_cast<double>(kSweepResidentBytes) / bytes : 0.0;
    work[NV * (1 + B) + kWorkStreamWord] = static_cast<int>(ceil(16.0 * over));
  }
}

__global__ __launch_bounds__(256) void k_classify(const int32_t* __restrict__ offsets,
                                                  const int32_t* __restrict__ keep, int B,
                                                  int32_t* __restrict__ work, int mode,
                                                  const int32_t* __restrict__ status) {
  if (status[0]) return;
  __shared__ __align__(16) unsigned char lds[kClassifyLdsBytes];
  classify_images(offsets, keep, B, work, mode, lds);
}

// Both of the above in one launch, for the fused calls.
__global__ __launch_bounds__(256) void k_scan_classify(const int32_t* __restrict__ offsets,
                                                       const int32_t* __restrict__ keep, int B,
                                                       int32_t* __restrict__ out_offsets,
                                                       long long* __restrict__ plan_offsets,
                                                       int32_t* __restrict__ work, int mode,
                                                       const int32_t* __restrict__ status) {
  if (status[0]) return;
  __shared__ __align__(16) unsigned char lds[kClassifyLdsBytes];   // (the two run one after the other)
  static_assert(kScanLdsBytes <= kClassifyLdsBytes, "shared work area");
  scan_images(offsets, keep, B, out_offsets, plan_offsets, lds);
  __syncthreads();
  classify_images(offsets, keep, B, work, mode, lds);
}

// All register-resident Sinkhorn work of a batch in one launch.  Workgroups are
// handed out longest-running role first: the wide teams, team C, team B, two-copy (48 columns),
// two-copy (32 columns), two-wave (two or four images per workgroup), one-wave (eight
// images per workgroup).  `cus`: compute units of the device.
__global__ __launch_bounds__(kDualThreads) void k_sinkhorn_regs(SinkhornArgs A,
                                                               const int32_t* __restrict__ work, int B, int cus,
                                                               const int32_t* __restrict__ status) {
  if (status[0]) return;
  constexpr int NV = kWorkLists;
  constexpr int kWavesPerBlock = kDualThreads / 64;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int blk = blockIdx.x;
  int cnt = work[kVariantWideC];
  if (blk < cnt) { sinkhorn_team_image<TeamWideC, float>(A, work[NV + kVariantWideC * B + blk], wave, lane); return; }
  blk -= cnt;
  cnt = work[kVariantWideB];
  if (blk < cnt) { sinkhorn_team_image<TeamWideB, float>(A, work[NV + kVariantWideB * B + blk], wave, lane); return; }
  blk -= cnt;
  cnt = work[kVariantWideA];
  if (blk < cnt) { sinkhorn_team_image<TeamWideA, float>(A, work[NV + kVariantWideA * B + blk], wave, lane); return; }
  blk -= cnt;
  cnt = work[kVariantC];
  if (blk < cnt) { sinkhorn_team_image<TeamC>(A, work[NV + kVariantC * B + blk], wave, lane); return; }
  blk -= cnt;
  cnt = work[kVariantB];
  if (blk < cnt) { sinkhorn_team_image<TeamB>(A, work[NV + kVariantB * B + blk], wave, lane); return; }
  blk -= cnt;
  cnt = work[kVariantDual48];
  if (blk < cnt) {
    const int img = work[NV + kVariantDual48 * B + blk];
    const int n_img = A.offsets[img + 1] - A.offsets[img];
    if (min(max(A.keep[img], 0), n_img) + 1 <= 8 * 52) sinkhorn_dual48_image<52, double>(A, img);
    else sinkhorn_dual48_image<64, float>(A, img);
    return;
  }
  blk -= cnt;
  cnt = work[kVariantDual];
  if (blk < cnt) { sinkhorn_dual_image(A, work[NV + kVariantDual * B + blk]); return; }
  blk -= cnt;
  // Two-wave images: four per workgroup, or - when the whole launch then still has
  // no more workgroups than the chip has CUs (a workgroup of this kernel fills a
  // CU's registers, so a surplus one waits for a CU to come free) - two, on the
  // first four waves, so that each wave has a SIMD to itself: the iteration is
  // bound by instruction issue (1.3 -> 0.7 us).  Waves without an image end at
  // once; a wave that has ended no longer counts at the workgroup's barriers.
  const int nA = work[kVariantA];
  const int nP = work[kVariantPair];
  const int others = work[kVariantWideA] + work[kVariantWideB] + work[kVariantWideC] + work[kVariantC] +
                     work[kVariantB] + work[kVariantDual48] +
                     (nA + kWavesPerBlock - 1) / kWavesPerBlock + work[kVariantDual];
  const int per_block = others + (nP + 1) / 2 <= cus ? 2 : kWavesPerBlock / PairShape::kWaves;
  cnt = (nP + per_block - 1) / per_block;
  if (blk < cnt) {
    const int slot = wave / PairShape::kWaves, idx = blk * per_block + slot;
    if (slot >= per_block || idx >= nP) return;
    sinkhorn_waves_image<PairShape>(A, work[NV + kVariantPair * B + idx], slot, wave % PairShape::kWaves, lane);
    return;
  }
  blk -= cnt;
  // one-wave images, eight per workgroup: the shortest-running role, handed out last
  cnt = (nA + kWavesPerBlock - 1) / kWavesPerBlock;
  if (blk < cnt) {
    const int idx = blk * kWavesPerBlock + wave;
    if (idx < nA) sinkhorn_waves_image<WaveShape>(A, work[NV + kVariantA * B + idx], wave, 0, lane);
  }
}

// The tall shapes (more than 512 rows), one image per workgroup, the longer-running
// role first: workgroup `blk` of that part of k_sinkhorn_large's launch (sinkhorn_cluster.hpp).
__device__ __forceinline__ void sinkhorn_tall_block(const SinkhornArgs& A, const int32_t* __restrict__ work, int B,
                                                    int blk) {
  constexpr int NV = kWorkLists;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int cnt = work[kVariantTeamTall];
  if (blk < cnt) {
    const int img = work[NV + kVariantTeamTall * B + blk];
    const int n_img = A.offsets[img + 1] - A.offsets[img];
    const int r_img = n_img - min(max(A.keep[img], 0), max(n_img, 0));
    if (r_img <= TeamTall32::kMaxR) sinkhorn_team_image<TeamTall32, float>(A, img, wave, lane);
    else if (r_img <= TeamTall48::kMaxR) sinkhorn_team_image<TeamTall48, float>(A, img, wave, lane);
    else sinkhorn_team_image<TeamTall, float>(A, img, wave, lane);
    return;
  }
  blk -= cnt;
  cnt = work[kVariantTall];
  if (blk < cnt) sinkhorn_waves_image<TallShape>(A, work[NV + kVariantTall * B + blk], 0, wave, lane);
}

// Team C's images held as fp32, one at a time per workgroup, two workgroups per
// compute unit (at most 128 registers per lane); the grid is at most two
// workgroups per compute unit, which take the list in turns.  Launched when the
// kernel matrix's range fits fp32.
__global__ __launch_bounds__(kDualThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_sinkhorn_c32(
    SinkhornArgs A, const int32_t* __restrict__ work, int B, const int32_t* __restrict__ status) {
  if (status[0]) return;
  const int cnt = work[kVariantC32];
  for (int blk = blockIdx.x; blk < cnt; blk += gridDim.x) {
    if (blk != static_cast<int>(blockIdx.x)) __syncthreads();   // the previous image's LDS is still being read
    sinkhorn_team_image<TeamC32, float>(A, work[kWorkLists + kVariantC32 * B + blk], threadIdx.x >> 6, threadIdx.x & 63);
  }
}

}  // namespace rtp
