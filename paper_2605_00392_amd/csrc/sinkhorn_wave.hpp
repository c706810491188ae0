// Sinkhorn (Appendix C) for one image on one or two waves, for the small pruned
// sets that dominate a batch of pages with a dynamic ratio.
//
// The dustbin row and column are ordinary entries of the augmented kernel
// Kb = exp((S_bar - shift)/eps), (M+1) x (R+1), with marginals a = [1_M, R],
// b = [1_R, M].  An image takes W waves; lane l of wave w holds RPT rows
// (64 w + l, then every 64 W) with all C columns, RPT C doubles:
//     WaveShape  W = 1, RPT = 7, C = 8    M + 1 <= 448, R + 1 <= 8
//     PairShape  W = 2, RPT = 4, C = 16   M + 1 <= 512, R + 1 <= 16
//   u-update  the row sums are lane-local; the y_j sit in scalar registers
//             (read from the lane that owns the column).
//   v-update  every lane forms C partial column sums over its rows.  The
//             64 x C partials of a wave are added up by a reduce-scatter:
//             halving exchanges over lane bits 5 and 4, an all-reduce of what
//             is left over the low lane bits, and one (C = 8) or two (C = 16)
//             more halvings over bits 2 and 3.  Each lane then owns the total
//             of one column (C = 8: 13 additions instead of 48); with two waves
//             the two totals meet in LDS (one barrier per iteration).  The
//             owner computes that column's y once.
#pragma once
#include "common.hpp"
#include "sinkhorn_team.hpp"

namespace rtp {

// Sum over the wave of t[0..C), scattered: the return value is the total of
// column `wave_column<C>(lane)`.
template <int C>
__device__ __forceinline__ int wave_column(int lane) {
  const int b5 = lane >> 5, b4 = (lane >> 4) & 1, b3 = (lane >> 3) & 1, b2 = (lane >> 2) & 1;
  return C == 8 ? 4 * b5 + 2 * b4 + b3 : 8 * b5 + 4 * b4 + 2 * b2 + b3;
}
template <int C>
__device__ __forceinline__ int column_lane(int c) {     // a lane that owns column c
  return C == 8 ? 32 * (c >> 2) + 16 * ((c >> 1) & 1) + 8 * (c & 1)
                : 32 * (c >> 3) + 16 * ((c >> 2) & 1) + 4 * ((c >> 1) & 1) + 8 * (c & 1);
}
template <int C>
__device__ __forceinline__ double reduce_scatter(const double (&t)[C], int lane) {
  static_assert(C == 8 || C == 16, "two shapes");
  const bool b3 = (lane & 8) != 0;
  double h[C / 2];
#pragma unroll
  for (int c = 0; c < C / 2; ++c) h[c] = halve32(t[c], t[c + C / 2]);       // bit 5 clear: the lower half
  double q[C / 4];
#pragma unroll
  for (int c = 0; c < C / 4; ++c) q[c] = halve16(h[c], h[c + C / 4]);       // bit 4 clear: the lower half
#pragma unroll
  for (int c = 0; c < C / 4; ++c) {
    q[c] += dpp_move<0xB1>(q[c]);                                           // lane ^ 1
    q[c] += dpp_move<0x4E>(q[c]);                                           // lane ^ 2
  }
  double v0, v1;
  if (C == 8) {
    v0 = q[0] + dpp_move<0x141>(q[0]);                                      // the other quad of the 8 lanes
    v1 = q[1] + dpp_move<0x141>(q[1]);
  } else {
    // the quads agree, so mirroring the 8 lanes pairs each quad with the other
    // one: bit 2 clear keeps the lower two values
    const bool b2 = (lane & 4) != 0;
    const double k0 = b2 ? q[C == 8 ? 0 : 2] : q[0], s0 = b2 ? q[0] : q[C == 8 ? 0 : 2];
    const double k1 = b2 ? q[C == 8 ? 1 : 3] : q[1], s1 = b2 ? q[1] : q[C == 8 ? 1 : 3];
    v0 = k0 + dpp_move<0x141>(s0);
    v1 = k1 + dpp_move<0x141>(s1);
  }
  const double keep = b3 ? v1 : v0, send = b3 ? v0 : v1;
  // C = 8: all 8 lanes agree, so mirroring the 16 lanes reaches bit 3's partner;
  // C = 16: rotate the row of 16 lanes by 8, which is lane ^ 8 exactly
  return keep + (C == 8 ? dpp_move<0x140>(send) : dpp_move<0x128>(send));
}

// The same scatter with the maximum of 64-bit keys in place of the sum: the return
// value is the largest of the wave's 64 candidates for column `wave_column<C>(lane)`.
__device__ __forceinline__ long long key_max(long long a, long long b) { return a > b ? a : b; }
__device__ __forceinline__ long long key_of(int hi, int lo) {
  return (static_cast<long long>(hi) << 32) | static_cast<unsigned>(lo);
}
template <int CTRL>
__device__ __forceinline__ long long dpp_move_key(long long v) {
  const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(v >> 32), CTRL, 0xF, 0xF, false);
  return key_of(hi, lo);
}
__device__ __forceinline__ long long max_halve32(long long a, long long b) {   // as halve32
  const auto lo = __builtin_amdgcn_permlane32_swap(static_cast<unsigned>(a), static_cast<unsigned>(b), false, false);
  const auto hi = __builtin_amdgcn_permlane32_swap(static_cast<unsigned>(a >> 32), static_cast<unsigned>(b >> 32), false, false);
  return key_max(key_of(static_cast<int>(hi[0]), static_cast<int>(lo[0])), key_of(static_cast<int>(hi[1]), static_cast<int>(lo[1])));
}
__device__ __forceinline__ long long max_halve16(long long a, long long b) {   // as halve16
  const auto lo = __builtin_amdgcn_permlane16_swap(static_cast<unsigned>(a), static_cast<unsigned>(b), false, false);
  const auto hi = __builtin_amdgcn_permlane16_swap(static_cast<unsigned>(a >> 32), static_cast<unsigned>(b >> 32), false, false);
  return key_max(key_of(static_cast<int>(hi[0]), static_cast<int>(lo[0])), key_of(static_cast<int>(hi[1]), static_cast<int>(lo[1])));
}
template <int C>
__device__ __forceinline__ long long max_scatter(const long long (&t)[C], int lane) {
  static_assert(C == 8 || C == 16, "two shapes");
  const bool b3 = (lane & 8) != 0;
  long long h[C / 2];
#pragma unroll
  for (int c = 0; c < C / 2; ++c) h[c] = max_halve32(t[c], t[c + C / 2]);
  long long q[C / 4];
#pragma unroll
  for (int c = 0; c < C / 4; ++c) q[c] = max_halve16(h[c], h[c + C / 4]);
#pragma unroll
  for (int c = 0; c < C / 4; ++c) {
    q[c] = key_max(q[c], dpp_move_key<0xB1>(q[c]));                         // lane ^ 1
    q[c] = key_max(q[c], dpp_move_key<0x4E>(q[c]));                         // lane ^ 2
  }
  long long v0, v1;
  if (C == 8) {
    v0 = key_max(q[0], dpp_move_key<0x141>(q[0]));
    v1 = key_max(q[1], dpp_move_key<0x141>(q[1]));
  } else {
    const bool b2 = (lane & 4) != 0;
    const long long k0 = b2 ? q[C == 8 ? 0 : 2] : q[0], s0 = b2 ? q[0] : q[C == 8 ? 0 : 2];
    const long long k1 = b2 ? q[C == 8 ? 1 : 3] : q[1], s1 = b2 ? q[1] : q[C == 8 ? 1 : 3];
    v0 = key_max(k0, dpp_move_key<0x141>(s0));
    v1 = key_max(k1, dpp_move_key<0x141>(s1));
  }
  const long long keep = b3 ? v1 : v0, send = b3 ? v0 : v1;
  return key_max(keep, C == 8 ? dpp_move_key<0x140>(send) : dpp_move_key<0x128>(send));
}

// One image on W waves.  `b` < 0 means no image: the waves only keep the
// workgroup's barriers company.  `slot` numbers the image inside the workgroup,
// `tw` the wave inside the image.
template <typename S>
__device__ __forceinline__ void sinkhorn_waves_image(const SinkhornArgs& A, int b, int slot, int tw, int lane) {
  constexpr int W = S::kWaves, RPT = S::kRows, C = S::kCols, TR = 64 * W;
  const DevParams& p = A.p;
  int lo = 0, m = 0, r = 0;
  bool active = false;
  if (b >= 0) {
    lo = A.offsets[b];
    const int n = A.offsets[b + 1] - lo;
    m = min(max(A.keep[b], 0), max(n, 0));
    r = max(n, 0) - m;
    active = n > 0 && S::fits(m, r);
  }
  int32_t* __restrict__ pair_out = A.pair_out;
  if (active && pair_out)
    for (int i = 64 * tw + lane; i < m; i += TR) pair_out[lo + i] = i;
  active = active && r > 0 && m > 0 && plan_fits(A.plan_offsets[b], m, r, A.plan_cap);
  if (W == 1 && !active) return;
  if (!active) { m = 0; r = 0; }
  const long long po = active ? A.plan_offsets[b] : 0;
  const double* __restrict__ Kg = A.kmat + po;
  const double kz = exp((p.z - p.shift) / p.eps);
  const int row0 = 64 * tw + lane;

  // Rows beyond the dustbin get a single 1 and a zero marginal, so their x is an
  // ordinary 0 and they add nothing to a column sum.
  double K[RPT][C], arow[RPT];
  // Loads are unconditional (from a clamped position of a valid image, or the
  // matrix's first entry otherwise) and all issued before the first of them is used,
  // so that they are in flight together (left to itself the compiler waits for each
  // one before the next: 20 us for a lane's 64 entries).  The matrix is stored column
  // by column (kKernelColsF64): the lanes of a load read consecutive entries.
#pragma unroll
  for (int a = 0; a < RPT; ++a) {
    const double* col0 = Kg + (active ? min(row0 + TR * a, m - 1) : 0);
#pragma unroll
    for (int c = 0; c < C; ++c) K[a][c] = col0[active ? static_cast<long long>(min(c, r - 1)) * m : 0];
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int a = 0; a < RPT; ++a) {
    const int i = row0 + TR * a;
#pragma unroll
    for (int c = 0; c < C; ++c) {
      double v = 0.0;
      if (active && i <= m && c <= r) v = (i < m && c < r) ? K[a][c] : kz;
      if ((i > m || !active) && c == 0) v = 1.0;
      K[a][c] = v;
    }
    arow[a] = !active ? 0.0 : i < m ? 1.0 : (i == m ? static_cast<double>(r) : 0.0);
  }
  const int own = wave_column<C>(lane);                 // the column this lane finishes
  const double bcol = own < r ? 1.0 : static_cast<double>(m);
  const bool own_valid = active && own <= r;

  __shared__ double xchg[2][kSinkhornBlockWaves][64];   // W = 2: the two waves' column totals

  double x[RPT], y[C];
  const double x_init = exp(p.shift / p.eps);          // T = 0 leaves u = 0
#pragma unroll
  for (int a = 0; a < RPT; ++a) x[a] = (active && row0 + TR * a <= m) ? x_init : 0.0;
#pragma unroll
  for (int c = 0; c < C; ++c) y[c] = (c <= r) ? 1.0 : 0.0;

  // The iteration is a fixed map of (x, y) in the device's arithmetic, so the end of
  // the T iterations is known as soon as the iterates repeat (`settled_stop`): the
  // rest is skipped without changing a bit of the result.  With several waves per image
  // the waves agree through LDS, and the waves of a settled image keep meeting the
  // workgroup's barrier, which the other images of the workgroup still use.
  __shared__ int moved[2][kSinkhornBlockWaves];
  int stop_at = p.iters;
  for (int it = 0; it < stop_at; ++it) {
    // ---- u-update ----
    bool differs = false;
#pragma unroll
    for (int a = 0; a < RPT; ++a) {
      double acc = K[a][0] * y[0];
#pragma unroll
      for (int c = 1; c < C; ++c) acc = fma(K[a][c], y[c], acc);
      const double xn = arow[a] * rcp64_tight(acc);
      differs |= __double_as_longlong(xn) != __double_as_longlong(x[a]);
      x[a] = xn;
    }
    int any_moved = __builtin_amdgcn_ballot_w64(differs) != 0 ? 1 : 0;
    // ---- v-update ----
    double t[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
      double acc = K[0][c] * x[0];
#pragma unroll
      for (int a = 1; a < RPT; ++a) acc = fma(K[a][c], x[a], acc);
      t[c] = acc;
    }
    double total = reduce_scatter<C>(t, lane);
    if (W > 1) {
      xchg[it & 1][W * slot + tw][lane] = total;
      if (lane == 0) moved[it & 1][W * slot + tw] = any_moved;
      __syncthreads();
      total = 0.0;
      any_moved = 0;
#pragma unroll
      for (int w = 0; w < W; ++w) {
        total += xchg[it & 1][W * slot + w][lane];   // same order in every wave
        any_moved |= moved[it & 1][W * slot + w];
      }
    }
    stop_at = settled_stop(stop_at, it, any_moved != 0);   // the same in every wave of the image
    const double y_own = own_valid ? bcol * rcp64_tight(total) : 0.0;
#pragma unroll
    for (int c = 0; c < C; ++c) y[c] = read_lane(y_own, column_lane<C>(c));
  }
  if (W > 1)
    for (int rest = stop_at; rest < p.iters; ++rest) __syncthreads();
  if (W == 1 && !active) return;

  // ---- plan and pairing (row m is the dustbin) ----
  float bv[C];
  int bi[C];
#pragma unroll
  for (int c = 0; c < C; ++c) { bv[c] = -1.f; bi[c] = 0x7fffffff; }
  if (active) {
    float* P = A.plan_out ? A.plan_out + po : nullptr;
    // rows recomputed from a value the compiler cannot relate to the one the
    // loads used, so that no entry offset stays in a register across the loop
    int row0_p = row0;
    forget_origin(row0_p);
#pragma unroll
    for (int a = 0; a < RPT; ++a) {
      const int i = row0_p + TR * a;
#pragma unroll
      for (int c = 0; c < C; ++c) {
        if (i <= m && c < r) {
          const float v = static_cast<float>(x[a] * K[a][c] * y[c]);
          if (P && i < m) P[static_cast<long long>(i) * r + c] = v;
          if (v > bv[c]) { bv[c] = v; bi[c] = i; }
        }
      }
    }
  }
  if (!pair_out) return;                               // the same for every wave of the workgroup
  // A column's best over the wave's lanes: the largest key (value bits, then the lower
  // row), found by the scatter that also adds up the column sums: 17 exchanges for 16
  // columns where a butterfly per column takes 96.
  long long key[C];
#pragma unroll
  for (int c = 0; c < C; ++c) key[c] = key_of(__float_as_int(bv[c]), 0x7fffffff - bi[c]);   // plan entries are >= 0
  const long long best = max_scatter<C>(key, lane);
  if (W == 1) {
    if (lane == column_lane<C>(own) && own < r) {
      const int i = 0x7fffffff - static_cast<int>(best);
      pair_out[lo + m + own] = i >= m ? -1 : i;
    }
  } else {
    __shared__ long long pk[kSinkhornBlockWaves][C];
    if (lane == column_lane<C>(own)) pk[W * slot + tw][own] = best;
    __syncthreads();
    if (active && tw == 0 && lane < r) {               // lane = column
      long long k = pk[W * slot][lane];
#pragma unroll
      for (int w = 1; w < W; ++w) k = key_max(k, pk[W * slot + w][lane]);
      const int i = 0x7fffffff - static_cast<int>(k);
      pair_out[lo + m + lane] = i >= m ? -1 : i;
    }
  }
}

}  // namespace rtp
