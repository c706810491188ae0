// Stage 2 and the merge, general-shape kernels: every image size and token
// width within the library's limits goes through these; they keep the Sinkhorn
// kernel matrix in global memory (L2-resident) and use plain fp64 / fp32 vector
// arithmetic.
//
//   k_scores   K_ij = exp((S_ij - shift) / eps), S = cosine of Eq. 3
//   k_sinkhorn T multiplicative Sinkhorn iterations on the dustbin-augmented
//              kernel (Appendix C in the exponentiated variables
//              x = exp(u), y = exp(v)), the plan, and the hard pairing
//   k_merge    Eq. 6 with compaction
#pragma once
#include "common.hpp"
#include "sinkhorn_team.hpp"

namespace rtp {

constexpr int kScoreRowsPerBlock = 16;

// Workgroup = 4 waves, each wave owns kept rows of a 16-row tile and walks all
// pruned rows; a (kept, pruned) dot product is accumulated in fp64 across the
// wave's lanes.  Lane layout as in k_norms.
template <typename T, int KMAX>
__global__ __launch_bounds__(256) void k_scores(
    const T* __restrict__ tokens, const int32_t* __restrict__ offsets, int D,
    const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ keep,
    const long long* __restrict__ plan_offsets, const double* __restrict__ norm64, DevParams p,
    double* __restrict__ kmat, long long plan_cap, double* __restrict__ scores_out,
    const int32_t* __restrict__ status) {
  if (status[0]) return;
  const int b = blockIdx.y;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  const int m = min(max(keep[b], 0), n), r = n - m;
  const int i0 = blockIdx.x * kScoreRowsPerBlock;
  if (r <= 0 || i0 >= m) return;
  if (!plan_fits(plan_offsets[b], m, r, plan_cap)) return;
  const int i1 = min(m, i0 + kScoreRowsPerBlock);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ngroups = D >> 2;
  const long long po = plan_offsets[b];
  const int k_layout = kernel_layout(p, m, r);
  const int32_t* sel = sel_idx + lo;
  const double inv_eps = 1.0 / p.eps;

  for (int i = i0 + wave; i < i1; i += 4) {
    const int ti = clamp_index(sel[i], n);
    const T* rowi = tokens + static_cast<size_t>(lo + ti) * D;
    float xi[KMAX][4];
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      const int g = lane + kWave * k;
      if (g < ngroups) load4(rowi + 4 * g, xi[k]);
      else xi[k][0] = xi[k][1] = xi[k][2] = xi[k][3] = 0.f;
    }
    const double ni = norm64[lo + ti];
    for (int j = 0; j < r; ++j) {
      const int tj = clamp_index(sel[m + j], n);
      const T* rowj = tokens + static_cast<size_t>(lo + tj) * D;
      double dot = 0.0;
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        const int g = lane + kWave * k;
        if (g < ngroups) {
          float xj[4];
          load4(rowj + 4 * g, xj);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            dot = fma(static_cast<double>(xi[k][e]), static_cast<double>(xj[e]), dot);
        }
      }
      dot = wave_sum(dot);
      if (lane == 0) {
        const double nj = norm64[lo + tj];
        const double s = dot / fmax(ni * nj, kTinyNorm * kTinyNorm);
        const long long at = static_cast<long long>(i) * r + j;
        store_kernel(kmat, po, i, j, m, r, exp_nonpositive((s - p.shift) * inv_eps), k_layout);
        if (scores_out) scores_out[po + at] = s;
      }
    }
  }
}

// One workgroup of 1024 threads per image.  With K = exp((S - shift)/eps) on the
// kept x pruned block and kz = exp((z - shift)/eps) on the dustbin row, column
// and corner, an iteration of Appendix C reads
//     x_i = mu_i / sum_j K_ij y_j      (u-update, i = 0..M; mu = [1_M, R])
//     y_j = nu_j / sum_i K_ij x_i      (v-update, j = 0..R; nu = [1_R, M])
// starting from y = 1; x is exp(u) up to the common factor exp(shift/eps),
// which cancels in P_bar_ij = x_i K_ij y_j.
__global__ __launch_bounds__(1024) void k_sinkhorn(
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ keep,
    const long long* __restrict__ plan_offsets, DevParams p, const double* __restrict__ kmat,
    long long plan_cap, float* __restrict__ plan_out, int32_t* __restrict__ pair_out,
    int skip_team_shapes, int mode, const int32_t* __restrict__ status) {
  if (status[0]) return;
  __shared__ double xy[kMaxTokens + 2];
  __shared__ double part[16][kWave];
  __shared__ float bestv[16][kWave];
  __shared__ int besti[16][kWave];
  __shared__ double red[16];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  if (n <= 0) return;
  const int m = min(max(keep[b], 0), n), r = n - m;
  if (skip_team_shapes && sinkhorn_variant(m, r, mode) != kGeneralVariant) return;   // done elsewhere
  if (pair_out)
    for (int i = tid; i < m; i += 1024) pair_out[lo + i] = i;
  if (r <= 0 || m <= 0) return;
  if (!plan_fits(plan_offsets[b], m, r, plan_cap)) return;
  const double* K = kmat + plan_offsets[b];
  double* x = xy;           // m + 1 entries
  double* y = xy + (m + 1);  // r + 1 entries
  const double kz = exp((p.z - p.shift) / p.eps);
  const double x_init = exp(p.shift / p.eps);   // T = 0: u = 0
  for (int i = tid; i <= m; i += 1024) x[i] = x_init;
  for (int j = tid; j <= r; j += 1024) y[j] = 1.0;
  double sum_y = static_cast<double>(r) + 1.0;
  __syncthreads();

  for (int it = 0; it < p.iters; ++it) {
    // u-update.
    const double y_dust = y[r];
    for (int i = wave; i < m; i += 16) {
      const double* Ki = K + static_cast<long long>(i) * r;
      double s = 0.0;
      for (int j = lane; j < r; j += kWave) s = fma(Ki[j], y[j], s);
      s = wave_sum(s);
      if (lane == 0) x[i] = 1.0 / fma(kz, y_dust, s);
    }
    if (tid == 0) x[m] = static_cast<double>(r) / (kz * sum_y);
    __syncthreads();
    // v-update.
    double lx = 0.0;
    for (int i = tid; i <= m; i += 1024) lx += x[i];
    const double sum_x = block_sum<1024>(lx, red);
    const double x_dust = x[m];
    for (int j0 = 0; j0 < r; j0 += kWave) {
      const int j = j0 + lane;
      double s = 0.0;
      if (j < r)
        for (int i = wave; i < m; i += 16) s = fma(K[static_cast<long long>(i) * r + j], x[i], s);
      part[wave][lane] = s;
      __syncthreads();
      if (wave == 0 && j < r) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += part[w][lane];
        y[j] = 1.0 / fma(kz, x_dust, t);
      }
      __syncthreads();
    }
    if (tid == 0) y[r] = static_cast<double>(m) / (kz * sum_x);
    __syncthreads();
    double ly = 0.0;
    for (int j = tid; j <= r; j += 1024) ly += y[j];
    sum_y = block_sum<1024>(ly, red);
  }

  // Plan (fp32) and pairing: column arg-max of the fp32 plan entries, lowest
  // kept rank first; the dustbin row wins only when strictly larger.
  if (plan_out) {
    float* P = plan_out + plan_offsets[b];
    for (int i = wave; i < m; i += 16) {
      const double xi = x[i];
      for (int j = lane; j < r; j += kWave)
        P[static_cast<long long>(i) * r + j] =
            static_cast<float>(xi * K[static_cast<long long>(i) * r + j] * y[j]);
    }
  }
  if (pair_out) {
    for (int j0 = 0; j0 < r; j0 += kWave) {
      const int j = j0 + lane;
      float bv = -1.f;
      int bi = 0x7fffffff;
      if (j < r) {
        const double yj = y[j];
        for (int i = wave; i < m; i += 16) {
          const float v = static_cast<float>(x[i] * K[static_cast<long long>(i) * r + j] * yj);
          if (v > bv) { bv = v; bi = i; }
        }
      }
      bestv[wave][lane] = bv;
      besti[wave][lane] = bi;
      __syncthreads();
      if (wave == 0 && j < r) {
        float v = bestv[0][lane];
        int idx = besti[0][lane];
#pragma unroll
        for (int w = 1; w < 16; ++w) {
          const float ov = bestv[w][lane];
          const int oi = besti[w][lane];
          if (ov > v || (ov == v && oi < idx)) { v = ov; idx = oi; }
        }
        const float dust = static_cast<float>(x[m] * kz * y[j]);
        pair_out[lo + m + j] = dust > v ? -1 : idx;
      }
      __syncthreads();
    }
  }
}

constexpr int kMergeRowsPerBlock = 4;

// Workgroup = 256 threads covers 4 kept rows; a thread owns 4-element groups
// g = tid + 256 k of the row.  fp32 accumulation, one rounding on store.
template <typename T, int KMAX>
__global__ __launch_bounds__(256) void k_merge(
    const T* __restrict__ tokens, const int32_t* __restrict__ offsets, int D,
    const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ keep,
    const int32_t* __restrict__ out_offsets, const float* __restrict__ plan,
    const long long* __restrict__ plan_offsets, float alpha, int max_tokens, MergeSkip skip, T* __restrict__ out,
    const int32_t* __restrict__ status) {
  if (status && status[0]) return;
  const int b = blockIdx.y;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  if (lo < 0 || n <= 0 || n > max_tokens) return;
  const int m = min(max(keep[b], 0), n), r = n - m;
  const int i0 = blockIdx.x * kMergeRowsPerBlock;
  if (i0 >= m || merge_elsewhere(skip, r)) return;   // larger pruned sets: the matrix-core kernels
  const int rows = min(kMergeRowsPerBlock, m - i0);
  const int ngroups = D >> 2;
  const int32_t* sel = sel_idx + lo;
  const float* P = (r > 0) ? plan + plan_offsets[b] : nullptr;
  const size_t obase = static_cast<size_t>(out_offsets[b]);

#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    const int g = threadIdx.x + 256 * k;
    if (g >= ngroups) break;
    float acc[kMergeRowsPerBlock][4];
#pragma unroll
    for (int a = 0; a < kMergeRowsPerBlock; ++a) acc[a][0] = acc[a][1] = acc[a][2] = acc[a][3] = 0.f;
    for (int j = 0; j < r; ++j) {
      float xj[4];
      load4(tokens + static_cast<size_t>(lo + clamp_index(sel[m + j], n)) * D + 4 * g, xj);
#pragma unroll
      for (int a = 0; a < kMergeRowsPerBlock; ++a) {
        if (a < rows) {
          const float pij = P[static_cast<long long>(i0 + a) * r + j];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[a][e] = fmaf(pij, xj[e], acc[a][e]);
        }
      }
    }
#pragma unroll
    for (int a = 0; a < kMergeRowsPerBlock; ++a) {
      if (a < rows) {
        float xi[4], o[4];
        load4(tokens + static_cast<size_t>(lo + clamp_index(sel[i0 + a], n)) * D + 4 * g, xi);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = fmaf(alpha, acc[a][e], xi[e]);
        store4_stream(out + (obase + i0 + a) * D + 4 * g, o);
      }
    }
  }
}

}  // namespace rtp
