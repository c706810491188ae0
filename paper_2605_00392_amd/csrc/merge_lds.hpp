// Merge and compaction (Eq. 6): out_i = T_i + alpha * sum_j P_ij T_j, streamed.
//
// A workgroup of 4 waves owns 32 consecutive kept rows of one image.  The
// pruned rows are staged through LDS in chunks (all of them at once when they
// fit, which is the common case: the pruned set is small), so every kept row
// is read from memory exactly once and written exactly once, and the pruned
// rows come from LDS for all 32 kept rows.  A wave merges two kept rows at a
// time: it holds both rows in registers (a lane owns the 4-element groups
// lane + 64 k), walks the staged pruned rows with the plan entries P_ij
// broadcast from a lane-distributed copy of the plan row, accumulates in fp32
// and rounds once on the store.
#pragma once
#include "common.hpp"

namespace rtp {

constexpr int kMergeBlockRows = 32;
constexpr int kMergeLdsBytes = 30 * 1024;
constexpr int kMergeMaxChunk = 64;   // pruned rows per LDS chunk, at most one per lane

template <typename T, int KMAX>
__global__ __launch_bounds__(256) void k_merge_lds(
    const T* __restrict__ tokens, const int32_t* __restrict__ offsets, int D,
    const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ keep,
    const int32_t* __restrict__ out_offsets, const float* __restrict__ plan,
    const long long* __restrict__ plan_offsets, float alpha, int max_tokens, T* __restrict__ out,
    const int32_t* __restrict__ status) {
  if (status && status[0]) return;
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[kMergeLdsBytes];
  T* lds = reinterpret_cast<T*>(lds_raw);
  const int b = blockIdx.y;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  if (lo < 0 || n <= 0 || n > max_tokens) return;
  const int m = min(max(keep[b], 0), n), r = n - m;
  const int i0 = blockIdx.x * kMergeBlockRows;
  if (i0 >= m) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ngroups = D >> 2;
  const int32_t* sel = sel_idx + lo;
  const float* P = (r > 0) ? plan + plan_offsets[b] : nullptr;
  const size_t obase = static_cast<size_t>(out_offsets[b]);
  const int chunk = min(min(kMergeMaxChunk, kMergeLdsBytes / static_cast<int>(D * sizeof(T))), max(r, 1));
  const int nchunks = (r + chunk - 1) / chunk;

  for (int pass = 0; pass < kMergeBlockRows / 8; ++pass) {
    if (i0 + pass * 8 >= m) break;                 // uniform over the workgroup
    const int ia = i0 + pass * 8 + wave * 2, ib = ia + 1;
    const bool va = ia < m, vb = ib < m;
    float xa[KMAX][4], xb[KMAX][4], acca[KMAX][4], accb[KMAX][4];
    const T* rowa = tokens + static_cast<size_t>(lo + clamp_index(sel[min(ia, m - 1)], n)) * D;
    const T* rowb = tokens + static_cast<size_t>(lo + clamp_index(sel[min(ib, m - 1)], n)) * D;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      const int g = lane + kWave * k;
      if (g < ngroups) {
        load4(rowa + 4 * g, xa[k]);
        load4(rowb + 4 * g, xb[k]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) xa[k][e] = xb[k][e] = 0.f;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) acca[k][e] = accb[k][e] = 0.f;
    }
    for (int c = 0; c < nchunks; ++c) {
      const int j0 = c * chunk, jn = min(chunk, r - j0);
      if (nchunks > 1 || pass == 0) {
        if (nchunks > 1) __syncthreads();          // the previous chunk is still being read
        for (int idx = threadIdx.x; idx < jn * ngroups; idx += 256) {
          const int j = idx / ngroups, g = idx - j * ngroups;
          const T* src = tokens + static_cast<size_t>(lo + clamp_index(sel[m + j0 + j], n)) * D + 4 * g;
          if (sizeof(T) == 2)
            *reinterpret_cast<uint2*>(lds + j * D + 4 * g) = *reinterpret_cast<const uint2*>(src);
          else
            *reinterpret_cast<uint4*>(lds + j * D + 4 * g) = *reinterpret_cast<const uint4*>(src);
        }
        __syncthreads();
      }
      // lane l holds the plan entries of pruned row j0 + l for the wave's two kept rows
      float pa = 0.f, pb = 0.f;
      if (lane < jn) {
        if (va) pa = P[static_cast<long long>(ia) * r + j0 + lane];
        if (vb) pb = P[static_cast<long long>(ib) * r + j0 + lane];
      }
      for (int j = 0; j < jn; ++j) {
        const float pja = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, pa), j));
        const float pjb = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, pb), j));
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
          const int g = lane + kWave * k;
          if (g < ngroups) {
            float xj[4];
            load4(lds + j * D + 4 * g, xj);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              acca[k][e] = fmaf(pja, xj[e], acca[k][e]);
              accb[k][e] = fmaf(pjb, xj[e], accb[k][e]);
            }
          }
        }
      }
    }
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      const int g = lane + kWave * k;
      if (g < ngroups) {
        float o[4];
        if (va) {
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = fmaf(alpha, acca[k][e], xa[k][e]);
          store4(out + (obase + ia) * D + 4 * g, o);
        }
        if (vb) {
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = fmaf(alpha, accb[k][e], xb[k][e]);
          store4(out + (obase + ib) * D + 4 * g, o);
        }
      }
    }
  }
}

}  // namespace rtp
