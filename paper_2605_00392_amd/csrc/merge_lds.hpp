// Merge and compaction (Eq. 6): out_i = T_i + alpha * sum_j P_ij T_j, streamed.
//
// A workgroup of 4 waves owns 16 consecutive kept rows of one image (measured:
// many small single-pass workgroups keep the memory system busier than fewer
// multi-pass ones, 0.38 ms against 0.46 ms at 64 rows on the 1024 x 400 batch,
// although the pruned rows are then re-read from L2 by more workgroups).  The
// pruned rows are staged through LDS in chunks (all of them at once when they
// fit, which is the common case: the pruned set is small), so every kept row
// is read from memory exactly once and written exactly once, and the pruned
// rows come from LDS for all the workgroup's kept rows.  A wave merges four kept rows at a
// time: their loads are issued together and stay packed in registers (a lane
// owns the 4-element groups lane + 64 k), the staged pruned rows are walked
// once for all four with the plan entries P_ij broadcast from a
// lane-distributed copy of the plan rows, accumulation is fp32, and the sum is
// rounded once on the store.
#pragma once
#include "common.hpp"

namespace rtp {

constexpr int kMergeBlockRows = 16;   // kept rows per workgroup
constexpr int kMergeWaveRows = 4;    // kept rows a wave merges at a time
constexpr int kMergeLdsBytes = 30 * 1024;
constexpr int kMergeMaxChunk = 64;   // pruned rows per LDS chunk, at most one per lane

// EXACT: D == 256 KMAX, every lane owns exactly KMAX groups (no bounds tests).
template <typename T, int KMAX, bool EXACT>
__global__ __launch_bounds__(256) void k_merge_lds(
    const T* __restrict__ tokens, const int32_t* __restrict__ offsets, int D,
    const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ keep,
    const int32_t* __restrict__ out_offsets, const float* __restrict__ plan,
    const long long* __restrict__ plan_offsets, float alpha, int max_tokens, MergeSkip skip, T* __restrict__ out,
    const int32_t* __restrict__ status) {
  typedef typename Raw4<T>::type raw_t;
  constexpr int NB = kMergeWaveRows;
  constexpr int kPassRows = 4 * NB;                // rows the workgroup finishes per pass
  if (status && status[0]) return;
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[kMergeLdsBytes];
  T* lds = reinterpret_cast<T*>(lds_raw);
  const int b = blockIdx.y;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  if (lo < 0 || n <= 0 || n > max_tokens) return;
  const int m = min(max(keep[b], 0), n), r = n - m;
  const int i0 = blockIdx.x * kMergeBlockRows;
  if (i0 >= m || merge_elsewhere(skip, r)) return;   // larger pruned sets: the matrix-core kernels
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ngroups = D >> 2;
  const int32_t* sel = sel_idx + lo;
  const float* P = (r > 0) ? plan + plan_offsets[b] : nullptr;
  const size_t obase = static_cast<size_t>(out_offsets[b]);
  const int chunk = min(min(kMergeMaxChunk, kMergeLdsBytes / static_cast<int>(D * sizeof(T))), max(r, 1));
  const int nchunks = (r + chunk - 1) / chunk;

  for (int pass = 0; pass < kMergeBlockRows / kPassRows; ++pass) {
    if (i0 + pass * kPassRows >= m) break;         // uniform over the workgroup
    const int ia = i0 + pass * kPassRows + wave * NB;
    raw_t raw[NB][KMAX];
    float acc[NB][KMAX][4];
    // the wave's NB token indices with one load, then all row loads back to back
    const int my_tok = clamp_index(sel[min(ia + min(lane, NB - 1), m - 1)], n);
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int tok = __builtin_amdgcn_readlane(my_tok, u);
      const T* row = tokens + static_cast<size_t>(lo + tok) * D;
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        const int g = lane + kWave * k;
        if (EXACT || g < ngroups) raw[u][k] = load_stream(reinterpret_cast<const raw_t*>(row + 4 * g));
        else raw[u][k] = raw_t{};
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[u][k][e] = 0.f;
      }
    }
    for (int c = 0; c < nchunks; ++c) {
      const int j0 = c * chunk, jn = min(chunk, r - j0);
      // lane l holds the plan entries of pruned row j0 + l for the wave's kept rows
      // (requested before the staging so that they travel together with it)
      float pl[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u)
        pl[u] = (lane < jn && ia + u < m) ? P[static_cast<long long>(ia + u) * r + j0 + lane] : 0.f;
      if (nchunks > 1 || pass == 0) {
        if (nchunks > 1) __syncthreads();          // the previous chunk is still being read
        // each wave stages whole pruned rows, two at a time: one load for the token
        // indices, then the rows' loads back to back, then the LDS writes
        const int p_tok = clamp_index(sel[m + j0 + min(lane, jn - 1)], n);
        for (int j = 2 * wave; j < jn; j += 8) {
          const int ja = j, jb = min(j + 1, jn - 1);
          const T* ra = tokens + static_cast<size_t>(lo + __builtin_amdgcn_readlane(p_tok, ja)) * D;
          const T* rb = tokens + static_cast<size_t>(lo + __builtin_amdgcn_readlane(p_tok, jb)) * D;
          raw_t va_[KMAX], vb_[KMAX];
#pragma unroll
          for (int k = 0; k < KMAX; ++k) {
            const int g = lane + kWave * k;
            if (EXACT || g < ngroups) {
              va_[k] = *reinterpret_cast<const raw_t*>(ra + 4 * g);
              vb_[k] = *reinterpret_cast<const raw_t*>(rb + 4 * g);
            }
          }
#pragma unroll
          for (int k = 0; k < KMAX; ++k) {
            const int g = lane + kWave * k;
            if (EXACT || g < ngroups) {
              *reinterpret_cast<raw_t*>(lds + ja * D + 4 * g) = va_[k];
              *reinterpret_cast<raw_t*>(lds + jb * D + 4 * g) = vb_[k];
            }
          }
        }
        __syncthreads();
      }
      for (int j = 0; j < jn; ++j) {
        float pj[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u)
          pj[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, pl[u]), j));
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
          const int g = lane + kWave * k;
          if (EXACT || g < ngroups) {
            float xj[4];
            unpack4(*reinterpret_cast<const raw_t*>(lds + j * D + 4 * g), xj);
#pragma unroll
            for (int u = 0; u < NB; ++u)
#pragma unroll
              for (int e = 0; e < 4; ++e) acc[u][k][e] = fmaf(pj[u], xj[e], acc[u][k][e]);
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      if (ia + u >= m) break;
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        const int g = lane + kWave * k;
        if (EXACT || g < ngroups) {
          float x[4], o[4];
          unpack4(raw[u][k], x);
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = fmaf(alpha, acc[u][k][e], x[e]);
          store4_stream(out + (obase + ia + u) * D + 4 * g, o);
        }
      }
    }
  }
}

}  // namespace rtp
