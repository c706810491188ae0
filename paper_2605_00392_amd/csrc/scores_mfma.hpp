// Cosine scores of Eq. 3 on the matrix cores, accurate to fp64 rounding.
//
// S = T_kept T_prop^T is the operator's one dense contraction.  bf16 x bf16
// products are exact in fp32, but a plain fp32 accumulation over D = 1280 terms
// is off by about 1e-6, which after the division by eps = 0.05 moves plan
// entries by 2e-5 - enough to flip arg-max pairings that the fp64 reference
// separates clearly.  So each v_mfma_f32_16x16x32_bf16 starts from a zero
// accumulator (a 32-term partial dot product, rounded once to fp32 relative to
// a sum 40 times smaller than the full one) and the partials are added in fp64
// vector registers.  Measured against an fp64 evaluation the cosine is off by
// at most 2e-8 (5e-9 rms), i.e. plan entries move by under 5e-7 relative at
// eps = 0.05, inside the 1e-6 band in which an index flip counts as a near-tie.
//
// One wave owns MT tiles of 16 kept rows and walks the pruned rows in groups of
// NT tiles of 16.  Operand fragments are read straight from global memory, 64
// elements of the contraction per step: lane l reads elements 16 (l / 16) .. + 15
// of row (l % 16), so four lanes cover one 128-byte line.  Which 32 of the 64
// elements a matrix instruction contracts is immaterial as long as both
// operands use the same assignment, which they do by construction.
#pragma once
#include "common.hpp"
#include "sinkhorn_team.hpp"

namespace rtp {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

#ifndef RTP_MFMA_ROWS_PER_WAVE
#define RTP_MFMA_ROWS_PER_WAVE 32
#endif
#ifndef RTP_MFMA_WAVES
#define RTP_MFMA_WAVES 1
#endif
constexpr int kMfmaRowsPerWave = RTP_MFMA_ROWS_PER_WAVE;   // MT tiles of 16 kept rows
constexpr int kMfmaWaves = RTP_MFMA_WAVES;
constexpr int kMfmaMinWidth = 1024;   // token widths below this take the fp64 vector score kernel

// Column tiles of 16 pruned rows a wave keeps accumulators for at once (NT of
// the kernel below), chosen on the host from the largest pruned set the call
// can produce: a larger NT reads the kept rows fewer times when R is large but
// costs registers, hence occupancy, when R is small.  Any NT is correct for any
// image: the kernel walks the pruned rows in groups of 16 NT.
inline int score_tiles_per_pass(int max_pruned) {
  const int need = (max_pruned + 15) >> 4;
  return need <= 1 ? 1 : (need == 2 ? 2 : 4);
}

template <int NT>
__global__ __launch_bounds__(64 * kMfmaWaves) void k_scores_mfma(
    const bf16_t* __restrict__ tokens, const int32_t* __restrict__ offsets, int B, int D,
    const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ keep,
    const long long* __restrict__ plan_offsets, const double* __restrict__ norm64, DevParams p,
    double* __restrict__ kmat, long long plan_cap, double* __restrict__ scores_out,
    const int32_t* __restrict__ status) {
  constexpr int MT = kMfmaRowsPerWave / 16;
  if (status[0]) return;
  // Images are taken last to first: the norm pass before this one walks them first
  // to last and the merge after it does so again, so each pass starts on the
  // images its predecessor touched last, which are the ones the memory-side cache
  // still holds (measured on 1 GB batches: 2 % off this kernel, 1 % off the merge).
  //
  // With more than one column tile per pass (NT > 1: the call may have pruned sets
  // of 17 tokens and more) every wave of an image re-reads a sizeable pruned set,
  // so the image's workgroups are given linear ids of one residue modulo eight:
  // workgroups are dealt to the eight XCDs in turn, and the set is then fetched
  // into one L2 instead of eight (1024 pages with 63 pruned tokens each: 2.4 GB
  // fetched from memory without this, against 1.05 GB of tokens).  The grid's y
  // extent is B rounded up to a multiple of eight for it.
  int by = blockIdx.y, bx = blockIdx.x;
  if (NT > 1) {
    const unsigned linear = blockIdx.x + gridDim.x * blockIdx.y, slot = linear >> 3;
    by = static_cast<int>(slot / gridDim.x) * 8 + static_cast<int>(linear & 7);
    bx = static_cast<int>(slot % gridDim.x);
    if (by >= B) return;
  }
  const int b = B - 1 - by;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  const int m = min(max(keep[b], 0), n), r = n - m;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i0 = (bx * kMfmaWaves + wave) * kMfmaRowsPerWave;
  if (r <= 0 || i0 >= m || r > kTiledMinPruned) return;   // larger pruned sets: k_scores_tiled
  if (!plan_fits(plan_offsets[b], m, r, plan_cap)) return;
  const long long po = plan_offsets[b];
  const bool k_f32 = kernel_is_f32(p, m, r);
  const int32_t* sel = sel_idx + lo;
  const int frow = lane & 15, fk = (lane >> 4) * 16;   // 16 elements = 32 bytes per lane and step
  const double inv_eps = 1.0 / p.eps;

  const bf16_t* arow[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int i = min(i0 + 16 * t + frow, m - 1);
    arow[t] = tokens + static_cast<size_t>(lo + clamp_index(sel[i], n)) * D + fk;
  }

  for (int j0 = 0; j0 < r; j0 += 16 * NT) {
    const bf16_t* brow[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      const int j = min(j0 + 16 * u + frow, r - 1);
      brow[u] = tokens + static_cast<size_t>(lo + clamp_index(sel[m + j], n)) * D + fk;
    }
    double acc[MT][NT][4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int u = 0; u < NT; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[t][u][v] = 0.0;

    // 64 elements per step: a lane reads 32 contiguous bytes of its row (four
    // lanes cover one 128-byte line) and feeds them to two matrix instructions.
    // The next step's fragments are requested before the current step's
    // arithmetic.
    uint4 fa[MT][2], fb[NT][2];
    auto load_step = [&](int k0, uint4 (&a)[MT][2], uint4 (&bb)[NT][2]) {
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        a[t][0] = *reinterpret_cast<const uint4*>(arow[t] + k0);
        a[t][1] = *reinterpret_cast<const uint4*>(arow[t] + k0 + 8);
      }
#pragma unroll
      for (int u = 0; u < NT; ++u) {
        bb[u][0] = *reinterpret_cast<const uint4*>(brow[u] + k0);
        bb[u][1] = *reinterpret_cast<const uint4*>(brow[u] + k0 + 8);
      }
    };
    auto compute_step = [&](const uint4 (&a)[MT][2], const uint4 (&bb)[NT][2]) {
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
          for (int u = 0; u < NT; ++u) {
            const floatx4_t zero = {0.f, 0.f, 0.f, 0.f};
            const floatx4_t c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8_t, a[t][h]), __builtin_bit_cast(bf16x8_t, bb[u][h]), zero, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[t][u][v] += static_cast<double>(c[v]);
          }
    };
    // two fragment buffers used alternately, so that the loads of one are in
    // flight while the other is consumed (no register copies between steps)
    uint4 ga[MT][2], gb[NT][2];
    // Loads are unconditional (the step index is clamped instead) so that the
    // number of loads in flight is fixed and the waits can be counted ones.
    // D is a multiple of 128 here, so steps come in pairs and nothing in the
    // loop body is conditional.
    const int last = D - 64;
    load_step(0, fa, fb);
    for (int k0 = 0; k0 < D; k0 += 128) {
      load_step(k0 + 64, ga, gb);
      __builtin_amdgcn_sched_barrier(0);   // keep the loads ahead of the arithmetic
      compute_step(fa, fb);
      __builtin_amdgcn_sched_barrier(0);
      load_step(min(k0 + 128, last), fa, fb);
      __builtin_amdgcn_sched_barrier(0);
      compute_step(ga, gb);
      __builtin_amdgcn_sched_barrier(0);
    }

    // accumulator element v of lane l is (kept row 4 (l / 16) + v, pruned row l % 16) of its tile
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      const int j = j0 + 16 * u + (lane & 15);
      if (j >= r) continue;
      const double nj = norm64[lo + clamp_index(sel[m + j], n)];
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int i = i0 + 16 * t + 4 * (lane >> 4) + v;
          if (i < m) {
            const double ni = norm64[lo + clamp_index(sel[i], n)];
            const double s = acc[t][u][v] / fmax(ni * nj, kTinyNorm * kTinyNorm);
            const long long at = static_cast<long long>(i) * r + j;
            store_kernel(kmat, po, i, j, r, exp((s - p.shift) * inv_eps), k_f32);
            if (scores_out) scores_out[po + at] = s;
          }
        }
    }
  }
}

}  // namespace rtp
