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
// The matrix instruction wants lane l to hold eight elements of row (l % 16),
// and 16 neighbouring lanes that read 16 different rows cost the texture-address
// unit one cache line per cycle (measured on L2-resident rows: 65 cycles per
// 16-byte-per-lane load against 18 when eight neighbouring lanes read one
// 128-byte line).  So rows are read in the second order and reach the operand
// order through LDS (rows 144 bytes apart: writes and reads are free of bank
// conflicts), and the four waves of a workgroup share the pruned rows: a
// workgroup takes 128 kept rows (32 per wave) against all, at most 64, pruned
// rows, 64 elements of the contraction per step, the next step's rows in flight
// while the current one is multiplied.  Column tiles of 16 pruned rows that an
// image does not have are skipped.  (A kernel that read its operands straight
// into the operand order, one wave per workgroup, came before this one: equal on
// 1024 pages with 7 pruned tokens each, where the pass is bound by HBM reads at
// 4.4 TB/s; 12 % slower on ragged pages with a few dozen, 20 % slower at 63.)
#pragma once
#include "common.hpp"
#include "stage1.hpp"
#include "sinkhorn_team.hpp"
#include "sinkhorn_dual.hpp"

namespace rtp {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kMfmaMinWidth = 1024;   // token widths below this take the fp64 vector score kernel

constexpr int kScoreThreads = 256;
constexpr int kScoreRows = 128;                      // kept rows per workgroup
constexpr int kScorePitch = 72;                      // bf16 per LDS row: 64 elements and 16 bytes
constexpr int kScoreBufElems = (64 + kScoreRows) * kScorePitch;

// What the fused calls ask of one extra workgroup of this launch: the batch-wide
// prefix sum of the kept counts (where the merge writes each image), the Sinkhorn work
// lists, and the per-image slots of the kernel matrix and the plan, as an array for the
// kernels after this one.  Nothing in this launch depends on it: with a job, an image's
// slot is the closed form plan_slot(offsets, b, stride), which this kernel evaluates for
// itself.  It takes a launch of its own (k_scan_classify) out of every fused call.
struct ScanJob {
  int on;
  int32_t* out_offsets;        // may be null
  long long* plan_offsets;
  int32_t* work;
  int mode;
  long long stride;
};

// Launched over tiles x rows8 workgroups (rows8 = B rounded up to a multiple of eight),
// plus one when `job.on`.
__global__ __launch_bounds__(kScoreThreads) void k_scores_mfma(
    const bf16_t* __restrict__ tokens, const int32_t* __restrict__ offsets, int B, int D,
    const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ keep,
    const long long* __restrict__ plan_offsets, const double* __restrict__ norm64, DevParams p,
    double* __restrict__ kmat, long long plan_cap, double* __restrict__ scores_out, int tiles, ScanJob job,
    const int32_t* __restrict__ status) {
  if (status[0]) return;
  __shared__ __align__(16) bf16_t stage[kScoreBufElems];
  const unsigned linear = blockIdx.x;
  if (job.on && linear == gridDim.x - 1) {
    static_assert(kClassifyLdsBytes <= sizeof(stage) && kScanLdsBytes <= sizeof(stage), "the job works in the stage buffer");
    static_assert(kScoreThreads == 256, "scan_images and classify_images are written for workgroups of 256 threads");
    scan_images(offsets, keep, B, job.out_offsets, job.plan_offsets, stage, job.stride);
    __syncthreads();
    classify_images(offsets, keep, B, job.work, job.mode, stage);
    return;
  }
  // Images are taken last to first: the norm pass before this one walks them first
  // to last and the merge after it does so again, so each pass starts on the
  // images its predecessor touched last, which are the ones the memory-side cache
  // still holds (measured on 1 GB batches: 2 % off this kernel, 1 % off the merge).
  // An image's workgroups get linear ids of one residue modulo eight: workgroups
  // are dealt to the eight XCDs in turn, so the image's pruned rows, which all its
  // workgroups read, are fetched into one L2 instead of eight (1024 pages with 63
  // pruned tokens each: 2.4 GB fetched from memory without this, against 1.05 GB of
  // tokens).  The launch covers B rounded up to a multiple of eight for it.
  const unsigned slot = linear >> 3;
  const int by = static_cast<int>(slot / tiles) * 8 + static_cast<int>(linear & 7);
  const int bx = static_cast<int>(slot % tiles);
  if (by >= B) return;
  const int b = B - 1 - by;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  const int m = min(max(keep[b], 0), n), r = n - m;
  const int i0 = bx * kScoreRows;
  if (r <= 0 || i0 >= m || r > kTiledMinPruned) return;   // (the same for the whole workgroup)
  const long long po = job.on ? plan_slot(offsets, b, job.stride) : plan_offsets[b];
  if (!plan_fits(po, m, r, plan_cap)) return;
  const int k_layout = kernel_layout(p, m, r);
  const int32_t* sel = sel_idx + lo;
  const double inv_eps = 1.0 / p.eps;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int iw = i0 + 32 * wave;                       // the wave's first kept row
  const bool active = iw < m;                          // the wave has kept rows
  const int ntiles = (r + 15) >> 4;                    // column tiles of 16 pruned rows that exist
  // Wave w brings in the pruned rows of column tile w.  A wave with neither kept rows nor a
  // column tile ends here (it no longer counts at the barriers): a workgroup's step costs a
  // memory latency whatever its size, so the 16 kept rows that a 400-token page leaves for
  // its fourth workgroup should hold one wave's registers, not four waves'.
  const bool feeds = wave < ntiles;
  if (!active && !feeds) return;
  constexpr int kPitch = kScorePitch;
  // 1 / max(norm, tiny) of the workgroup's rows, for the end: pruned rows 0 .. 63, then the 128
  // kept rows.  Fetched now by the first wave (which always stays), so that the two dependent
  // loads behind each value are not waited for after the last step.
  __shared__ double rnorm[64 + kScoreRows];
  if (wave == 0) {
#pragma unroll
    for (int q = 0; q < (64 + kScoreRows) / 64; ++q) {
      const int e = lane + 64 * q;
      const int pos = e < 64 ? m + min(e, r - 1) : min(i0 + e - 64, m - 1);
      rnorm[e] = 1.0 / fmax(norm64[lo + clamp_index(sel[pos], n)], kTinyNorm);
    }
  }

  // reading: eight lanes per row.  Pruned rows 16 w + l / 8 + 8 q (q = 0, 1) by wave w when
  // that column tile exists; kept rows l / 8 + 8 q (q = 0 .. 3) of the wave's 32 by each wave.
  const char* base = reinterpret_cast<const char*>(tokens + static_cast<size_t>(lo) * D);
  const int chunk = tid & 7;
  uint32_t poff[2], koff[4];                           // byte offsets within the image (at most 8192 rows of 8 KB)
#pragma unroll
  for (int q = 0; q < 2; ++q)
    poff[q] = static_cast<uint32_t>(clamp_index(sel[m + min(16 * wave + (lane >> 3) + 8 * q, r - 1)], n) * D + 8 * chunk) * 2u;
#pragma unroll
  for (int q = 0; q < 4; ++q)
    koff[q] = static_cast<uint32_t>(clamp_index(sel[min(iw + (lane >> 3) + 8 * q, m - 1)], n) * D + 8 * chunk) * 2u;
  // LDS rows 0 .. 63: pruned; 64 + 32 wave ..: the wave's kept rows
  const int wr_p = (16 * wave + (lane >> 3)) * kPitch + 8 * chunk;          // + 8 q rows
  const int wr_k = (64 + 32 * wave + (lane >> 3)) * kPitch + 8 * chunk;    // + 8 q rows
  // (instruction h of a step contracts elements 16 g + 8 h .. + 7, g = 0 .. 3; which 32
  // of the 64 is immaterial as long as both operands use the same assignment)
  const int rd = (lane & 15) * kPitch + 16 * (lane >> 4);                  // + tile's first row, + 8 h elements

  double acc[2][4][4];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[t][u][v] = 0.0;

  u32x4_t gp[2] = {}, gk[4] = {};
  auto load_step = [&](int k0, u32x4_t (&gp)[2], u32x4_t (&gk)[4]) {
    if (feeds) {
#pragma unroll
      for (int q = 0; q < 2; ++q) gp[q] = *reinterpret_cast<const u32x4_t*>(base + poff[q] + 2 * k0);
    }
    if (active) {
#pragma unroll
      for (int q = 0; q < 4; ++q) gk[q] = *reinterpret_cast<const u32x4_t*>(base + koff[q] + 2 * k0);
    }
  };
  auto stage_step = [&](bf16_t* buf, const u32x4_t (&gp)[2], const u32x4_t (&gk)[4]) {
    if (feeds) {
#pragma unroll
      for (int q = 0; q < 2; ++q) *reinterpret_cast<u32x4_t*>(buf + wr_p + 8 * q * kPitch) = gp[q];
    }
    if (active) {
#pragma unroll
      for (int q = 0; q < 4; ++q) *reinterpret_cast<u32x4_t*>(buf + wr_k + 8 * q * kPitch) = gk[q];
    }
  };
  const int last = D - 64;
  load_step(0, gp, gk);
  stage_step(stage, gp, gk);
  for (int k0 = 0; k0 < D; k0 += 64) {
    load_step(min(k0 + 64, last), gp, gk);             // unconditional: the step index is clamped instead
    __syncthreads();                                   // this step's rows are in LDS
    const bf16_t* cur = stage + rd;
    if (active) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        bf16x8_t a[2], bb[4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
          a[t] = *reinterpret_cast<const bf16x8_t*>(cur + (64 + 32 * wave + 16 * t) * kPitch + 8 * h);
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (u < ntiles) bb[u] = *reinterpret_cast<const bf16x8_t*>(cur + 16 * u * kPitch + 8 * h);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (u < ntiles) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
              const floatx4_t zero = {0.f, 0.f, 0.f, 0.f};
              const floatx4_t c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t], bb[u], zero, 0, 0, 0);
#pragma unroll
              for (int v = 0; v < 4; ++v) acc[t][u][v] += static_cast<double>(c[v]);
            }
          }
        }
      }
    }
    __syncthreads();                                   // and have been read by every wave
    stage_step(stage, gp, gk);
  }
  if (!active) return;

  // accumulator element v of lane l is (kept row 4 (l / 16) + v, pruned row l % 16) of its tile
  // (rnorm was written before the first of the loop's barriers)
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    if (u >= ntiles) break;
    const int j = 16 * u + (lane & 15);
    const double rnj = rnorm[j];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int il = 32 * wave + 16 * t + 4 * (lane >> 4) + v, i = i0 + il;
        const double sc = acc[t][u][v] * rnorm[64 + il] * rnj;
        const double kv = exp_nonpositive((sc - p.shift) * inv_eps);
        if (i < m && j < r) {
          store_kernel(kmat, po, i, j, m, r, kv, k_layout);
          if (scores_out) scores_out[po + static_cast<long long>(i) * r + j] = sc;
        }
      }
  }
}

}  // namespace rtp
