// Cosine scores of Eq. 3 for images with many pruned tokens (R > kTiledMinPruned:
// other OCR models' pages, aggressive ratios), where S = T_kept T_prop^T is a
// real GEMM: a workgroup computes a 128 x 64 tile of S, staging 64 elements of
// the contraction per step of both operands in LDS (double-buffered) so that
// every token row is fetched once per tile instead of once per 16-row sub-tile.
//
// Accuracy: the same v_mfma_f32_16x16x32_bf16 as k_scores_mfma, but the two of a
// step (64 terms of the contraction) are chained on one fp32 accumulator before
// the partial is added to the fp64 sum, which halves the fp64 vector work per
// matrix instruction.  Measured against the fp64 oracle on 1083- to 4512-token
// pages the cosine is off by at most 4.2e-8 (k_scores_mfma: 2e-8) and plan
// entries by at most 7.7e-7 relative - still inside the 1e-6 band in which an
// index flip counts as a near-tie; chaining four (128 terms) gave 8e-8 and was
// rejected.  Both kernels write the same quantities; an image goes to exactly
// one of them.
//
// Workgroup = 4 waves as 2 x 2, a wave owns 64 x 32 = 4 x 2 matrix tiles; two
// workgroups share a CU, so one's arithmetic hides the other's loads.  LDS
// rows are 128 bytes without padding; the 16-byte pieces of a row are permuted
// by the row's number so that the 16 lanes of a fragment read fall into
// distinct banks.
#pragma once
#include "common.hpp"
#include "scores_mfma.hpp"
#include "sinkhorn_team.hpp"

namespace rtp {

constexpr int kTileRows = 128;         // kept rows per workgroup tile
constexpr int kTileCols = 64;          // pruned rows per workgroup tile
constexpr int kTileStep = 64;          // contraction elements per step (128 bytes per row)
constexpr int kTilePitch = 128;        // LDS bytes per staged row: eight 16-byte slots, no padding
constexpr int kTiledThreads = 256;

__host__ __device__ inline bool score_is_tiled(int r) { return r > kTiledMinPruned; }

// What both launch forms of the kernel pass on.
struct ScoresTiledArgs {
  const bf16_t* tokens;
  const int32_t* offsets;
  int D;
  const int32_t* sel_idx;
  const int32_t* keep;
  const long long* plan_offsets;
  const double* norm64;
  DevParams p;
  double* kmat;
  long long plan_cap;
  double* scores_out;
  int tiles_n;
};

// Tile `tile` (kept-row tile major) of image b.
__device__ __forceinline__ void scores_tile(const ScoresTiledArgs& A, int b, int tile) {
  const bf16_t* __restrict__ tokens = A.tokens;
  const int32_t* __restrict__ offsets = A.offsets;
  const int D = A.D;
  const int32_t* __restrict__ sel_idx = A.sel_idx;
  const long long* __restrict__ plan_offsets = A.plan_offsets;
  const double* __restrict__ norm64 = A.norm64;
  const DevParams& p = A.p;
  double* __restrict__ kmat = A.kmat;
  double* __restrict__ scores_out = A.scores_out;
  const long long plan_cap = A.plan_cap;
  const int tiles_n = A.tiles_n;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  const int m = min(max(A.keep[b], 0), n), r = n - m;
  if (!score_is_tiled(r)) return;
  const int tm = tile / tiles_n, tn = tile - tm * tiles_n;
  const int i0 = tm * kTileRows, j0 = tn * kTileCols;
  if (i0 >= m || j0 >= r) return;
  if (!plan_fits(plan_offsets[b], m, r, plan_cap)) return;
  const long long po = plan_offsets[b];
  const bool k_f32 = kernel_is_f32(p, m, r);
  // the sweep kernels' images take exp through the fp32 unit; the on-chip shapes' entries are
  // the fp64 exp rounded once, as those kernels themselves used to round them on load
  const bool fast_exp = k_f32 && sinkhorn_variant(m, r, p.mode) == kVariantSweep;
  const int32_t* sel = sel_idx + lo;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;          // the wave's 64 x 32 part of the tile
  const double inv_eps = 1.0 / p.eps;

  // [buffer][kept rows, pruned rows]; piece c (16 bytes) of row i sits in slot c ^ (i / 2 % 8), so
  // that the 16 rows of a fragment read fall into different banks without padding
  constexpr int kBufBytes = (kTileRows + kTileCols) * kTilePitch;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kBufBytes];
  unsigned char* const lds_a = lds;
  unsigned char* const lds_b = lds + kTileRows * kTilePitch;
  __shared__ double rnorm[kTileRows + kTileCols];    // reciprocal norms of the tile's rows and columns

  // staging: thread t moves piece t % 8 (16 bytes) of rows t / 8 + 32 q of each operand
  constexpr int QA = kTileRows / 32, QB = kTileCols / 32;
  static_assert(QA == 4 && QB == 2, "the staging below is written out for these counts");
  const int piece = tid & 7, srow = tid >> 3;
  const bf16_t* aptr[QA];
  const bf16_t* bptr[QB];
#pragma unroll
  for (int q = 0; q < QA; ++q) {
    const int i = min(i0 + srow + 32 * q, m - 1);
    aptr[q] = tokens + static_cast<size_t>(lo + clamp_index(sel[i], n)) * D + 8 * piece;
  }
#pragma unroll
  for (int q = 0; q < QB; ++q) {
    const int j = min(j0 + srow + 32 * q, r - 1);
    bptr[q] = tokens + static_cast<size_t>(lo + clamp_index(sel[m + j], n)) * D + 8 * piece;
  }
  // the reciprocal norms the last part needs, fetched now (two dependent loads) instead of
  // when every wave waits for them
  if (tid < kTileRows + kTileCols) {
    const int at = tid < kTileRows ? min(i0 + tid, m - 1) : m + min(j0 + tid - kTileRows, r - 1);
    rnorm[tid] = 1.0 / fmax(norm64[lo + clamp_index(sel[at], n)], kTinyNorm);
  }

  // Rows are requested two steps before their arithmetic (a step is shorter than a trip to
  // memory that misses the L2) into one of two sets of registers, and go to the LDS buffer
  // that the previous step has finished with.  Named registers, not arrays or structs: an
  // array that lives across the step loop can end up in LDS, with a wait for the rows
  // right behind their request.
  const int steps = D / kTileStep;                   // even: D is a multiple of 128 on this path
  uint4 xa0, xa1, xa2, xa3, xb0, xb1, ya0, ya1, ya2, ya3, yb0, yb1;
  const int stage_off = srow * kTilePitch + 16 * (piece ^ ((srow >> 1) & 7));   // rows + 32 q: the same slot
#define RTP_TILED_FETCH(w, k0)                                 \
  do {                                                         \
    w##a0 = *reinterpret_cast<const uint4*>(aptr[0] + (k0));   \
    w##a1 = *reinterpret_cast<const uint4*>(aptr[1] + (k0));   \
    w##a2 = *reinterpret_cast<const uint4*>(aptr[2] + (k0));   \
    w##a3 = *reinterpret_cast<const uint4*>(aptr[3] + (k0));   \
    w##b0 = *reinterpret_cast<const uint4*>(bptr[0] + (k0));   \
    w##b1 = *reinterpret_cast<const uint4*>(bptr[1] + (k0));   \
  } while (0)
#define RTP_TILED_STAGE(buf, w)                                                 \
  do {                                                                          \
    unsigned char* sa_ = lds_a + (buf) * kBufBytes + stage_off;                 \
    unsigned char* sb_ = lds_b + (buf) * kBufBytes + stage_off;                 \
    *reinterpret_cast<uint4*>(sa_) = w##a0;                                     \
    *reinterpret_cast<uint4*>(sa_ + 32 * kTilePitch) = w##a1;                   \
    *reinterpret_cast<uint4*>(sa_ + 64 * kTilePitch) = w##a2;                   \
    *reinterpret_cast<uint4*>(sa_ + 96 * kTilePitch) = w##a3;                   \
    *reinterpret_cast<uint4*>(sb_) = w##b0;                                     \
    *reinterpret_cast<uint4*>(sb_ + 32 * kTilePitch) = w##b1;                   \
  } while (0)

  // fp64 sums of the flushed partials, and two sets of fp32 accumulators for the matrix
  // instructions: while a step's instructions fill one set, the previous step's partials
  // leave the other for the fp64 sums, so that the vector unit's conversions and additions
  // run under the matrix unit's work instead of after it
  double acc[4][2][4];
  floatx4_t part0[4][2], part1[4][2];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      part0[t][u] = floatx4_t{0.f, 0.f, 0.f, 0.f};
      part1[t][u] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[t][u][v] = 0.0;
    }

  // fragment of a 16-row tile for half h of the step: lane l reads the 16 bytes
  // at row l % 16, elements 16 (l / 16) + 8 h .. + 7 of the step - the same
  // assignment of contraction elements to lanes for both operands
  const int frag_row = (lane & 15) * kTilePitch, frag_slot = (2 * (lane >> 4)) ^ ((lane & 15) >> 1);
  const int frag_off[2] = {frag_row + 16 * frag_slot, frag_row + 16 * (frag_slot ^ 1)};   // halves 0 and 1
  const unsigned char* frag_a = lds_a + wm * 64 * kTilePitch;
  const unsigned char* frag_b = lds_b + wn * 32 * kTilePitch;
  // one step: the two matrix instructions per 16 x 16 tile of the wave, the first on a zero
  // accumulator, into `now`; and `before`, the previous step's partials, added to the sums
  auto step = [&](int buf, floatx4_t (&now)[4][2], const floatx4_t (&before)[4][2]) {
    const unsigned char* A = frag_a + buf * kBufBytes;
    const unsigned char* B = frag_b + buf * kBufBytes;
    const floatx4_t zero{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint4 fa[4], fb[2];
#pragma unroll
      for (int t = 0; t < 4; ++t) fa[t] = *reinterpret_cast<const uint4*>(A + 16 * t * kTilePitch + frag_off[h]);
#pragma unroll
      for (int u = 0; u < 2; ++u) fb[u] = *reinterpret_cast<const uint4*>(B + 16 * u * kTilePitch + frag_off[h]);
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u)
          now[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              __builtin_bit_cast(bf16x8_t, fa[t]), __builtin_bit_cast(bf16x8_t, fb[u]),
              h == 0 ? zero : now[t][u], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[t][u][v] += static_cast<double>(before[t][u][v]);
  };

  // The last steps ask for the last step's rows again, so that the requests and the staging
  // are the same instructions in every step; the barriers for the instruction scheduler
  // keep the requests ahead of the arithmetic and the staging behind it.
  RTP_TILED_FETCH(x, 0);
  RTP_TILED_STAGE(0, x);
  RTP_TILED_FETCH(x, kTileStep);                      // step 1's
  __syncthreads();
  for (int s = 0; s < steps; s += 2) {                // steps is even
    RTP_TILED_FETCH(y, min(s + 2, steps - 1) * kTileStep);
    __builtin_amdgcn_sched_barrier(0);
    step(0, part0, part1);
    __builtin_amdgcn_sched_barrier(0);
    RTP_TILED_STAGE(1, x);
    __syncthreads();
    RTP_TILED_FETCH(x, min(s + 3, steps - 1) * kTileStep);
    __builtin_amdgcn_sched_barrier(0);
    step(1, part1, part0);
    __builtin_amdgcn_sched_barrier(0);
    RTP_TILED_STAGE(0, y);
    __syncthreads();
  }
#undef RTP_TILED_FETCH
#undef RTP_TILED_STAGE
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[t][u][v] += static_cast<double>(part1[t][u][v]);

  // accumulator element v of lane l is (kept row 4 (l / 16) + v, pruned row l % 16) of its tile.
  // exp through the fp32 unit when K is stored in fp32 for the sweep kernels: with
  // y = x log2(e) = k + f, |f| <= 1/2 split in fp64, exp(x) = 2^k 2^f and v_exp_f32 gives
  // 2^f to about 1e-7 relative, which on the score is eps * 1e-7.
  const int il0 = 64 * wm + 4 * (lane >> 4), jl0 = 32 * wn + (lane & 15);
  auto kernel_f32 = [&](double x) -> float {
    if (!fast_exp) return static_cast<float>(exp_nonpositive(x));
    const double y = x * 1.4426950408889634;
    const double k = rint(y);
    return ldexpf(__builtin_amdgcn_exp2f(static_cast<float>(y - k)), static_cast<int>(k));
  };
  if (k_f32 && !scores_out) {
    // the tile's entries go through LDS (the staging buffers are free: every wave is past
    // the loop's last barrier), so that they leave as whole 16-byte pieces of rows
    constexpr int kOutPitch = kTileCols + 4;         // floats
    static_assert(kTileRows * kOutPitch * 4 <= 2 * kBufBytes, "the output tile fits the staging buffers");
    float* tile = reinterpret_cast<float*>(lds);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int jl = jl0 + 16 * u;
      const double rnj = rnorm[kTileRows + jl];
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int il = il0 + 16 * t + v;
          float kv = 0.f;
          if (i0 + il < m && j0 + jl < r) {
            kv = kernel_f32((acc[t][u][v] * rnorm[il] * rnj - p.shift) * inv_eps);
          }
          tile[il * kOutPitch + jl] = kv;
        }
    }
    __syncthreads();
    float* kout = k32_base(kmat, po);
    const int pitch = k32_pitch(r);                  // a multiple of 4: r > kTiledMinPruned
    const int c4 = 4 * (tid & 15);
#pragma unroll
    for (int q = 0; q < kTileRows / 16; ++q) {
      const int il = (tid >> 4) + 16 * q;
      if (i0 + il < m && j0 + c4 < pitch)
        *reinterpret_cast<float4*>(kout + static_cast<long long>(i0 + il) * pitch + j0 + c4) =
            *reinterpret_cast<const float4*>(tile + il * kOutPitch + c4);
    }
    return;
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int jl = jl0 + 16 * u, j = j0 + jl;
    if (j >= r) continue;
    const double rnj = rnorm[kTileRows + jl];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int il = il0 + 16 * t + v, i = i0 + il;
        if (i < m) {
          const double sc = acc[t][u][v] * rnorm[il] * rnj;
          const long long at = static_cast<long long>(i) * r + j;
          const double x = (sc - p.shift) * inv_eps;
          if (k_f32) k32_base(kmat, po)[static_cast<long long>(i) * k32_pitch(r) + j] = kernel_f32(x);
          else kmat[po + at] = exp_nonpositive(x);
          if (scores_out) scores_out[po + at] = sc;
        }
      }
  }
}

// One workgroup per (tile, image): for calls whose images are known to be large
// (the hardware hands out workgroups as CUs come free, which balances best).
__global__ __launch_bounds__(kTiledThreads, 2) void k_scores_tiled(ScoresTiledArgs A, const int32_t* __restrict__ status) {
  if (status[0]) return;
  scores_tile(A, blockIdx.y, blockIdx.x);
}

// A fixed number of workgroups that walk the tiles of the images on the tiled
// work list: for calls that may well have no such image (kept counts decided on
// the device), where a grid sized for the worst case would cost more to launch
// empty than the rest of the call's small kernels together.
__global__ __launch_bounds__(kTiledThreads, 2) void k_scores_tiled_list(ScoresTiledArgs A, int tiles,
                                                                    const int32_t* __restrict__ work, int B,
                                                                    const int32_t* __restrict__ status) {
  if (status[0]) return;
  const int count = work[kListTiled];
  const long long items = static_cast<long long>(count) * tiles;
  for (long long item = blockIdx.x; item < items; item += gridDim.x) {
    __syncthreads();   // the previous tile's last LDS reads
    const int k = static_cast<int>(item / tiles);
    scores_tile(A, work[kWorkLists + kListTiled * B + k], static_cast<int>(item - static_cast<long long>(k) * tiles));
  }
}

}  // namespace rtp
