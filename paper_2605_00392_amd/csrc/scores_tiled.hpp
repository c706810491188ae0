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
constexpr int kTileCols = 64;          // pruned rows per workgroup tile (128, eight waves: the same time)
constexpr int kTileStep = 64;          // contraction elements per step (128 bytes per row)
constexpr int kTilePitch = 128;        // LDS bytes per staged row: eight 16-byte slots, no padding
constexpr int kTiledWavesN = kTileCols / 32;                   // waves side by side on the pruned rows
constexpr int kTiledThreads = 64 * 2 * kTiledWavesN;          // 2 x kTiledWavesN waves of 64 x 32

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

// Sixteen bytes per lane from memory straight into LDS: lane l's land at LDS byte address
// `lds_base` + 16 l (`lds_base` the same in all lanes).  Written as assembly because the
// compiler, for the builtin of the same instruction, makes LDS reads wait for every such load
// in flight when it cannot tell their buffers apart, which would undo requesting rows two
// steps ahead; the caller waits for them itself (they count in vmcnt, and are done when
// their data is in LDS).  M0 holds the LDS base for the instruction and is put back.
__device__ __forceinline__ void load_to_lds_16(const void* src, uint32_t lds_base) {
  uint32_t m0_before;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, off\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(m0_before)
      : "v"(src), "s"(lds_base)
      : "memory");
}

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
  const int wm = wave / kTiledWavesN, wn = wave % kTiledWavesN;   // the wave's 64 x 32 part of the tile
  const double inv_eps = 1.0 / p.eps;

  // Three staging buffers, [kept rows, pruned rows] each, separate arrays so that the compiler
  // can tell a buffer that loads are writing from the one being read.  Piece c (16 bytes) of
  // row i sits in slot c ^ (i / 2 % 8), so that the 16 rows of a fragment read fall into
  // different banks without padding.
  constexpr int kBufBytes = (kTileRows + kTileCols) * kTilePitch;
  constexpr int kBufB = kTileRows * kTilePitch;      // where a buffer's pruned rows start
  __shared__ __attribute__((aligned(16))) unsigned char lds[3 * kBufBytes];
  unsigned char* const lds0 = lds;
  unsigned char* const lds1 = lds + kBufBytes;
  unsigned char* const lds2 = lds + 2 * kBufBytes;
  __shared__ double rnorm[kTileRows + kTileCols];    // reciprocal norms of the tile's rows and columns

  // Staging: the rows go from memory straight into LDS (global_load_lds_dwordx4: lane l's 16
  // bytes land at the wave's LDS base + 16 l, so a wave's request fills eight rows): thread t
  // fills slot t % 8 of rows t / 8 + 32 q of each operand, i.e. fetches piece
  // (t % 8) ^ (row / 2 % 8) of that row.
  constexpr int kPass = kTiledThreads / 8;           // rows the workgroup's requests fill at a time
  constexpr int QA = kTileRows / kPass, QB = kTileCols / kPass;
  const int srow = tid >> 3, piece = (tid & 7) ^ ((srow >> 1) & 7);   // rows + kPass q: the same piece
  const bf16_t* aptr[QA];
  const bf16_t* bptr[QB];
#pragma unroll
  for (int q = 0; q < QA; ++q) {
    const int i = min(i0 + srow + kPass * q, m - 1);
    aptr[q] = tokens + static_cast<size_t>(lo + clamp_index(sel[i], n)) * D + 8 * piece;
  }
#pragma unroll
  for (int q = 0; q < QB; ++q) {
    const int j = min(j0 + srow + kPass * q, r - 1);
    bptr[q] = tokens + static_cast<size_t>(lo + clamp_index(sel[m + j], n)) * D + 8 * piece;
  }
  // the reciprocal norms the last part needs, fetched now (two dependent loads) instead of
  // when every wave waits for them
  if (tid < kTileRows + kTileCols) {
    const int at = tid < kTileRows ? min(i0 + tid, m - 1) : m + min(j0 + tid - kTileRows, r - 1);
    rnorm[tid] = 1.0 / fmax(norm64[lo + clamp_index(sel[at], n)], kTinyNorm);
  }

  // Rows are requested two steps before their arithmetic (a step is shorter than a trip to
  // memory that misses the L2), into the buffer that the previous step has finished with.
  const int steps = D / kTileStep;                   // even: D is a multiple of 128 on this path
  // LDS byte addresses of the eight rows this wave's requests fill (+ 32 q rows), per buffer
  typedef __attribute__((address_space(3))) unsigned char* lds_ptr_t;
  const uint32_t wave_rows = 8 * wave * kTilePitch;
  const uint32_t base0 = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)lds0)) + wave_rows);
  const uint32_t base1 = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)lds1)) + wave_rows);
  const uint32_t base2 = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)lds2)) + wave_rows);
#define RTP_TILED_REQUEST(base, k0)                                                            \
  do {                                                                                         \
    _Pragma("unroll") for (int q = 0; q < QA; ++q)                                             \
      load_to_lds_16(aptr[q] + (k0), (base) + kPass * q * kTilePitch);                         \
    _Pragma("unroll") for (int q = 0; q < QB; ++q)                                             \
      load_to_lds_16(bptr[q] + (k0), (base) + kBufB + kPass * q * kTilePitch);                    \
  } while (0)
  // Before the workgroup meets, a wave's requests but the latest QA + QB (one step's) have
  // landed in LDS (vmcnt counts a request done when its data is written) and its LDS reads
  // are over.  The wait is written out: a workgroup-scope fence would wait for every request,
  // the latest too.  The wavefront-scope fences emit nothing; they keep the compiler from
  // moving LDS accesses across the meeting.
#define RTP_TILED_MEET(newest)                                                           \
  do {                                                                                   \
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");                               \
    if (newest) __builtin_amdgcn_s_waitcnt(0x0070 | (QA + QB)); /* vmcnt(one step's requests) lgkmcnt(0) */ \
    else __builtin_amdgcn_s_waitcnt(0x0070);        /* vmcnt(0) lgkmcnt(0) */            \
    __builtin_amdgcn_s_barrier();                                                        \
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");                               \
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
  const int frag_a = wm * 64 * kTilePitch, frag_b = kBufB + wn * 32 * kTilePitch;
  // one step: the two matrix instructions per 16 x 16 tile of the wave, the first on a zero
  // accumulator, into `now`; and `before`, the previous step's partials, added to the sums
  auto step = [&](const unsigned char* buf, floatx4_t (&now)[4][2], const floatx4_t (&before)[4][2]) {
    const unsigned char* A = buf + frag_a;
    const unsigned char* B = buf + frag_b;
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

  // Step s reads buffer s % 3 and accumulates in set s % 2, so the loop is written out for six
  // steps; the last steps ask for the last step's rows again, so that every step issues the
  // same requests.  The barriers for the instruction scheduler keep the requests ahead of
  // the arithmetic.
#define RTP_TILED_STEP(i, rd, wr, now, before)                             \
  if (s + (i) < steps) {                                                   \
    RTP_TILED_REQUEST(wr, min(s + (i) + 2, steps - 1) * kTileStep);        \
    __builtin_amdgcn_sched_barrier(0);                                     \
    step(rd, now, before);                                                 \
    __builtin_amdgcn_sched_barrier(0);                                     \
    RTP_TILED_MEET(true);                                                  \
  }
  RTP_TILED_REQUEST(base0, 0);
  RTP_TILED_REQUEST(base1, kTileStep);
  RTP_TILED_MEET(true);
  for (int s = 0; s < steps; s += 6) {
    RTP_TILED_STEP(0, lds0, base2, part0, part1)
    RTP_TILED_STEP(1, lds1, base0, part1, part0)
    RTP_TILED_STEP(2, lds2, base1, part0, part1)
    RTP_TILED_STEP(3, lds0, base2, part1, part0)
    RTP_TILED_STEP(4, lds1, base0, part0, part1)
    RTP_TILED_STEP(5, lds2, base1, part1, part0)
  }
  RTP_TILED_MEET(false);                              // every request has landed: the buffers are free
#undef RTP_TILED_STEP
#undef RTP_TILED_REQUEST
#undef RTP_TILED_MEET
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
    static_assert(kTileRows * kOutPitch * 4 <= 3 * kBufBytes, "the output tile fits the staging buffers");
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
          if (i0 + il < m && j0 + jl < r)
            kv = kernel_f32((acc[t][u][v] * rnorm[il] * rnj - p.shift) * inv_eps);
          tile[il * kOutPitch + jl] = kv;
        }
    }
    __syncthreads();
    float* kout = k32_base(kmat, po);
    const int pitch = k32_pitch(r);                  // a multiple of 4: r > kTiledMinPruned
    constexpr int kRowLanes = kTileCols / 4;         // lanes that cover a row of the tile, 16 bytes each
    constexpr int kRowsAtOnce = kTiledThreads / kRowLanes;
    const int c4 = 4 * (tid % kRowLanes);
#pragma unroll
    for (int q = 0; q < kTileRows / kRowsAtOnce; ++q) {
      const int il = tid / kRowLanes + kRowsAtOnce * q;
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
