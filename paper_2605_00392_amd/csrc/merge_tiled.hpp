// Merge and compaction (Eq. 6) for images with many pruned tokens
// (R > kTiledMinPruned), where out = T_kept + alpha P T_prop is a real GEMM
// (M x R times R x D) and belongs on the matrix cores.
//
// The plan is fp32 and must not lose precision to bf16 (one rounding would put
// 2e-3 alpha |T| on every merged feature), so every entry is split on the fly
// into two bf16 numbers, P = hi + lo with |P - hi - lo| <= 2^-18 |P|, and each
// product is two v_mfma_f32_16x16x32_bf16, accumulated in fp32 like the vector
// kernel's sum.  The pruned token rows are bf16 already; the matrix instruction
// wants eight consecutive pruned rows of one feature per lane, so their tile is
// transposed on its way into LDS.
//
// Workgroup = 4 waves as 2 x 2 on a tile of 128 kept rows x 128 features, 32
// pruned rows per step, LDS double-buffered; a wave owns 64 x 64 = 4 x 4 matrix
// tiles.  P's LDS rows are 64 bytes of payload on a pitch of 80.  A feature row of
// the turned pruned rows has its four 16-byte pieces (eight pruned rows each) in
// four of eight slots, slot = piece ^ (feature / 16 % 8), on a pitch of 144: the
// 64 lanes of a turning 4-byte write (16 groups of eight features x 4 pairs of
// pruned rows) then fall into 64 different banks (with the pieces in place they
// fell into 8), and the fragment reads stay conflict-free.  The finished tile
// goes through LDS once more so that the kept rows are read and the merged rows
// written 16 bytes per lane.
#pragma once
#include "common.hpp"
#include "scores_mfma.hpp"
#include "sinkhorn_team.hpp"

namespace rtp {

constexpr int kMergeTileRows = 128;    // kept rows per workgroup tile
constexpr int kMergeTileCols = 128;    // features per workgroup tile
constexpr int kMergeTileStep = 32;     // pruned rows per step
constexpr int kMergeTilePitch = 80;    // LDS bytes per staged row of P (32 bf16 + padding)
constexpr int kMergeTurnedPitch = 144; // LDS bytes per feature row of the turned pruned rows: eight 16-byte slots + padding
constexpr int kMergeTiledThreads = 256;
constexpr int kMergeTiledLdsBytes = 2 * 128 * (2 * kMergeTilePitch + kMergeTurnedPitch);   // merge_tile's LDS buffer (its staging tiles; the output tile fits too)
constexpr int kMergeOutPitch = kMergeTileCols + 4;   // floats per row of the output staging tile

// What both launch forms of the kernel pass on.
struct MergeTiledArgs {
  const bf16_t* tokens;
  const int32_t* offsets;
  int D;
  const int32_t* sel_idx;
  const int32_t* keep;
  const int32_t* out_offsets;
  const float* plan;
  const long long* plan_offsets;
  float alpha;
  int max_tokens, tiles_d;
  bf16_t* out;
};

// Tile `tile` (kept-row tile major, feature tile minor) of image b.
__device__ __forceinline__ void merge_tile(const MergeTiledArgs& A, int b, int tile, unsigned char* lds) {
  const bf16_t* __restrict__ tokens = A.tokens;
  const int32_t* __restrict__ offsets = A.offsets;
  const int D = A.D;
  const int32_t* __restrict__ sel_idx = A.sel_idx;
  const int32_t* __restrict__ out_offsets = A.out_offsets;
  const float* __restrict__ plan = A.plan;
  const long long* __restrict__ plan_offsets = A.plan_offsets;
  const float alpha = A.alpha;
  const int max_tokens = A.max_tokens, tiles_d = A.tiles_d;
  bf16_t* __restrict__ out = A.out;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  if (lo < 0 || n <= 0 || n > max_tokens) return;
  const int m = min(max(A.keep[b], 0), n), r = n - m;
  if (r <= kTiledMinPruned) return;                  // k_merge_lds
  const int ti = tile / tiles_d, td = tile - ti * tiles_d;
  const int i0 = ti * kMergeTileRows, d0 = td * kMergeTileCols;
  if (i0 >= m) return;
  const int32_t* sel = sel_idx + lo;
  const float* __restrict__ P = plan + plan_offsets[b];
  const size_t obase = static_cast<size_t>(out_offsets[b]);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;

  constexpr int kOperand = kMergeTileRows * kMergeTilePitch;          // P hi, P lo: one staged operand each
  constexpr int kBuffer = 2 * kOperand + kMergeTileCols * kMergeTurnedPitch;   // [P hi, P lo, T^T]
  constexpr int kStageBytes = 2 * kBuffer;
  constexpr int kOutBytes = 64 * kMergeOutPitch * 4;                  // half of the output tile, fp32
  static_assert(kMergeTiledLdsBytes >= kStageBytes && kMergeTiledLdsBytes >= kOutBytes, "the caller's LDS buffer");

  // staging of P: thread t takes entries 4 (t % 8) .. + 3 of the step for rows t / 8 + 32 q
  const int pj = 4 * (tid & 7), prow = tid >> 3;
  const float* pptr[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) pptr[q] = P + static_cast<long long>(min(i0 + prow + 32 * q, m - 1)) * r;
  // staging of T_prop: thread t takes features 8 (t % 16) .. + 7 of the two pruned rows 2 (t / 16), + 1 of the step
  const int tdg = tid & 15, tjp = tid >> 4;
  float pv[4][4];
  uint4 tv[2];
  auto fetch = [&](int j0) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = j0 + pj + e;
        pv[q][e] = pptr[q][min(j, r - 1)];
      }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int j = min(j0 + 2 * tjp + h, r - 1);
      tv[h] = *reinterpret_cast<const uint4*>(tokens + static_cast<size_t>(lo + clamp_index(sel[m + j], n)) * D +
                                              d0 + 8 * tdg);
    }
  };
  auto stage = [&](int buf, int j0) {
    unsigned char* base = lds + buf * kBuffer;
    // only the last step can reach past the last pruned row: there, what lies past it is zero
    if (j0 + kMergeTileStep > r) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (j0 + pj + e >= r) pv[q][e] = 0.f;
      if (j0 + 2 * tjp >= r) tv[0] = make_uint4(0u, 0u, 0u, 0u);
      if (j0 + 2 * tjp + 1 >= r) tv[1] = make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float hi[4], lo4[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float v = pv[q][e];
        hi[e] = bf16_to_f32(f32_to_bf16(v));
        lo4[e] = v - hi[e];
      }
      uint2 h2, l2;
      h2.x = pack_bf16x2(hi[0], hi[1]);
      h2.y = pack_bf16x2(hi[2], hi[3]);
      l2.x = pack_bf16x2(lo4[0], lo4[1]);
      l2.y = pack_bf16x2(lo4[2], lo4[3]);
      const int off = (prow + 32 * q) * kMergeTilePitch + 2 * pj;
      *reinterpret_cast<uint2*>(base + off) = h2;
      *reinterpret_cast<uint2*>(base + kOperand + off) = l2;
    }
    // turned: feature row 8 tdg + e gets the pair (pruned row 2 tjp, 2 tjp + 1)
    const uint32_t w0[4] = {tv[0].x, tv[0].y, tv[0].z, tv[0].w}, w1[4] = {tv[1].x, tv[1].y, tv[1].z, tv[1].w};
    // features 8 tdg .. + 7 share feature / 16, hence the slot of this thread's piece tjp / 4
    unsigned char* turned = base + 2 * kOperand + 8 * tdg * kMergeTurnedPitch +
                            16 * ((tjp >> 2) ^ ((tdg >> 1) & 7)) + 4 * (tjp & 3);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t a = (e & 1) ? w0[e >> 1] >> 16 : w0[e >> 1] & 0xffffu;
      const uint32_t c = (e & 1) ? w1[e >> 1] & 0xffff0000u : w1[e >> 1] << 16;
      *reinterpret_cast<uint32_t*>(turned + e * kMergeTurnedPitch) = a | c;
    }
  };

  floatx4_t acc[4][4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[t][u] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  // fragment: lane l reads the 16 bytes (eight consecutive pruned rows 8 (l / 16) .. + 7) of row l % 16
  const int frag_off = (lane & 15) * kMergeTilePitch + 16 * (lane >> 4);
  const int steps = (r + kMergeTileStep - 1) / kMergeTileStep;
  fetch(0);
  stage(0, 0);
  __syncthreads();
  for (int s = 0; s < steps; ++s) {
    const int buf = s & 1;
    if (s + 1 < steps) fetch((s + 1) * kMergeTileStep);
    const unsigned char* base = lds + buf * kBuffer;
    uint4 fh[4], fl[4], fb[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      fh[t] = *reinterpret_cast<const uint4*>(base + (64 * wm + 16 * t) * kMergeTilePitch + frag_off);
      fl[t] = *reinterpret_cast<const uint4*>(base + kOperand + (64 * wm + 16 * t) * kMergeTilePitch + frag_off);
      fb[t] = *reinterpret_cast<const uint4*>(base + 2 * kOperand + (64 * wn + 16 * t + (lane & 15)) * kMergeTurnedPitch +
                                              16 * ((lane >> 4) ^ ((4 * wn + t) & 7)));
    }
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, fh[t]),
                                                            __builtin_bit_cast(bf16x8_t, fb[u]), acc[t][u], 0, 0, 0);
        acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, fl[t]),
                                                            __builtin_bit_cast(bf16x8_t, fb[u]), acc[t][u], 0, 0, 0);
      }
    if (s + 1 < steps) stage(buf ^ 1, (s + 1) * kMergeTileStep);
    __syncthreads();
  }

  // accumulator element v of lane l is (kept row 4 (l / 16) + v, feature l % 16) of its tile.
  // Half of the tile (64 kept rows) at a time: through LDS as fp32, then each
  // thread adds eight features of one kept row and writes them as 16 bytes.
  // The thread's eight kept rows' pieces are all requested first (their indices together, then
  // the rows together): two trips to memory instead of sixteen one after the other.
  float* ot = reinterpret_cast<float*>(lds);
  const int dd = 8 * (tid & 15);
  int krow[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) krow[k] = sel[min(i0 + (tid >> 4) + 16 * k, m - 1)];
  uint4 kept[8];
#pragma unroll
  for (int k = 0; k < 8; ++k)
    kept[k] = *reinterpret_cast<const uint4*>(tokens + static_cast<size_t>(lo + clamp_index(krow[k], n)) * D + d0 + dd);
  for (int half = 0; half < 2; ++half) {
    __syncthreads();                                   // the previous use of this LDS is over
    if (wm == half) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            ot[(16 * t + 4 * (lane >> 4) + v) * kMergeOutPitch + 64 * wn + 16 * u + (lane & 15)] = acc[t][u][v];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int row = (tid >> 4) + 16 * q;             // 0 .. 63
      const int i = i0 + 64 * half + row;
      if (i >= m) continue;
      const uint4 kr = half ? kept[4 + q] : kept[q];
      const uint32_t kw[4] = {kr.x, kr.y, kr.z, kr.w};
      const float* src = ot + row * kMergeOutPitch + dd;
      uint32_t ow[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float x0 = __uint_as_float(kw[e] << 16), x1 = __uint_as_float(kw[e] & 0xffff0000u);
        ow[e] = pack_bf16x2(fmaf(alpha, src[2 * e], x0), fmaf(alpha, src[2 * e + 1], x1));
      }
      store_stream(out + (obase + i) * D + d0 + dd, make_uint4(ow[0], ow[1], ow[2], ow[3]));
    }
  }
}

// One workgroup per (tile, image): the staged call, and fused calls whose images
// are known to be large.
__global__ __launch_bounds__(kMergeTiledThreads) void k_merge_tiled(MergeTiledArgs A,
                                                                   const int32_t* __restrict__ status) {
  if (status && status[0]) return;
  __shared__ __attribute__((aligned(16))) unsigned char lds[kMergeTiledLdsBytes];
  merge_tile(A, blockIdx.y, blockIdx.x, lds);
}

}  // namespace rtp
