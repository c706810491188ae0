// Merge and compaction (Eq. 6) on the matrix cores for images with a middling
// number of pruned tokens (kMergeMidMin < R <= kTiledMinPruned = 64): too many for
// the vector kernel, which is then bound by its multiply-adds (1.3 ms for 1024
// pages with 63 pruned tokens each), too few for the LDS-tiled kernel to repay
// its staging of both operands and of the result.  Here the kept rows and the
// result never touch LDS, and the kernel is a stream over the kept rows again.
//
//   out = T_kept + alpha P T_prop      (kept rows x features)
//
// v_mfma_f32_16x16x32_bf16 contracts 32 pruned rows at a time.  Its first
// operand is a 16 x 32 block of P: a lane's eight consecutive pruned rows of one
// kept row are eight consecutive floats of a plan row; each is split into two
// bf16 numbers, P = hi + lo with |P - hi - lo| <= 2^-18 |P| (one bf16 rounding
// would put 2e-3 alpha |T| on the merged features), so each product is two
// matrix instructions accumulated in fp32.  The second operand is a 32 x 16
// block of T_prop, of which a lane wants eight consecutive pruned rows of one
// feature: the workgroup reads the pruned rows as they lie in memory (eight
// lanes per 128-byte line) and turns them round on their way into LDS, two
// bytes at a time, so that each operand is one 16-byte LDS read.  The
// accumulator holds, per lane, four kept rows of one operand column; the columns
// of four instructions stand for features 4 c + h (c the lane's column, h the
// instruction), so a lane ends up with four adjacent features of each of its
// rows and 16 lanes cover 128 contiguous bytes of a kept row, both for the read
// of T_kept and for the write.
//
// A wave owns 16 RB kept rows (their blocks of P split once and kept in
// registers) and walks the features 64 at a time; a workgroup is four waves,
// which share each step's turned pruned rows.
#pragma once
#include "common.hpp"
#include "scores_mfma.hpp"
#include "sinkhorn_team.hpp"
#include "merge_tiled.hpp"

namespace rtp {

static_assert(kTiledMinPruned == 64, "two operand blocks of 32 pruned rows");
constexpr int kMergeMidFeatures = 64;                 // features per step: four instructions' columns
constexpr int kMergeMidRB = 2;                        // 16-row blocks per wave
constexpr int kMergeMidWaveRows = 16 * kMergeMidRB;
constexpr int kMergeMidBlockRows = 4 * kMergeMidWaveRows;
constexpr int kMergeMidThreads = 256;
constexpr int kMergeMidPitch = 72;                    // bf16 per LDS row: 64 pruned rows and 16 bytes
constexpr int kMergeMidBufElems = 64 * kMergeMidPitch;  // one step's turned pruned rows: 64 features x 64 rows

struct MergeMidArgs {
  const bf16_t* tokens;
  const int32_t* offsets;
  int D;
  const int32_t* sel_idx;
  const int32_t* keep;
  const int32_t* out_offsets;
  const float* plan;
  const long long* plan_offsets;
  float alpha;
  int max_tokens;
  bf16_t* out;
};

// Rows i0 .. i0 + kMergeMidBlockRows - 1 of image b.  `bbuf` holds two steps' turned
// pruned rows: the workgroup fetches step s + 1 while it computes step s, as each
// wave does with its kept rows.  LDS row 16 h + c of a step holds feature 4 c + h,
// one bf16 per pruned row (rows 144 bytes apart: the 16 lanes of an operand read
// hit 16 different bank groups).  SPI feature steps are taken per barrier (D / 64 is
// a multiple of SPI): with two, a kept row is read and written 256 contiguous
// bytes at a time.
template <int SPI>
__device__ __forceinline__ void merge_mid_tile(const MergeMidArgs& A, int b, int i0, bf16_t* bbuf) {
  constexpr int RB = kMergeMidRB;
  constexpr int kPitch = kMergeMidPitch;
  const int D = A.D;
  const int lo = A.offsets[b];
  const int n = A.offsets[b + 1] - lo;
  if (lo < 0 || n <= 0 || n > A.max_tokens) return;    // (these are the same for the whole workgroup)
  const int m = min(max(A.keep[b], 0), n), r = n - m;
  if (!merge_is_mid(r) || i0 >= m) return;
  const int steps = D / kMergeMidFeatures;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int iw = i0 + kMergeMidWaveRows * wave;        // the wave's first kept row
  const bool active = iw < m;                          // else the wave only helps to fetch
  const int32_t* sel = A.sel_idx + lo;
  const float* __restrict__ P = A.plan + A.plan_offsets[b];
  const int c = lane & 15, kq = lane >> 4;

  // first operands: kept row iw + 16 rb + c, pruned rows 32 kb + 8 kq .. + 7, as hi and lo
  bf16x8_t phi[RB][2], plo[RB][2];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int i = iw + 16 * rb + c;
    const float* prow = P + static_cast<long long>(min(i, m - 1)) * r;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      uint32_t h[4], l[4];
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const int k = 32 * kb + 8 * kq + e;
        float v0 = prow[min(k, r - 1)], v1 = prow[min(k + 1, r - 1)];
        if (!(i < m && k < r)) v0 = 0.f;
        if (!(i < m && k + 1 < r)) v1 = 0.f;
        const float h0 = bf16_to_f32(f32_to_bf16(v0)), h1 = bf16_to_f32(f32_to_bf16(v1));
        h[e >> 1] = pack_bf16x2(h0, h1);
        l[e >> 1] = pack_bf16x2(v0 - h0, v1 - h1);
      }
      phi[rb][kb] = __builtin_bit_cast(bf16x8_t, make_uint4(h[0], h[1], h[2], h[3]));
      plo[rb][kb] = __builtin_bit_cast(bf16x8_t, make_uint4(l[0], l[1], l[2], l[3]));
    }
  }
  const bool two_blocks = r > 32;                      // pruned rows 32 .. 63 exist (uniform)

  // accumulator element v of block rb: kept row iw + 16 rb + 4 kq + v, features 4 c .. 4 c + 3 of the step
  const char* tbase = reinterpret_cast<const char*>(A.tokens + static_cast<size_t>(lo) * D);
  char* obase = reinterpret_cast<char*>(A.out + static_cast<size_t>(A.out_offsets[b]) * D);
  uint32_t koff[RB][4];                                // byte offsets within the image (at most 8192 rows of 8 KB)
  bool live[RB][4];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int i = iw + 16 * rb + 4 * kq + v;
      live[rb][v] = i < m;
      koff[rb][v] = static_cast<uint32_t>(clamp_index(sel[min(max(i, 0), m - 1)], n) * D + 4 * c) * 2u;
    }
  const uint32_t ooff = static_cast<uint32_t>((iw + 4 * kq) * D + 4 * c) * 2u;
  // fetching: thread t takes pruned rows t / 8 and t / 8 + 32, bytes 16 (t % 8) .. + 15 of the step's 128
  const int pk = tid >> 3, pchunk = tid & 7;
  uint32_t poff[2];
  bool pthere[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int k = pk + 32 * q;
    pthere[q] = k < r;
    poff[q] = static_cast<uint32_t>(clamp_index(sel[m + min(k, r - 1)], n) * D + 8 * pchunk) * 2u;
  }
  // turning: feature 8 pchunk + j of row k goes to LDS row 16 (j % 4) + 2 pchunk + j / 4, column k
  auto turn = [&](bf16_t* buf, const uint4& v0, const uint4& v1) {   // one step
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const uint4& v = q ? v1 : v0;
      const uint32_t w[4] = {pthere[q] ? v.x : 0u, pthere[q] ? v.y : 0u, pthere[q] ? v.z : 0u, pthere[q] ? v.w : 0u};
      bf16_t* dst = buf + 2 * pchunk * kPitch + pk + 32 * q;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        dst[(16 * (j & 3) + (j >> 2)) * kPitch] = static_cast<bf16_t>(w[j >> 1] >> (16 * (j & 1)));
    }
  };

  constexpr int kStepBytes = kMergeMidFeatures * 2;
  __syncthreads();                                     // the previous tile's last step may still read bbuf
#pragma unroll
  for (int ss = 0; ss < SPI; ++ss) {
    const uint4 b0 = *reinterpret_cast<const uint4*>(tbase + poff[0] + ss * kStepBytes);
    const uint4 b1 = *reinterpret_cast<const uint4*>(tbase + poff[1] + ss * kStepBytes);
    turn(bbuf + ss * kMergeMidBufElems, b0, b1);
  }
  uint2 kept[SPI][RB][4];
#pragma unroll
  for (int ss = 0; ss < SPI; ++ss)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v) kept[ss][rb][v] = *reinterpret_cast<const uint2*>(tbase + koff[rb][v] + ss * kStepBytes);

  const int iters = steps / SPI;
  for (int it = 0; it < iters; ++it) {
    // the next steps' operands and kept rows (the last iteration fetches its own again)
    const int nbytes = min(it + 1, iters - 1) * (SPI * kStepBytes);
    uint4 nb[SPI][2];
    uint2 nk[SPI][RB][4];
#pragma unroll
    for (int ss = 0; ss < SPI; ++ss) {
      nb[ss][0] = *reinterpret_cast<const uint4*>(tbase + poff[0] + nbytes + ss * kStepBytes);
      nb[ss][1] = *reinterpret_cast<const uint4*>(tbase + poff[1] + nbytes + ss * kStepBytes);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          nk[ss][rb][v] = *reinterpret_cast<const uint2*>(tbase + koff[rb][v] + nbytes + ss * kStepBytes);
    }
    __syncthreads();                                   // this iteration's operands are in bbuf
    const bf16_t* cur = bbuf + (it & 1) * (SPI * kMergeMidBufElems) + c * kPitch + 8 * kq;
    if (active) {
#pragma unroll
      for (int ss = 0; ss < SPI; ++ss) {
        bf16x8_t t[4][2];
#pragma unroll
        for (int h = 0; h < 4; ++h)
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
            t[h][kb] = *reinterpret_cast<const bf16x8_t*>(cur + ss * kMergeMidBufElems + 16 * h * kPitch + 32 * kb);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          floatx4_t acc[4];
#pragma unroll
          for (int h = 0; h < 4; ++h) {
            const floatx4_t zero = {0.f, 0.f, 0.f, 0.f};
            acc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi[rb][0], t[h][0], zero, 0, 0, 0);
            acc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo[rb][0], t[h][0], acc[h], 0, 0, 0);
            if (two_blocks) {
              acc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi[rb][1], t[h][1], acc[h], 0, 0, 0);
              acc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo[rb][1], t[h][1], acc[h], 0, 0, 0);
            }
          }
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const uint32_t w0 = kept[ss][rb][v].x, w1 = kept[ss][rb][v].y;
            const float x0 = __uint_as_float(w0 << 16), x1 = __uint_as_float(w0 & 0xffff0000u);
            const float x2 = __uint_as_float(w1 << 16), x3 = __uint_as_float(w1 & 0xffff0000u);
            const uint2 o = make_uint2(pack_bf16x2(fmaf(A.alpha, acc[0][v], x0), fmaf(A.alpha, acc[1][v], x1)),
                                       pack_bf16x2(fmaf(A.alpha, acc[2][v], x2), fmaf(A.alpha, acc[3][v], x3)));
            if (live[rb][v])
              store_stream(obase + ooff + static_cast<uint32_t>((16 * rb + v) * D) * 2u +
                               static_cast<uint32_t>(it * SPI + ss) * kStepBytes, o);
          }
        }
      }
    }
    // into the other buffer, which every wave has finished reading before this iteration's barrier
#pragma unroll
    for (int ss = 0; ss < SPI; ++ss)
      turn(bbuf + (((it + 1) & 1) * SPI + ss) * kMergeMidBufElems, nb[ss][0], nb[ss][1]);
#pragma unroll
    for (int ss = 0; ss < SPI; ++ss)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int v = 0; v < 4; ++v) kept[ss][rb][v] = nk[ss][rb][v];
  }
}

// The list forms of both matrix-core merge kernels in one launch (the sizes of the
// pruned sets were decided on the device): a fixed number of workgroups, a multiple
// of eight, first walk the tiles of the images on the tiled list (more than 64
// pruned tokens; merge_tiled.hpp), then the row tiles of the images on this file's
// list.  For the latter, workgroups being dealt to the eight XCDs in turn, item q
// runs on XCD q % 8: the tiles of one image are given items of one residue, and
// its pruned rows are fetched into one L2 only.  `tiles_t` / `tiles_m` = 0: that
// role is not wanted.  Both roles use the same LDS buffer.
template <int SPI>
__global__ __launch_bounds__(kMergeMidThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_merge_lists(
    MergeTiledArgs TA, int tiles_t, MergeMidArgs A, int tiles_m, const int32_t* __restrict__ work, int B, int mid_min,
    const int32_t* __restrict__ status) {
  if (status[0]) return;
  static_assert(kMergeTiledThreads == kMergeMidThreads, "one workgroup shape for both roles");
  constexpr int kLdsBytes = kMergeTiledLdsBytes > 2 * SPI * kMergeMidBufElems * 2 ? kMergeTiledLdsBytes
                                                                                  : 2 * SPI * kMergeMidBufElems * 2;
  __shared__ __attribute__((aligned(16))) unsigned char lds[kLdsBytes];
  if (tiles_t > 0) {
    const int count = work[kListTiled];
    const long long items = static_cast<long long>(count) * tiles_t;
    for (long long item = blockIdx.x; item < items; item += gridDim.x) {
      __syncthreads();   // the previous tile's last LDS reads
      const int k = static_cast<int>(item / tiles_t);
      merge_tile(TA, work[kWorkLists + kListTiled * B + k], static_cast<int>(item - static_cast<long long>(k) * tiles_t), lds);
    }
  }
  if (tiles_m > 0 && merge_mid_runs(work + kListMid, mid_min)) {
    const int count = work[kListMid];
    const long long items = static_cast<long long>((count + 7) / 8) * 8 * tiles_m;
    for (long long q = blockIdx.x; q < items; q += gridDim.x) {
      const long long s = q >> 3;
      const int k = static_cast<int>(s / tiles_m) * 8 + static_cast<int>(q & 7);
      if (k >= count) continue;
      merge_mid_tile<SPI>(A, work[kWorkLists + kListMid * B + k], kMergeMidBlockRows * static_cast<int>(s % tiles_m),
                          reinterpret_cast<bf16_t*>(lds));
    }
  }
}

}  // namespace rtp
