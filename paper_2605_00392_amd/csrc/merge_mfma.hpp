// Merge and compaction (Eq. 6) on the matrix cores for images with a middling
// number of pruned tokens (kMergeMidMin < R <= kTiledMinPruned = 64): too many for
// the vector kernel, which is then bound by its multiply-adds (1.3 ms for 1024
// pages with 63 pruned tokens each), too few for the LDS-tiled kernel to repay
// its staging.  Here nothing is staged: both operands come straight from memory
// in the layout the matrix instruction wants, and the kernel is a stream over
// the kept rows again.
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
// feature: a small kernel writes those beforehand (k_transpose_pruned), one
// kilobyte per operand in lane order, so that the load is one contiguous
// kilobyte per wave.  The accumulator holds, per lane, four kept rows of one
// operand column; the columns of four instructions stand for features
// 4 c + h (c the lane's column, h the instruction), so a lane ends up with four
// adjacent features of each of its rows and 16 lanes cover 128 contiguous bytes
// of a kept row, both for the read of T_kept and for the write.
//
// A wave owns 16 RB kept rows (their blocks of P split once and kept in
// registers) and walks the features 64 at a time; a workgroup is four waves.
#pragma once
#include "common.hpp"
#include "scores_mfma.hpp"
#include "sinkhorn_team.hpp"

namespace rtp {

static_assert(kTiledMinPruned == 64, "two operand blocks of 32 pruned rows");
constexpr int kMergeMidFeatures = 64;                 // features per step: four instructions' columns
constexpr int kMergeMidRB = 2;                        // 16-row blocks per wave
constexpr int kMergeMidWaveRows = 16 * kMergeMidRB;
constexpr int kMergeMidBlockRows = 4 * kMergeMidWaveRows;
constexpr int kMergeMidThreads = 256;
// elements of the transposed copy per image: D / 64 steps x 4 instructions x 2 blocks of pruned rows x 64 lanes x 8
__host__ __device__ inline size_t merge_mid_copy_elems(int D) { return static_cast<size_t>(D) * 64; }

// The second operands of every image on the list.  For image b, step s (features
// 64 s ..), instruction h, block kb of 32 pruned rows and lane (kq = lane / 16,
// c = lane % 16), eight bf16: T_prop[32 kb + 8 kq + e][64 s + 4 c + h], e = 0 .. 7,
// zero beyond R.  One workgroup per (step, list entry) at a time.
__global__ __launch_bounds__(256) void k_transpose_pruned(
    const bf16_t* __restrict__ tokens, const int32_t* __restrict__ offsets, int D,
    const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ keep, bf16_t* __restrict__ tpt,
    const int32_t* __restrict__ work, int B, int mid_min, const int32_t* __restrict__ status) {
  if (status[0] || !merge_mid_runs(work + kListMid, mid_min)) return;
  const int count = work[kListMid];
  const int steps = D / kMergeMidFeatures;
  constexpr int kPitch = 72;                           // 64 features and 16 bytes: rows 36 words apart
  __shared__ __align__(16) bf16_t tile[64 * kPitch];
  for (long long item = blockIdx.x; item < static_cast<long long>(count) * steps; item += gridDim.x) {
    const int k_img = static_cast<int>(item / steps), step = static_cast<int>(item - static_cast<long long>(k_img) * steps);
    const int b = work[kWorkLists + kListMid * B + k_img];
    const int lo = offsets[b];
    const int n = offsets[b + 1] - lo;
    const int m = min(max(keep[b], 0), n), r = n - m;
    __syncthreads();                                   // the previous tile is still being read
    if (!merge_is_mid(r)) continue;                    // the list holds nothing else
    const int32_t* sel = sel_idx + lo;
    // 64 pruned rows x 64 features: eight lanes take a row's 128 bytes
    for (int idx = threadIdx.x; idx < 64 * 8; idx += 256) {
      const int k = idx >> 3, seg = idx & 7;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (k < r)
        v = *reinterpret_cast<const uint4*>(tokens + static_cast<size_t>(lo + clamp_index(sel[m + k], n)) * D +
                                            kMergeMidFeatures * step + 8 * seg);
      *reinterpret_cast<uint4*>(&tile[k * kPitch + 8 * seg]) = v;
    }
    __syncthreads();
    bf16_t* dst = tpt + static_cast<size_t>(b) * merge_mid_copy_elems(D) + static_cast<size_t>(step) * (8 * 64 * 8);
    for (int idx = threadIdx.x; idx < 8 * 64; idx += 256) {
      const int lane = idx & 63, kb = (idx >> 6) & 1, h = idx >> 7;
      const int k0 = 32 * kb + 8 * (lane >> 4), f = 4 * (lane & 15) + h;
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 8; e += 2)
        w[e >> 1] = static_cast<uint32_t>(tile[(k0 + e) * kPitch + f]) |
                    (static_cast<uint32_t>(tile[(k0 + e + 1) * kPitch + f]) << 16);
      *reinterpret_cast<uint4*>(dst + static_cast<size_t>(idx) * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}

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
  const bf16_t* tpt;
  bf16_t* out;
};

// Rows i0 .. i0 + kMergeMidBlockRows - 1 of image b.  The four waves share each
// step's second operands (8 KB) through `bbuf` (two such buffers): the workgroup
// fetches step s + 1 while it computes step s, as each wave does with its kept rows.
__device__ __forceinline__ void merge_mid_tile(const MergeMidArgs& A, int b, int i0, bf16_t* bbuf) {
  constexpr int RB = kMergeMidRB;
  constexpr int kStepElems = 8 * 64 * 8;               // the second operands of one step
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
  const bf16_t* __restrict__ tp = A.tpt + static_cast<size_t>(b) * merge_mid_copy_elems(D) + 8 * tid;

  __syncthreads();                                     // the previous tile's last step may still read bbuf
  {
    const uint4 b0 = *reinterpret_cast<const uint4*>(tp), b1 = *reinterpret_cast<const uint4*>(tp + 2048);
    *reinterpret_cast<uint4*>(bbuf + 8 * tid) = b0;
    *reinterpret_cast<uint4*>(bbuf + 2048 + 8 * tid) = b1;
  }
  uint2 kept[RB][4];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) kept[rb][v] = *reinterpret_cast<const uint2*>(tbase + koff[rb][v]);

  for (int s = 0; s < steps; ++s) {
    // the next step's operands and kept rows (the last step fetches its own again)
    const int sn = min(s + 1, steps - 1);
    const bf16_t* tn = tp + static_cast<size_t>(sn) * kStepElems;
    const uint4 nb0 = *reinterpret_cast<const uint4*>(tn), nb1 = *reinterpret_cast<const uint4*>(tn + 2048);
    uint2 nk[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        nk[rb][v] = *reinterpret_cast<const uint2*>(tbase + koff[rb][v] + sn * (kMergeMidFeatures * 2));
    __syncthreads();                                   // this step's operands are in bbuf
    const bf16_t* cur = bbuf + (s & 1) * kStepElems + 8 * lane;
    if (active) {
      bf16x8_t t[4][2];
#pragma unroll
      for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) t[h][kb] = *reinterpret_cast<const bf16x8_t*>(cur + (2 * h + kb) * 512);
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
          const uint32_t w0 = kept[rb][v].x, w1 = kept[rb][v].y;
          const float x0 = __uint_as_float(w0 << 16), x1 = __uint_as_float(w0 & 0xffff0000u);
          const float x2 = __uint_as_float(w1 << 16), x3 = __uint_as_float(w1 & 0xffff0000u);
          const uint2 o = make_uint2(pack_bf16x2(fmaf(A.alpha, acc[0][v], x0), fmaf(A.alpha, acc[1][v], x1)),
                                     pack_bf16x2(fmaf(A.alpha, acc[2][v], x2), fmaf(A.alpha, acc[3][v], x3)));
          if (live[rb][v])
            *reinterpret_cast<uint2*>(obase + ooff + static_cast<uint32_t>((16 * rb + v) * D + s * kMergeMidFeatures) * 2u) = o;
        }
      }
    }
    // into the other buffer, which every wave has finished reading before this step's barrier
    bf16_t* nxt = bbuf + ((s + 1) & 1) * kStepElems + 8 * tid;
    *reinterpret_cast<uint4*>(nxt) = nb0;
    *reinterpret_cast<uint4*>(nxt + 2048) = nb1;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v) kept[rb][v] = nk[rb][v];
  }
}

// A fixed number of workgroups (a multiple of eight) over the row tiles of the
// images on the list.  Workgroups are dealt to the eight XCDs in turn, so item q
// runs on XCD q % 8: the tiles of one image are given items of one residue, and
// its transposed rows are fetched into one L2 only.
__global__ __launch_bounds__(kMergeMidThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void k_merge_mfma(
    MergeMidArgs A, int tiles, const int32_t* __restrict__ work, int B, int mid_min,
    const int32_t* __restrict__ status) {
  if (status[0] || !merge_mid_runs(work + kListMid, mid_min)) return;
  __shared__ __align__(16) bf16_t bbuf[2 * 8 * 64 * 8];
  const int count = work[kListMid];
  const long long items = static_cast<long long>((count + 7) / 8) * 8 * tiles;
  for (long long q = blockIdx.x; q < items; q += gridDim.x) {
    const long long s = q >> 3;
    const int k = static_cast<int>(s / tiles) * 8 + static_cast<int>(q & 7);
    if (k >= count) continue;
    merge_mid_tile(A, work[kWorkLists + kListMid * B + k], kMergeMidBlockRows * static_cast<int>(s % tiles), bbuf);
  }
}

}  // namespace rtp
