// Textual density (Sec. 3.3.3, Eq. 8; Appendix B): the fraction of pixels whose
// Sobel gradient magnitude reaches tau, per token patch and per image.
//
// Everything is exact integer arithmetic on the 8-bit pixels: the BT.601 luma in
// units of 1/1000 (299 R + 587 G + 114 B), the 3x3 Sobel sums G_x, G_y, and the
// test G_x^2 + G_y^2 >= (tau * 255 * 1000)^2, which is the paper's G >= tau on
// intensities scaled to [0, 1].  The comparison runs in fp32 when it is clear by
// 2e-6 relative and in exact fp64 otherwise, so the edge map does not depend on
// rounding.  Border pixels see their nearest neighbour repeated.
//
// A workgroup takes a strip of `strip` image rows (a divisor of the patch
// height, so a strip never straddles two patch rows) over the full width:
//   1. the strip's rows plus one row above and below are read once, 12 bytes
//      (four pixels) per lane, and their luma goes to LDS;
//   2. every thread walks its columns down the strip with a sliding window of
//      per-row horizontal differences (r - l) and sums (l + 2 c + r);
//   3. per-patch counts are added up in LDS and leave with one integer atomic
//      per patch (integer addition: the result does not depend on the order).
#pragma once
#include "common.hpp"

namespace rtp {

constexpr int kDensityThreads = 256;
constexpr int kDensityLdsBytes = 60 * 1024;   // per workgroup: three or four workgroups share a CU

// Largest divisor of patch_h that is <= 16 and whose strip (plus halo) fits LDS.
inline int density_strip_rows(int patch_h, int max_width) {
  for (int s = 16; s >= 1; --s)
    if (patch_h % s == 0 && static_cast<long long>(s + 2) * (max_width + 2) * 4 <= kDensityLdsBytes) return s;
  return 0;
}

// Zero the patch counters and check every image's geometry.
__global__ __launch_bounds__(256) void k_density_prepare(
    const long long* __restrict__ pixel_offsets, const int32_t* __restrict__ heights,
    const int32_t* __restrict__ widths, int B, int max_h, int max_w, int patch_h, int patch_w,
    int32_t* __restrict__ counts, long long ncounts, int32_t* __restrict__ status) {
  const long long gid = blockIdx.x * 256ll + threadIdx.x;
  for (long long i = gid; i < ncounts; i += 256ll * gridDim.x) counts[i] = 0;
  if (blockIdx.x != 0) return;
  __shared__ int bad;
  if (threadIdx.x == 0) bad = 0;
  __syncthreads();
  int flags = 0;
  for (int b = threadIdx.x; b < B; b += 256) {
    const int h = heights[b], w = widths[b];
    if (h < 0 || w < 0 || h > max_h || w > max_w || h % patch_h != 0 || w % patch_w != 0 ||
        pixel_offsets[b] < 0 || pixel_offsets[b + 1] - pixel_offsets[b] < 3ll * h * w)
      flags |= RTP_DEV_BAD_IMAGE;
  }
  if (flags) atomicOr(&bad, flags);
  __syncthreads();
  if (threadIdx.x == 0) status[0] = bad;
}

// Byte N of a dword as fp32 (the compiler folds the extraction into v_cvt_f32_ubyteN).
template <int N>
__device__ __forceinline__ float byte_f32(uint32_t d) { return static_cast<float>((d >> (8 * N)) & 255u); }

__device__ __forceinline__ int luma_milli(uint32_t r, uint32_t g, uint32_t b) {
  return static_cast<int>(299u * r + 587u * g + 114u * b);
}

__global__ __launch_bounds__(kDensityThreads) void k_density_sobel(
    const unsigned char* __restrict__ pixels, const long long* __restrict__ pixel_offsets,
    const int32_t* __restrict__ heights, const int32_t* __restrict__ widths, int strip, int patch_h,
    int patch_w, int patches_max, float thr2_lo, float thr2_hi, double thr2, int32_t* __restrict__ counts,
    const int32_t* __restrict__ status) {
  if (status[0]) return;
  extern __shared__ __attribute__((aligned(16))) int density_lds[];
  const int b = blockIdx.y;
  const int h = heights[b], w = widths[b];
  const int y0 = blockIdx.x * strip;
  if (y0 >= h || w <= 0) return;
  const int tid = threadIdx.x;
  const unsigned char* img = pixels + pixel_offsets[b];
  const int pitch = w + 2;                      // LDS row: luma of x = -1 .. w
  const int rows = strip + 2;
  int* gray = density_lds;
  int* pcount = density_lds + rows * pitch;     // one counter per patch column
  const int pcols = w / patch_w;
  for (int i = tid; i < pcols; i += kDensityThreads) pcount[i] = 0;

  // ---- 1. luma of rows y0 - 1 .. y0 + strip (clamped) ----
  const bool aligned = ((reinterpret_cast<uintptr_t>(img) | static_cast<uintptr_t>(3 * w)) & 3u) == 0;
  for (int rr = 0; rr < rows; ++rr) {
    const int y = min(max(y0 - 1 + rr, 0), h - 1);
    const unsigned char* row = img + static_cast<size_t>(y) * 3 * w;
    int* g = gray + rr * pitch + 1;
    if (aligned) {
      const uint32_t* row32 = reinterpret_cast<const uint32_t*>(row);
      for (int q = tid; q < (w >> 2); q += kDensityThreads) {
        const uint32_t a = row32[3 * q], c = row32[3 * q + 1], d = row32[3 * q + 2];
        g[4 * q + 0] = luma_milli(a & 255u, (a >> 8) & 255u, (a >> 16) & 255u);
        g[4 * q + 1] = luma_milli(a >> 24, c & 255u, (c >> 8) & 255u);
        g[4 * q + 2] = luma_milli((c >> 16) & 255u, c >> 24, d & 255u);
        g[4 * q + 3] = luma_milli((d >> 8) & 255u, (d >> 16) & 255u, d >> 24);
      }
      for (int x = (w & ~3) + tid; x < w; x += kDensityThreads)
        g[x] = luma_milli(row[3 * x], row[3 * x + 1], row[3 * x + 2]);
    } else {
      for (int x = tid; x < w; x += kDensityThreads)
        g[x] = luma_milli(row[3 * x], row[3 * x + 1], row[3 * x + 2]);
    }
  }
  __syncthreads();
  for (int rr = tid; rr < rows; rr += kDensityThreads) {       // replicate the left and right borders
    int* g = gray + rr * pitch;
    g[0] = g[1];
    g[w + 1] = g[w];
  }
  __syncthreads();

  // ---- 2. Sobel down each column ----
  const int y1 = min(h, y0 + strip);
  for (int x = tid; x < w; x += kDensityThreads) {
    const int* g = gray + x;                    // g[0], g[1], g[2] = left, centre, right of row rr
    int hd0, hd1, hs0, hs1;
    {
      const int l = g[0], c = g[1], r = g[2];
      hd0 = r - l;
      hs0 = l + 2 * c + r;
      const int l1 = g[pitch], c1 = g[pitch + 1], r1 = g[pitch + 2];
      hd1 = r1 - l1;
      hs1 = l1 + 2 * c1 + r1;
    }
    int active = 0;
    for (int y = y0; y < y1; ++y) {
      const int* gn = g + (y - y0 + 2) * pitch;
      const int l = gn[0], c = gn[1], r = gn[2];
      const int hd2 = r - l, hs2 = l + 2 * c + r;
      const int gx = hd0 + 2 * hd1 + hd2;       // right column minus left column, weights 1 2 1
      const int gy = hs0 - hs2;                 // top row minus bottom row, weights 1 2 1
      const float fx = static_cast<float>(gx), fy = static_cast<float>(gy);
      const float f = fmaf(fx, fx, fy * fy);
      bool on;
      if (f > thr2_hi) on = true;
      else if (f < thr2_lo) on = false;
      else {
        const double dx = static_cast<double>(gx), dy = static_cast<double>(gy);
        on = (dx * dx + dy * dy) >= thr2;       // exact: both products and their sum are integers < 2^53
      }
      active += on ? 1 : 0;
      hd0 = hd1; hd1 = hd2;
      hs0 = hs1; hs1 = hs2;
    }
    if (active) atomicAdd(&pcount[x / patch_w], active);
  }
  __syncthreads();
  // ---- 3. one atomic per patch ----
  const int prow = y0 / patch_h;
  for (int i = tid; i < pcols; i += kDensityThreads)
    if (pcount[i]) atomicAdd(&counts[static_cast<long long>(b) * patches_max + prow * pcols + i], pcount[i]);
}

// The same count without LDS, for patch widths that are a multiple of four (every
// native mode: 64 x 64 pixels per token).  A wave walks one patch row of a
// 248-column band: lane l owns the four columns 4 (g0 - 1 + l) .. + 3, reads its
// 12 bytes of each image row straight from memory (three dwords; byte by byte
// when the image does not start on a 4-byte boundary), forms the four lumas and
// gets the two neighbouring columns from the adjacent lanes; lanes 0 and 63 only
// serve as those neighbours.  The three-row window slides down in registers, the
// loads of the next rows are issued six rows ahead.
constexpr int kDensityBand = 62;          // column groups a wave produces
constexpr int kDensityAhead = 6;          // rows in flight; a multiple of 3, so the three-row window
                                          // rotates through statically named registers

// ALIGNED: the page starts on a 4-byte boundary (rows are a multiple of 12 bytes long), so a
// lane's twelve bytes are three dwords.  The choice is made once per page, outside the row
// loop: as a branch around every row's loads it made the compiler copy the whole ring of
// prefetched rows at each row (a quarter of the loop's vector instructions).
template <bool ALIGNED>
__device__ __forceinline__ void density_rows_body(
    const unsigned char* __restrict__ img, int b, int h, int w, int patch_h, int patch_w,
    int patches_max, float thr2_lo, float thr2_hi, double thr2, int32_t* __restrict__ counts) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ngroups = w >> 2;                           // w is a multiple of patch_w, hence of 4
  const int g0 = (blockIdx.x * 4 + wave) * kDensityBand;
  const int y0 = blockIdx.y * patch_h;
  if (g0 >= ngroups || y0 >= h) return;                 // uniform over the wave
  const int gl = g0 - 1 + lane;                         // this lane's column group (may lie outside)
  const int gc = min(max(gl, 0), ngroups - 1);
  const bool produces = lane >= 1 && lane <= kDensityBand && gl < ngroups;
  const size_t pitch = static_cast<size_t>(3) * w;
  const int nrows = patch_h + 2;                        // rows y0 - 1 .. y0 + patch_h, clamped into the image

  auto load_row = [&](int k, uint32_t (&d)[3]) {
    const int y = min(max(y0 - 1 + min(k, nrows - 1), 0), h - 1);
    const unsigned char* p = img + y * pitch + 12 * static_cast<size_t>(gc);
    if (ALIGNED) {
      const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
      d[0] = q[0]; d[1] = q[1]; d[2] = q[2];
    } else {
#pragma unroll
      for (int t = 0; t < 3; ++t)
        d[t] = p[4 * t] | (static_cast<uint32_t>(p[4 * t + 1]) << 8) | (static_cast<uint32_t>(p[4 * t + 2]) << 16) |
               (static_cast<uint32_t>(p[4 * t + 3]) << 24);
    }
  };
  // Horizontal Sobel parts of one image row for the lane's four columns.  All in
  // fp32: bytes are converted directly (v_cvt_f32_ubyte), and every value here is
  // an integer below 2^24 (luma <= 255000, Sobel sums <= 4 x that), so the
  // arithmetic is exact and equals the integer definition.
  auto luma = [](float r, float g, float bl) { return fmaf(299.f, r, fmaf(587.f, g, 114.f * bl)); };
  auto row_parts = [&](const uint32_t (&d)[3], float (&hd)[4], float (&hs)[4]) {
    float g[6];
    g[1] = luma(byte_f32<0>(d[0]), byte_f32<1>(d[0]),
                byte_f32<2>(d[0]));
    g[2] = luma(byte_f32<3>(d[0]), byte_f32<0>(d[1]),
                byte_f32<1>(d[1]));
    g[3] = luma(byte_f32<2>(d[1]), byte_f32<3>(d[1]),
                byte_f32<0>(d[2]));
    g[4] = luma(byte_f32<1>(d[2]), byte_f32<2>(d[2]),
                byte_f32<3>(d[2]));
    const float from_left = __shfl_up(g[4], 1, 64), from_right = __shfl_down(g[1], 1, 64);
    g[0] = gl <= 0 ? g[1] : from_left;                  // the image border repeats its pixel
    g[5] = gl >= ngroups - 1 ? g[4] : from_right;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      hd[c] = g[c + 2] - g[c];
      hs[c] = fmaf(2.f, g[c + 1], g[c]) + g[c + 2];
    }
  };

  uint32_t ring[kDensityAhead][3];
#pragma unroll
  for (int k = 0; k < kDensityAhead; ++k) load_row(k, ring[k]);
  float hd[3][4], hs[3][4];                             // window: row k sits in slot k % 3
  int active = 0;
  // rows are taken six at a time so that ring and window are indexed statically
  for (int kb = 0; kb < nrows; kb += kDensityAhead) {
#pragma unroll
    for (int u = 0; u < kDensityAhead; ++u) {
      const int k = kb + u;
      constexpr int kSlots = 3;
      const int s2 = u % kSlots, s1 = (u + 2) % kSlots, s0 = (u + 1) % kSlots;   // rows k, k - 1, k - 2
      row_parts(ring[u], hd[s2], hs[s2]);               // every lane, also past the last row (shuffles)
      load_row(k + kDensityAhead, ring[u]);             // clamped: always a valid row
      if (k >= 2 && k < nrows && y0 + (k - 2) < h) {    // output row y0 + k - 2 has its three rows
        float gx[4], gy[4];
        bool unsure = false;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          gx[c] = fmaf(2.f, hd[s1][c], hd[s0][c]) + hd[s2][c];
          gy[c] = hs[s0][c] - hs[s2][c];
          const float fx = gx[c], fy = gy[c];
          const float f = fmaf(fx, fx, fy * fy);     // (never a NaN: finite integers)
          const bool above = f > thr2_hi, reaches = f >= thr2_lo;
          active += above ? 1 : 0;
          unsure = unsure || (above != reaches);
        }
        if (unsure) {                                   // within 2e-6 of the threshold: exact, in fp64
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const float fx = gx[c], fy = gy[c];
            const float f = fmaf(fx, fx, fy * fy);
            if (!(f > thr2_hi) && !(f < thr2_lo)) {
              const double dx = static_cast<double>(gx[c]), dy = static_cast<double>(gy[c]);
              active += (dx * dx + dy * dy) >= thr2 ? 1 : 0;
            }
          }
        }
      }
    }
  }
  if (produces && active) {
    const int pcols = w / patch_w;
    atomicAdd(&counts[static_cast<long long>(b) * patches_max + blockIdx.y * pcols + (4 * gl) / patch_w], active);
  }
}

__global__ __launch_bounds__(256) void k_density_rows(
    const unsigned char* __restrict__ pixels, const long long* __restrict__ pixel_offsets,
    const int32_t* __restrict__ heights, const int32_t* __restrict__ widths, int patch_h, int patch_w,
    int patches_max, float thr2_lo, float thr2_hi, double thr2, int32_t* __restrict__ counts,
    const int32_t* __restrict__ status) {
  if (status[0]) return;
  const int b = blockIdx.z;
  const unsigned char* img = pixels + pixel_offsets[b];
  if ((reinterpret_cast<uintptr_t>(img) & 3u) == 0)
    density_rows_body<true>(img, b, heights[b], widths[b], patch_h, patch_w, patches_max, thr2_lo, thr2_hi, thr2, counts);
  else
    density_rows_body<false>(img, b, heights[b], widths[b], patch_h, patch_w, patches_max, thr2_lo, thr2_hi, thr2, counts);
}

// rho_k = count_k / (patch area) and rho = mean over patches, one workgroup per image.
__global__ __launch_bounds__(256) void k_density_finish(
    const int32_t* __restrict__ heights, const int32_t* __restrict__ widths, int patch_h, int patch_w,
    int patches_max, const int32_t* __restrict__ counts, float* __restrict__ density,
    float* __restrict__ patch_density, const int32_t* __restrict__ patch_offsets,
    const int32_t* __restrict__ status) {
  if (status[0]) return;
  __shared__ double red[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int k = (heights[b] / patch_h) * (widths[b] / patch_w);
  const double area = static_cast<double>(patch_h) * static_cast<double>(patch_w);
  const int32_t* c = counts + static_cast<long long>(b) * patches_max;
  double total = 0.0;                                   // integer-valued, exact
  for (int i = tid; i < k; i += 256) {
    const int v = c[i];
    total += static_cast<double>(v);
    if (patch_density) patch_density[patch_offsets[b] + i] = static_cast<float>(static_cast<double>(v) / area);
  }
  total = block_sum<256>(total, red);
  if (tid == 0) density[b] = k > 0 ? static_cast<float>(total / (static_cast<double>(k) * area)) : 0.f;
}

}  // namespace rtp
