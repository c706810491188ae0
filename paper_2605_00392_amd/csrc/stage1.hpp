// Stage 1 and the dynamic ratio: token norms (Eq. 1), the similarity statistic
// phi (Eq. 7) through the identity
//     sum_{i<j} cos(T_i, T_j) = ( || sum_k T_k/||T_k|| ||^2 - sum_k ||T_k/||T_k|| ||^2 ) / 2,
// the retention of Eq. 9, the kept count M = N(1-r), and the top-M selection.
#pragma once
#include "common.hpp"

namespace rtp {

constexpr int kNormRowsPerChunk = 80;   // token rows one workgroup of k_norms covers
constexpr int kNormThreads = 256;

// Validate the ragged layout; every later kernel of the call skips its work
// when the status word is nonzero.  Called by all 256 threads of one workgroup.
__device__ __forceinline__ void validate_offsets(const int32_t* __restrict__ offsets, int B,
                                                 long long total_tokens, int max_tokens,
                                                 int32_t* __restrict__ status) {
  __shared__ int bad;
  if (threadIdx.x == 0) bad = 0;
  __syncthreads();
  int flags = 0;
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    const int lo = offsets[b], hi = offsets[b + 1];
    if (hi < lo || lo < 0) flags |= RTP_DEV_BAD_OFFSETS;
    else if (hi - lo > max_tokens) flags |= RTP_DEV_IMAGE_TOO_LONG;
  }
  if (threadIdx.x == 0) {
    if (offsets[0] != 0) flags |= RTP_DEV_BAD_OFFSETS;
    if (static_cast<long long>(offsets[B]) != total_tokens) flags |= RTP_DEV_BAD_OFFSETS;
  }
  if (flags) atomicOr(&bad, flags);
  __syncthreads();
  if (threadIdx.x == 0) {
    status[0] = bad;
  }
}

__global__ __launch_bounds__(256) void k_prepare(const int32_t* __restrict__ offsets, int B,
                                                 long long total_tokens, int max_tokens,
                                                 int32_t* __restrict__ status) {
  validate_offsets(offsets, B, total_tokens, max_tokens, status);
}

// The fused calls fold the validation into the norm pass, their first kernel: its
// first workgroup validates the whole layout and writes the status word for the
// kernels after it, and every workgroup checks its own image's extent before it reads
// a token (the norm pass writes to the workspace only, so nothing of the caller's is
// touched before the status word exists).
struct NormCheck {
  int on;                  // 0: read the status word k_prepare wrote
  int B;
  long long total_tokens;
  int max_tokens;
  int32_t* status;
};

// One wave per token row.  A lane owns the 4-element groups g = lane + 64 k,
// k < KMAX, of the row (D <= 256 KMAX).  The squared norm is accumulated in
// fp64 (bf16 x bf16 and fp32 x fp32 products are exact in fp64), so its fp32
// rounding - the selection score - does not depend on summation order except
// in astronomically rare rounding-boundary cases.
//
// When `dynamic`, the workgroup also sums T_k / max(||T_k||, tiny) over its rows
// and writes the D-vector (plus sum_k ||unit_k||^2 as element D) to
// partial[(b * parts_per_image + part) * (D + 1) ...].
//
// KFULL = number of k whose 64 groups all lie inside the row (their loads need
// no guard); the remaining k read a clamped address and are zeroed by a select.
//
// VARIANCE: the selection score is the population variance of the row's D values
// instead of its squared norm - the mean first (fp64), then the squared
// deviations from it (fp64), as the definition reads; the norm is still formed
// for the cosines of stage 2.
template <typename T, int KMAX, int KFULL, int NB, bool VARIANCE>
struct NormRows {
  typedef typename Raw4<T>::type raw_t;
  static constexpr int kStep = kNormThreads / kWave;   // row stride between a wave's rows

  // Issue the loads of rows rb, rb + kStep, ... (clamped to last_row), still packed.
  static __device__ __forceinline__ void load(raw_t (&raw)[NB][KMAX], const T* __restrict__ tokens, int lo,
                                              int rb, int last_row, int D, int ngroups, int lane) {
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int r = min(rb + kStep * u, last_row);
      const T* row = tokens + static_cast<size_t>(lo + r) * D;
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        const int g = lane + kWave * k;
        raw[u][k] = load_stream(reinterpret_cast<const raw_t*>(row + 4 * (k < KFULL ? g : min(g, ngroups - 1))));
      }
    }
  }

  // Norms and scores of the loaded rows (those below r1), and their unit vectors
  // into acc32 / wsum.
  static __device__ __forceinline__ void reduce(raw_t (&raw)[NB][KMAX], int lo, int rb, int r1, int ngroups,
                                                int D, int lane, int dynamic, double* __restrict__ norm64,
                                                float* __restrict__ score, float* __restrict__ norms_out,
                                                float (&acc32)[KMAX][4], double& wsum) {
#pragma unroll
    for (int k = KFULL; k < KMAX; ++k)
      if (lane + kWave * k >= ngroups) {
#pragma unroll
        for (int u = 0; u < NB; ++u) raw[u][k] = raw_t{};
      }
    double q[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      double a = 0.0;
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        float x[4];
        unpack4(raw[u][k], x);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const double v = static_cast<double>(x[e]);
          a = fma(v, v, a);
        }
      }
      q[u] = a;
    }
    if constexpr (NB == 4 && !VARIANCE) {
      // The four rows' 64 partial sums each are added up by a reduce-scatter: two
      // halving exchanges leave lane group u = lane / 16 with row u's partials, four
      // steps inside the group finish it (7 additions where four butterflies take
      // 24).  Square root, reciprocal and the stores then run once for the four rows,
      // each lane group on its own row.  (bf16 products have 16-bit significands, so
      // their fp64 sums are exact and no order of additions changes a bit; fp32
      // products round at 1e-16 of the sum, far below the fp32 score's last bit.)
      const double mine = group_sum<4>(halve16(halve32(q[0], q[2]), halve32(q[1], q[3])));
      const int u_own = lane >> 4;                       // = 2 (lane / 32) + (lane / 16) % 2
      const int r_own = rb + kStep * u_own;
      const double nrm = sqrt(mine);
      if ((lane & 15) == 0 && r_own < r1) {
        norm64[lo + r_own] = nrm;
        score[lo + r_own] = static_cast<float>(mine);
        if (norms_out) norms_out[lo + r_own] = static_cast<float>(nrm);
      }
      if (dynamic) {
        const double inv = 1.0 / fmax(nrm, kTinyNorm);
        if (r_own < r1) wsum += mine * inv * inv;        // per lane group; the groups are added at the end
        const float inv_own = static_cast<float>(inv);
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          if (rb + kStep * u >= r1) break;
          const float inv32 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, inv_own), 16 * u));
#pragma unroll
          for (int k = 0; k < KMAX; ++k) {
            forget_origin(raw[u][k]);      // widen again rather than keep 80 floats alive
            float x[4];
            unpack4(raw[u][k], x);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc32[k][e] = fmaf(x[e], inv32, acc32[k][e]);
          }
        }
      }
      return;
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) q[u] = wave_sum_dpp(q[u]);
    double var[NB];
    if (VARIANCE) {
      double mean[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        double a = 0.0;
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
          float x[4];
          unpack4(raw[u][k], x);
#pragma unroll
          for (int e = 0; e < 4; ++e) a += static_cast<double>(x[e]);   // padding groups hold zeros
        }
        mean[u] = a;
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) mean[u] = wave_sum_dpp(mean[u]) / static_cast<double>(D);
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        double a = 0.0;
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
          float x[4];
          unpack4(raw[u][k], x);
          const bool inside = k < KFULL || lane + kWave * k < ngroups;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const double dev = static_cast<double>(x[e]) - mean[u];
            a = inside ? fma(dev, dev, a) : a;
          }
        }
        var[u] = a;
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) var[u] = wave_sum_dpp(var[u]) / static_cast<double>(D);
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int r = rb + kStep * u;
      if (r >= r1) break;
      const double nrm = sqrt(q[u]);
      if (lane == 0) {
        norm64[lo + r] = nrm;
        score[lo + r] = static_cast<float>(VARIANCE ? var[u] : q[u]);
        if (norms_out) norms_out[lo + r] = static_cast<float>(nrm);
      }
      if (dynamic) {
        const double inv = 1.0 / fmax(nrm, kTinyNorm);
        wsum += q[u] * inv * inv;
        const float inv32 = static_cast<float>(inv);
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
          forget_origin(raw[u][k]);      // widen again rather than keep 80 floats alive
          float x[4];
          unpack4(raw[u][k], x);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc32[k][e] = fmaf(x[e], inv32, acc32[k][e]);
        }
      }
    }
  }
};

template <typename T, int KMAX, int KFULL, bool VARIANCE>
__global__ __launch_bounds__(kNormThreads) void k_norms(
    const T* __restrict__ tokens, const int32_t* __restrict__ offsets, int D, int dynamic,
    double* __restrict__ norm64, float* __restrict__ score, float* __restrict__ norms_out,
    double* __restrict__ partial, int parts_per_image, int chunks_per_part,
    NormCheck check) {
  // a workgroup takes `chunks_per_part` consecutive chunks of kNormRowsPerChunk rows
  // of its image and writes one partial vector for all of them
  const int b = blockIdx.y, part = blockIdx.x;
  if (check.on) {
    if (b == 0 && part == 0) validate_offsets(offsets, check.B, check.total_tokens, check.max_tokens, check.status);
  } else if (check.status[0]) {
    return;
  }
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;
  if (check.on && (lo < 0 || n < 0 || n > check.max_tokens || static_cast<long long>(lo) + n > check.total_tokens))
    return;
  if (part * chunks_per_part * kNormRowsPerChunk >= n) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ngroups = D >> 2;

  // Unit vectors x / ||x|| are formed in fp32 (an exact 8- or 24-bit significand
  // times a rounded reciprocal) and a wave adds up those of its own rows - a
  // quarter of the workgroup's rows - in fp32; across waves and workgroups the
  // sums continue in fp64.  The fp32 rounding errors are
  // independent, at most 2^-24 of a partial sum of a few units each, and far
  // below what moves the fp32 value of phi.
  float acc32[KMAX][4];
#pragma unroll
  for (int k = 0; k < KMAX; ++k)
#pragma unroll
    for (int e = 0; e < 4; ++e) acc32[k][e] = 0.f;
  double wsum = 0.0;

  // A wave takes its rows four at a time: the four rows' loads are issued
  // together (raw, still packed), their four squared norms go through the lane
  // butterfly interleaved, and only then are the unit vectors accumulated.
  constexpr int NB = KMAX <= 5 ? 4 : 1;
  typedef NormRows<T, KMAX, KFULL, NB, VARIANCE> Rows;
  constexpr int kStride = Rows::kStep * NB;             // rows between a wave's successive groups
  constexpr int kGroups = kNormRowsPerChunk / kStride;  // groups per wave in a full chunk
  for (int cc = 0; cc < chunks_per_part; ++cc) {
  const int r0 = (part * chunks_per_part + cc) * kNormRowsPerChunk;
  if (r0 >= n) break;
  const int r1 = min(n, r0 + kNormRowsPerChunk);
  if (NB == 4 && kGroups >= 2 && r1 - r0 == kNormRowsPerChunk) {
    // Full chunk: straight-line code over two register buffers, the next group's
    // loads always in flight while the current one is reduced.
    typename Rows::raw_t bufa[NB][KMAX], bufb[NB][KMAX];
    Rows::load(bufa, tokens, lo, r0 + wave, r1 - 1, D, ngroups, lane);
#pragma unroll
    for (int i = 0; i < kGroups; ++i) {
      if (i + 1 < kGroups)
        Rows::load((i & 1) ? bufa : bufb, tokens, lo, r0 + wave + kStride * (i + 1), r1 - 1, D, ngroups, lane);
      __builtin_amdgcn_sched_barrier(0);
      Rows::reduce((i & 1) ? bufb : bufa, lo, r0 + wave + kStride * i, r1, ngroups, D, lane, dynamic, norm64,
                   score,
                   norms_out, acc32, wsum);
    }
  } else {
    for (int rb = r0 + wave; rb < r1; rb += kStride) {
      typename Rows::raw_t raw[NB][KMAX];
      Rows::load(raw, tokens, lo, rb, r1 - 1, D, ngroups, lane);
      Rows::reduce(raw, lo, rb, r1, ngroups, D, lane, dynamic, norm64, score, norms_out, acc32, wsum);
    }
  }
  }
  if (!dynamic) return;

  // The four waves' vectors meet in LDS, laid out by column; every thread then
  // adds the four partials of its columns in fp64 and writes them out.
  constexpr int kWaves = kNormThreads / kWave;
  constexpr int kCols = 4 * kWave * KMAX;
  __shared__ __attribute__((aligned(16))) float lds[kWaves][kCols];
#pragma unroll
  for (int k = 0; k < KMAX; ++k)
    *reinterpret_cast<float4*>(&lds[wave][4 * (lane + kWave * k)]) =
        make_float4(acc32[k][0], acc32[k][1], acc32[k][2], acc32[k][3]);
  __syncthreads();
  double* out = partial + (static_cast<size_t>(b) * parts_per_image + part) * (D + 1);
  for (int c = threadIdx.x; c < D; c += kNormThreads) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += static_cast<double>(lds[w][c]);
    out[c] = s;
  }
  // sum_k ||unit_k||^2: the waves' counts go through the first words of the
  // (now idle) vector buffer
  __syncthreads();
  double* lds_w = reinterpret_cast<double*>(&lds[0][0]);
  if (NB == 4 && !VARIANCE)   // each group of 16 lanes has counted its own rows
    wsum = read_lane(wsum, 0) + read_lane(wsum, 16) + read_lane(wsum, 32) + read_lane(wsum, 48);
  if (lane == 0) lds_w[wave] = wsum;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds_w[w];
    out[D] = s;
  }
}

// One workgroup per image: phi and the retention (when dynamic), the kept
// count, and (when `do_select`) the top-M selection.
//
// Selection: a score's fp32 bit pattern orders like its value (scores are
// >= 0; NaN patterns sort above +inf, which keeps the order total).  The rank
// of token k is the number of tokens that precede it in (score descending,
// index ascending) order; it is kept iff rank < M.  Kept and pruned indices
// are then written in ascending order.
// Up to this many tokens every rank is counted directly; above it the selection
// threshold is found by radix passes (measured: faster from a few hundred tokens on).
constexpr int kRankCountMaxTokens = 128;

struct SelectArgs {
  const int32_t* offsets;
  int D;
  DevParams p;
  const float* density;
  const int32_t* keep_in;
  const float* score;
  const double* partial;
  int parts_per_image, rows_per_part, do_select, max_tokens;
  float* phi_out;
  float* ratio_out;
  int32_t* keep_out;
  int32_t* sel_idx;
};

// Image blockIdx.x on a workgroup of NT threads.
template <int NT>
__device__ __forceinline__ void select_image(const SelectArgs& A) {
  const int32_t* __restrict__ offsets = A.offsets;
  const int D = A.D;
  const DevParams& p = A.p;
  const float* __restrict__ density = A.density;
  const int32_t* __restrict__ keep_in = A.keep_in;
  const float* __restrict__ score = A.score;
  const double* __restrict__ partial = A.partial;
  const int parts_per_image = A.parts_per_image, rows_per_part = A.rows_per_part, do_select = A.do_select,
            max_tokens = A.max_tokens;
  float* __restrict__ phi_out = A.phi_out;
  float* __restrict__ ratio_out = A.ratio_out;
  int32_t* __restrict__ keep_out = A.keep_out;
  int32_t* __restrict__ sel_idx = A.sel_idx;
  // dynamic LDS: 8-byte keys for n_pad = 2 * ceil(max_tokens / 2) tokens, then one flag byte each
  extern __shared__ __attribute__((aligned(16))) unsigned char select_lds[];
  unsigned long long* keys = reinterpret_cast<unsigned long long*>(select_lds);
  unsigned char* kept_flag = select_lds + 8 * static_cast<size_t>((max_tokens + 1) & ~1);
  __shared__ double red[NT / 64];
  __shared__ int counts[NT];
  __shared__ int s_m;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int lo = offsets[b];
  const int n = offsets[b + 1] - lo;

  double phi = 0.0;
  float ret32 = p.ratio;
  if (p.dynamic) {
    if (n >= 2) {
      const int nchunks = (n + rows_per_part - 1) / rows_per_part;
      const double* base = partial + static_cast<size_t>(b) * parts_per_image * (D + 1);
      double local = 0.0;
      for (int d = tid; d < D; d += NT) {
        double s = 0.0;
        for (int c = 0; c < nchunks; ++c) s += base[static_cast<size_t>(c) * (D + 1) + d];
        local = fma(s, s, local);
      }
      const double ss = block_sum<NT>(local, red);
      double w = 0.0;
      for (int c = 0; c < nchunks; ++c) w += base[static_cast<size_t>(c) * (D + 1) + D];
      phi = (ss - w) / (static_cast<double>(n) * static_cast<double>(n - 1));
    }
    ret32 = dynamic_retention(phi, density[b], p);
  }
  if (tid == 0) {
    int m;
    if (keep_in && !p.dynamic) {
      m = keep_in[b];
      m = n > 0 ? min(n, max(1, m)) : 0;
    } else {
      m = kept_count(ret32, n);
    }
    s_m = m;
    keep_out[b] = m;
    if (phi_out) phi_out[b] = static_cast<float>(phi);
    if (ratio_out) ratio_out[b] = ret32;
  }
  if (!do_select || n == 0) return;
  // 64-bit key = (score bits, ~index): token l precedes token k in (score
  // descending, index ascending) order exactly when key_l > key_k.
  const int n_pad = (n + 1) & ~1;
  for (int k = tid; k < n_pad; k += NT)
    keys[k] = k < n ? (static_cast<unsigned long long>(__float_as_uint(score[lo + k])) << 32) |
                          (0xffffffffu - static_cast<uint32_t>(k))
                    : 0ull;                                   // padding precedes nothing
  __syncthreads();
  const int m = s_m;

  if (n <= kRankCountMaxTokens) {
    // few tokens: count every token's rank directly (n^2 comparisons of LDS keys)
    const ulonglong2* keys2 = reinterpret_cast<const ulonglong2*>(keys);
    for (int kb = tid; kb < n; kb += 4 * NT) {
      unsigned long long mine[4];
      int rank[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        mine[u] = keys[min(kb + NT * u, n - 1)];
        rank[u] = 0;
      }
      for (int l2 = 0; l2 < n_pad / 2; ++l2) {
        const ulonglong2 o = keys2[l2];                         // same address in every lane
#pragma unroll
        for (int u = 0; u < 4; ++u) rank[u] += (o.x > mine[u]) + (o.y > mine[u]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (kb + NT * u < n) kept_flag[kb + NT * u] = rank[u] < m;
    }
  } else {
    // many tokens: find the M-th largest key byte by byte from the top (keys are
    // distinct).  Each pass histograms the next byte of the keys that share the
    // bytes found so far and picks the bin that holds the M-th largest; it can
    // stop as soon as that bin is needed whole.
    __shared__ int hist[256];
    __shared__ int s_bin, s_need, s_whole;
    unsigned long long prefix = 0;     // the bytes found so far, right-aligned
    int need = m, shift = 56;
    for (;; shift -= 8) {
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      for (int k = tid; k < n; k += NT) {
        const unsigned long long key = keys[k];
        if (shift == 56 || (key >> (shift + 8)) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1);
      }
      __syncthreads();
      if (tid < 64) {
        // lane l holds bins 4 l .. 4 l + 3; `above` = keys in bins higher than the lane's
        const int h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
        const int mine = h0 + h1 + h2 + h3;
        int above = mine;                                   // inclusive suffix sum over lanes >= l
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int v = __shfl_down(above, o, kWave);
          if (tid + o < 64) above += v;
        }
        above -= mine;
        if (above < need && need <= above + mine) {         // exactly one lane
          int bin = 4 * tid + 3, cnt = h3, left = need - above;
          if (left > cnt) { left -= cnt; bin = 4 * tid + 2; cnt = h2;
            if (left > cnt) { left -= cnt; bin = 4 * tid + 1; cnt = h1;
              if (left > cnt) { left -= cnt; bin = 4 * tid; cnt = h0; } } }
          s_bin = bin;
          s_need = left;
          s_whole = left == cnt;
        }
      }
      __syncthreads();
      prefix = (prefix << 8) | static_cast<unsigned long long>(s_bin);
      need = s_need;
      if (s_whole || shift == 0) break;                     // at shift 0 a bin holds one key
    }
    for (int k = tid; k < n; k += NT) kept_flag[k] = (keys[k] >> shift) >= prefix;
  }
  __syncthreads();

  // Each thread owns a contiguous span of tokens; exclusive scan of the spans'
  // kept counts gives every token its position in the ascending kept / pruned lists.
  const int span = (n + NT - 1) / NT;
  const int k0 = min(n, tid * span), k1 = min(n, k0 + span);
  int c = 0;
  for (int k = k0; k < k1; ++k) c += kept_flag[k];
  counts[tid] = c;
  __syncthreads();
  for (int o = 1; o < NT; o <<= 1) {
    const int v = tid >= o ? counts[tid - o] : 0;
    __syncthreads();
    counts[tid] += v;
    __syncthreads();
  }
  int kept_before = counts[tid] - c;
  for (int k = k0; k < k1; ++k) {
    if (kept_flag[k]) {
      sel_idx[lo + kept_before] = k;
      ++kept_before;
    } else {
      sel_idx[lo + m + (k - kept_before)] = k;
    }
  }
}

template <int NT>
__global__ __launch_bounds__(NT) void k_select(SelectArgs A, const int32_t* __restrict__ status) {
  if (status[0]) return;
  select_image<NT>(A);
}

// Exclusive prefix sums over the images: out_offsets = scan(M_b) (int32),
// plan_offsets = scan(M_b * R_b) (int64).  One workgroup of 256 threads.
// `plan_stride` > 0 (the fused calls): plan_offsets[b] = offsets[b] * plan_stride
// instead, a slot of N_b * plan_stride >= M_b R_b entries per image that needs no
// sum over the other images (see plan_slot).
__device__ __forceinline__ long long plan_slot(const int32_t* __restrict__ offsets, int b, long long plan_stride) {
  return static_cast<long long>(offsets[b]) * plan_stride;
}
constexpr int kScanLdsBytes = 2 * 256 * 8;   // LDS scan_images works in
__device__ __forceinline__ void scan_images(const int32_t* __restrict__ offsets,
                                            const int32_t* __restrict__ keep, int B,
                                            int32_t* __restrict__ out_offsets,
                                            long long* __restrict__ plan_offsets, void* lds,
                                            long long plan_stride = 0) {
  long long* sm = static_cast<long long*>(lds);   // [256]
  long long* sp = sm + 256;                       // [256]
  const int tid = threadIdx.x;
  const int span = (B + 255) / 256;
  const int b0 = min(B, tid * span), b1 = min(B, b0 + span);
  long long cm = 0, cp = 0;
  for (int b = b0; b < b1; ++b) {
    const long long m = keep[b];
    const long long n = offsets[b + 1] - offsets[b];
    cm += m;
    cp += m * (n - m);
  }
  sm[tid] = cm;
  sp[tid] = cp;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const long long vm = tid >= o ? sm[tid - o] : 0, vp = tid >= o ? sp[tid - o] : 0;
    __syncthreads();
    sm[tid] += vm;
    sp[tid] += vp;
    __syncthreads();
  }
  long long am = sm[tid] - cm, ap = sp[tid] - cp;
  for (int b = b0; b < b1; ++b) {
    if (out_offsets) out_offsets[b] = static_cast<int32_t>(am);
    if (plan_offsets) plan_offsets[b] = plan_stride > 0 ? plan_slot(offsets, b, plan_stride) : ap;
    const long long m = keep[b];
    const long long n = offsets[b + 1] - offsets[b];
    am += m;
    ap += m * (n - m);
  }
  if (tid == 255) {
    if (out_offsets) out_offsets[B] = static_cast<int32_t>(sm[255]);
    if (plan_offsets) plan_offsets[B] = plan_stride > 0 ? plan_slot(offsets, B, plan_stride) : sp[255];
  }
}

__global__ __launch_bounds__(256) void k_scan(const int32_t* __restrict__ offsets,
                                              const int32_t* __restrict__ keep, int B,
                                              int32_t* __restrict__ out_offsets,
                                              long long* __restrict__ plan_offsets,
                                              const int32_t* __restrict__ status) {
  if (status[0]) return;
  __shared__ __align__(16) unsigned char lds[kScanLdsBytes];
  scan_images(offsets, keep, B, out_offsets, plan_offsets, lds);
}

}  // namespace rtp
