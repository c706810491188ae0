// Sequence splice: the pruned, merged visual tokens go straight into the
// language model's prefill input (the pruning runs before the prefill stage,
// Sec. 4.3) - per image: text embeddings before the image, the kept visual
// tokens, text embeddings after it - with a position id per token.
//
//   k_splice_check  validates the two text-span offset arrays (adds to the status word)
//   k_splice_scan   seq_offsets[b] = sum_{b' < b} (P + M + S), and the row at which
//                   image b's visual tokens start (what the merge kernel writes to)
//   k_splice_text   copies the text rows and writes every position id
#pragma once
#include "common.hpp"

namespace rtp {

struct TextSpans {
  const void* prefix;
  const int32_t* prefix_offsets;   // null: no prefix anywhere
  long long prefix_rows;
  const void* suffix;
  const int32_t* suffix_offsets;   // null: no suffix anywhere
  long long suffix_rows;
};

__device__ __forceinline__ int span_len(const int32_t* __restrict__ off, int b) {
  return off ? off[b + 1] - off[b] : 0;
}

__global__ __launch_bounds__(256) void k_splice_check(TextSpans t, int B, int32_t* __restrict__ status) {
  int flags = 0;
  for (int b = threadIdx.x; b < B; b += 256) {
    if (t.prefix_offsets && (t.prefix_offsets[b + 1] < t.prefix_offsets[b] || t.prefix_offsets[b] < 0))
      flags |= RTP_DEV_BAD_OFFSETS;
    if (t.suffix_offsets && (t.suffix_offsets[b + 1] < t.suffix_offsets[b] || t.suffix_offsets[b] < 0))
      flags |= RTP_DEV_BAD_OFFSETS;
  }
  if (threadIdx.x == 0) {
    if (t.prefix_offsets && (t.prefix_offsets[0] != 0 || t.prefix_offsets[B] != t.prefix_rows)) flags |= RTP_DEV_BAD_OFFSETS;
    if (t.suffix_offsets && (t.suffix_offsets[0] != 0 || t.suffix_offsets[B] != t.suffix_rows)) flags |= RTP_DEV_BAD_OFFSETS;
  }
  if (flags) atomicOr(status, flags);
}

// One workgroup; image order.
__global__ __launch_bounds__(256) void k_splice_scan(TextSpans t, const int32_t* __restrict__ keep, int B,
                                                     int32_t* __restrict__ seq_offsets,
                                                     int32_t* __restrict__ visual_start,
                                                     const int32_t* __restrict__ status) {
  if (status[0]) return;
  __shared__ long long sm[256];
  const int tid = threadIdx.x;
  const int span = (B + 255) / 256;
  const int b0 = min(B, tid * span), b1 = min(B, b0 + span);
  long long c = 0;
  for (int b = b0; b < b1; ++b) c += span_len(t.prefix_offsets, b) + keep[b] + span_len(t.suffix_offsets, b);
  sm[tid] = c;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const long long v = tid >= o ? sm[tid - o] : 0;
    __syncthreads();
    sm[tid] += v;
    __syncthreads();
  }
  long long at = sm[tid] - c;
  for (int b = b0; b < b1; ++b) {
    seq_offsets[b] = static_cast<int32_t>(at);
    visual_start[b] = static_cast<int32_t>(at + span_len(t.prefix_offsets, b));
    at += span_len(t.prefix_offsets, b) + keep[b] + span_len(t.suffix_offsets, b);
  }
  if (tid == 255) seq_offsets[B] = static_cast<int32_t>(sm[255]);
}

// Workgroup (x, b): rows x, x + gridDim.x, ... of image b's sequence.  A row of
// D elements is D * sizeof(T) / 16 sixteen-byte pieces (the library's width
// limits make that exact).
template <typename T>
__global__ __launch_bounds__(256) void k_splice_text(TextSpans t, const int32_t* __restrict__ offsets,
                                                     const int32_t* __restrict__ keep,
                                                     const int32_t* __restrict__ sel_idx, int D, int mode,
                                                     const int32_t* __restrict__ seq_offsets,
                                                     T* __restrict__ seq, int32_t* __restrict__ position_ids,
                                                     const int32_t* __restrict__ status) {
  if (status[0]) return;
  const int b = blockIdx.y;
  const int lo = offsets[b], n = offsets[b + 1] - lo;
  const int P = span_len(t.prefix_offsets, b), S = span_len(t.suffix_offsets, b);
  const int M = min(max(keep[b], 0), n);
  const int len = P + M + S;
  const long long base = seq_offsets[b];
  const int pieces = static_cast<int>(static_cast<long long>(D) * sizeof(T) / 16);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int k = blockIdx.x * 4 + wave; k < len; k += gridDim.x * 4) {
    int pos;
    const uint4* src = nullptr;
    if (k < P) {
      pos = k;
      src = reinterpret_cast<const uint4*>(static_cast<const T*>(t.prefix) +
                                           static_cast<size_t>(t.prefix_offsets[b] + k) * D);
    } else if (k < P + M) {
      const int i = k - P;                                   // the merge kernel writes this row
      pos = mode == 0 ? k : P + clamp_index(sel_idx[lo + i], n);
    } else {
      const int q = k - P - M;
      pos = mode == 0 ? k : P + n + q;
      src = reinterpret_cast<const uint4*>(static_cast<const T*>(t.suffix) +
                                           static_cast<size_t>(t.suffix_offsets[b] + q) * D);
    }
    if (lane == 0 && position_ids) position_ids[base + k] = pos;
    if (src) {
      uint4* dst = reinterpret_cast<uint4*>(seq + static_cast<size_t>(base + k) * D);
      for (int g = lane; g < pieces; g += 64) store_stream(dst + g, src[g]);
    }
  }
}

}  // namespace rtp
