// Shared device helpers for the RTPrune HIP kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace rtp {

constexpr int kWave = 64;
constexpr int kMaxTokens = 8192;   // per image
constexpr int kMaxD = 4096;
constexpr int kMaxImages = 65535;  // per call: an image is a row (y) of the launch grids
constexpr double kTinyNorm = 1e-12;

typedef unsigned short bf16_t;     // raw bfloat16 bit pattern

// Hyper-parameters widened once on the host; z, alpha, eps are the doubles of
// the float32 values the caller passed.
// Images with more pruned tokens than this take the LDS-tiled matrix-core
// kernels for the scores and the merge (bf16 tokens, width a multiple of 128).
// (Measured on 1024 pages of 400 tokens: from 65 pruned tokens on the tiled merge is
// 1.3 to 2 times faster than the vector kernel and the tiled scores are level or
// better.)
constexpr int kTiledMinPruned = 64;
// Between kMergeMidMin and kTiledMinPruned pruned tokens the merge runs on the
// matrix cores with only the pruned rows staged (merge_mfma.hpp; bf16 tokens, width a multiple of 64).
constexpr int kMergeMidMin = 16;
__host__ __device__ inline bool merge_is_mid(int r) { return r > kMergeMidMin && r <= kTiledMinPruned; }
// Which images the vector merge kernels leave to the others.  The middling ones
// only when the call has many (`mid_count`, counted on the device, at least
// `mid_min`): a few of them cost less inside the vector kernel's one large launch
// than as two short launches of their own.
constexpr int kSkipTiled = 1, kSkipMid = 2;
struct MergeSkip {
  int mask;
  const int32_t* mid_count;   // device; read only when mask has kSkipMid
  int mid_min;
};
__device__ __forceinline__ bool merge_mid_runs(const int32_t* mid_count, int mid_min) { return *mid_count >= mid_min; }
__device__ __forceinline__ bool merge_elsewhere(const MergeSkip& k, int r) {
  if ((k.mask & kSkipTiled) && r > kTiledMinPruned) return true;
  return (k.mask & kSkipMid) && merge_is_mid(r) && merge_mid_runs(k.mid_count, k.mid_min);
}

struct DevParams {
  double z, alpha, eps;
  double shift;      // max(1, z): exp((s - shift) / eps) <= 1 for every score s
  float ratio, ratio_min, ratio_max, phi_lo, phi_hi;
  int iters, dynamic, metric;
  int mid_min;  // rtprune_params::mid_merge_min_images (0: decided by the size of the chip)
  int mode;    // which Sinkhorn kernels the call launches (kMode... bits)
  int k32;     // those images' kernel matrix is stored in fp32 (its range allows it)
};

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// Round to nearest even; NaN stays NaN.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}

// Four consecutive elements of a token row, widened to float.
__device__ __forceinline__ void load4(const bf16_t* p, float (&x)[4]) {
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  x[0] = __uint_as_float(u.x << 16);
  x[1] = __uint_as_float(u.x & 0xffff0000u);
  x[2] = __uint_as_float(u.y << 16);
  x[3] = __uint_as_float(u.y & 0xffff0000u);
}
__device__ __forceinline__ void load4(const float* p, float (&x)[4]) {
  const float4 u = *reinterpret_cast<const float4*>(p);
  x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w;
}
// fp32 -> bf16, round to nearest even, two at a time (v_cvt_pk_bf16_f32).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const floatx2_t f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}
__device__ __forceinline__ void store4(bf16_t* p, const float (&x)[4]) {
  uint2 u;
  u.x = pack_bf16x2(x[0], x[1]);
  u.y = pack_bf16x2(x[2], x[3]);
  *reinterpret_cast<uint2*>(p) = u;
}
__device__ __forceinline__ void store4(float* p, const float (&x)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
}

// The same as streaming stores, for the rows of the output: nothing in the call reads them
// again, and left in the caches as ordinary dirty lines they are written back while the next
// call's first pass reads (measured on 1024 pages of 400 tokens: that pass 229 -> 204 us).
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store4_stream(bf16_t* p, const float (&x)[4]) {
  const u32x2_t u = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3])};
  __builtin_nontemporal_store(u, reinterpret_cast<u32x2_t*>(p));
}
__device__ __forceinline__ void store4_stream(float* p, const float (&x)[4]) {
  const f32x4_t u = {x[0], x[1], x[2], x[3]};
  __builtin_nontemporal_store(u, reinterpret_cast<f32x4_t*>(p));
}
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_stream(void* p, const uint2& v) {
  const u32x2_t u = {v.x, v.y};
  __builtin_nontemporal_store(u, static_cast<u32x2_t*>(p));
}
__device__ __forceinline__ void store_stream(void* p, const uint4& v) {
  const u32x4_t u = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(u, static_cast<u32x4_t*>(p));
}
__device__ __forceinline__ uint2 load_stream(const uint2* p) {
  const u32x2_t u = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
  return make_uint2(u.x, u.y);
}
__device__ __forceinline__ float4 load_stream(const float4* p) {
  const f32x4_t u = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  return make_float4(u.x, u.y, u.z, u.w);
}

// A 4-element group of a token row as it sits in memory, and its widening.
template <typename T> struct Raw4;
template <> struct Raw4<bf16_t> { typedef uint2 type; };
template <> struct Raw4<float> { typedef float4 type; };
__device__ __forceinline__ void unpack4(const uint2& u, float (&x)[4]) {
  x[0] = __uint_as_float(u.x << 16);
  x[1] = __uint_as_float(u.x & 0xffff0000u);
  x[2] = __uint_as_float(u.y << 16);
  x[3] = __uint_as_float(u.y & 0xffff0000u);
}
__device__ __forceinline__ void unpack4(const float4& u, float (&x)[4]) {
  x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w;
}

// Make the compiler forget where a register value came from (blocks common
// subexpression elimination across the call; emits no instruction).
__device__ __forceinline__ void forget_origin(uint2& u) { asm volatile("" : "+v"(u.x), "+v"(u.y)); }
__device__ __forceinline__ void forget_origin(float& u) { asm volatile("" : "+v"(u)); }
__device__ __forceinline__ void forget_origin(int& u) { asm volatile("" : "+v"(u)); }
__device__ __forceinline__ void forget_origin(double& u) { asm volatile("" : "+v"(u)); }
__device__ __forceinline__ void forget_origin(float4& u) {
  asm volatile("" : "+v"(u.x), "+v"(u.y), "+v"(u.z), "+v"(u.w));
}

// Butterfly sum over the 64 lanes of a wave; every lane gets the total.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
// The same total with register-to-register lane exchanges only (no LDS
// crossbar): two quad permutes and two mirror steps inside each row of 16
// lanes - after the quad steps all lanes of a quad agree, so mirroring 8 and
// then 16 lanes pairs each group with its neighbour - then the row swap and
// half swap instructions, which hand each lane its partner's value in the other
// operand.  Every lane gets the total.
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, false);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_sum_dpp(double v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror
  {
    const unsigned lo = __double2loint(v), hi = __double2hiint(v);
    const auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    v = __hiloint2double(static_cast<int>(b[0]), static_cast<int>(a[0])) +
        __hiloint2double(static_cast<int>(b[1]), static_cast<int>(a[1]));
  }
  {
    const unsigned lo = __double2loint(v), hi = __double2hiint(v);
    const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    v = __hiloint2double(static_cast<int>(b[0]), static_cast<int>(a[0])) +
        __hiloint2double(static_cast<int>(b[1]), static_cast<int>(a[1]));
  }
  return v;
}
// v + (the value of lane ^ MASK) for one lane bit.  Bits 0, 1 and 3 have an exact
// register-to-register permutation (quad permutes, a rotation by 8 inside a row
// of 16), bits 4 and 5 the swap instructions; bit 2 goes through the LDS crossbar.
template <int MASK>
__device__ __forceinline__ double add_xor_lane(double v) {
  static_assert(MASK == 1 || MASK == 2 || MASK == 4 || MASK == 8 || MASK == 16 || MASK == 32, "one lane bit");
  if constexpr (MASK == 1) return v + dpp_move<0xB1>(v);
  else if constexpr (MASK == 2) return v + dpp_move<0x4E>(v);
  else if constexpr (MASK == 4) return v + __shfl_xor(v, 4, kWave);
  else if constexpr (MASK == 8) return v + dpp_move<0x128>(v);
  else {
    const unsigned lo = __double2loint(v), hi = __double2hiint(v);
    if constexpr (MASK == 16) {
      const auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
      const auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
      return __hiloint2double(static_cast<int>(b[0]), static_cast<int>(a[0])) +
             __hiloint2double(static_cast<int>(b[1]), static_cast<int>(a[1]));
    } else {
      const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
      const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
      return __hiloint2double(static_cast<int>(b[0]), static_cast<int>(a[0])) +
             __hiloint2double(static_cast<int>(b[1]), static_cast<int>(a[1]));
    }
  }
}
// Sum over each aligned group of 2^LOG lanes (every lane of the group gets it):
// the first LOG steps of wave_sum_dpp, whose mirror steps rely on the lanes
// below already agreeing.
template <int LOG>
__device__ __forceinline__ double group_sum(double v) {
  if constexpr (LOG >= 1) v += dpp_move<0xB1>(v);
  if constexpr (LOG >= 2) v += dpp_move<0x4E>(v);
  if constexpr (LOG >= 3) v += dpp_move<0x141>(v);
  if constexpr (LOG >= 4) v += dpp_move<0x140>(v);
  if constexpr (LOG >= 5) v = add_xor_lane<16>(v);
  if constexpr (LOG >= 6) v = add_xor_lane<32>(v);
  return v;
}
// Sum over the lanes that share the low LOG lane bits (every one of them gets it).
template <int LOG>
__device__ __forceinline__ double cross_sum(double v) {
  if constexpr (LOG <= 0) v = add_xor_lane<1>(v);
  if constexpr (LOG <= 1) v = add_xor_lane<2>(v);
  if constexpr (LOG <= 2) v = add_xor_lane<4>(v);
  if constexpr (LOG <= 3) v = add_xor_lane<8>(v);
  if constexpr (LOG <= 4) v = add_xor_lane<16>(v);
  if constexpr (LOG <= 5) v = add_xor_lane<32>(v);
  return v;
}
// a + (the partner's b) on lanes whose bit is clear, (the partner's a) + b on
// the others, the partner being lane ^ 32: the low half keeps a, the high half b.
__device__ __forceinline__ double halve32(double a, double b) {
  const auto lo = __builtin_amdgcn_permlane32_swap(__double2loint(a), __double2loint(b), false, false);
  const auto hi = __builtin_amdgcn_permlane32_swap(__double2hiint(a), __double2hiint(b), false, false);
  return __hiloint2double(static_cast<int>(hi[0]), static_cast<int>(lo[0])) +
         __hiloint2double(static_cast<int>(hi[1]), static_cast<int>(lo[1]));
}
// The same over lane ^ 16: even 16-lane rows keep a, odd rows keep b.
__device__ __forceinline__ double halve16(double a, double b) {
  const auto lo = __builtin_amdgcn_permlane16_swap(__double2loint(a), __double2loint(b), false, false);
  const auto hi = __builtin_amdgcn_permlane16_swap(__double2hiint(a), __double2hiint(b), false, false);
  return __hiloint2double(static_cast<int>(hi[0]), static_cast<int>(lo[0])) +
         __hiloint2double(static_cast<int>(hi[1]), static_cast<int>(lo[1]));
}
__device__ __forceinline__ double read_lane(double v, int src) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), src),
                          __builtin_amdgcn_readlane(__double2loint(v), src));
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Sum over a workgroup of NT threads (NT a multiple of 64, <= 1024).  `red`
// holds at least NT / 64 doubles of LDS.  Every thread gets the total.
template <int NT>
__device__ __forceinline__ double block_sum(double v, double* red) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  v = wave_sum(v);
  __syncthreads();               // `red` may still be read from a previous call
  if (lane == 0) red[wave] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) t += red[w];
  return t;
}

// exp(x) for x in [-700, 1] (the kernel matrix's exponents: never above a rounding error over 0,
// and the host refuses parameters that could bring them below -600), without the library routine's special cases: x = k ln 2 + f with |f| <= ln 2 / 2
// (ln 2 in two parts, so that f is exact to the last bit), exp(f) by its Taylor polynomial of
// degree 13 (remainder below 4e-18 relative), times 2^k.  About 20 instructions, relative error
// 2e-16.
__device__ __forceinline__ double exp_nonpositive(double x) {
  const double k = rint(x * 1.4426950408889634074);
  double f = fma(k, -6.93147180369123816490e-01, x);
  f = fma(k, -1.90821492927058770002e-10, f);
  double q = 1.0 / 6227020800.0;
  q = fma(q, f, 1.0 / 479001600.0);
  q = fma(q, f, 1.0 / 39916800.0);
  q = fma(q, f, 1.0 / 3628800.0);
  q = fma(q, f, 1.0 / 362880.0);
  q = fma(q, f, 1.0 / 40320.0);
  q = fma(q, f, 1.0 / 5040.0);
  q = fma(q, f, 1.0 / 720.0);
  q = fma(q, f, 1.0 / 120.0);
  q = fma(q, f, 1.0 / 24.0);
  q = fma(q, f, 1.0 / 6.0);
  q = fma(q, f, 0.5);
  q = fma(q, f, 1.0);
  q = fma(q, f, 1.0);
  return ldexp(q, static_cast<int>(k));
}

// Index and extent guards for arrays that arrive from the caller (staged calls):
// a wrong entry may give a wrong result but never an out-of-bounds access.
__device__ __forceinline__ int clamp_index(int t, int n) { return min(max(t, 0), n - 1); }
__device__ __forceinline__ bool plan_fits(long long off, int m, int r, long long cap) {
  return off >= 0 && off + static_cast<long long>(m) * r <= cap;
}

// Kept count M = ceil(retention * N - 1e-3) clamped to [1, N] (0 for N = 0).
// The product and the subtraction are rounded separately (no fused multiply-add)
// so that the integer is the same one a host evaluation in doubles gives.
__host__ __device__ inline int kept_count(float retention, int n) {
#pragma clang fp contract(off)
  if (n <= 0) return 0;
  if (!(retention == retention)) return n;
  const double prod = static_cast<double>(retention) * static_cast<double>(n);
  const double v = prod - 1e-3;
  double c = ceil(v);
  if (c < 1.0) c = 1.0;
  if (c > static_cast<double>(n)) c = static_cast<double>(n);
  return static_cast<int>(c);
}

// Retention 1 - f_normalize(phi) (1 - rho), clamped (Eq. 9); each operation
// rounded on its own, phi entering as its float32 value.
__device__ __forceinline__ float dynamic_retention(double phi, float rho, const DevParams& p) {
#pragma clang fp contract(off)
  const double phi32 = static_cast<double>(static_cast<float>(phi));
  const double lo = static_cast<double>(p.phi_lo), hi = static_cast<double>(p.phi_hi);
  const double f = fmin(1.0, fmax(0.0, (phi32 - lo) / (hi - lo)));
  const double r = f * (1.0 - static_cast<double>(rho));
  const double keep = 1.0 - r;
  double ret = fmin(static_cast<double>(p.ratio_max), fmax(static_cast<double>(p.ratio_min), keep));
  if (!(ret == ret)) ret = static_cast<double>(p.ratio_max);
  return static_cast<float>(ret);
}

}  // namespace rtp
