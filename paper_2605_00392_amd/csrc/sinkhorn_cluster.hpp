// Sinkhorn (Appendix C) for images with more kept rows than one workgroup's
// registers hold (tiled pages pruned harder than most, the page sizes of other OCR
// models): the kernel matrix stays on chip for all T iterations, spread over a small
// cluster of workgroups.
//
// With at most 128 pruned tokens a cluster is G <= 8 workgroups; workgroup `rank` holds rows 448 rank .. 448 rank +
// 447 of the kept x pruned kernel matrix as fp32 in its registers (the 448 x 128
// shape of the one-workgroup kernel: 512 threads as 32 row slots x 16 column slots,
// 14 x 8 entries per thread, widened at each use; all sums and both scalings fp64).
// (Strips of 224 rows, 7 x 8 entries per thread, while eight of them cover the image: half the
// arithmetic per workgroup and iteration for the same exchange.)
// An iteration is one pass over a workgroup's rows - a row's x as soon as its sum is
// known, then its share of every column sum - followed by the only exchange there
// is: each workgroup publishes its partial sums (columns, and the sum of its x) and
// adds all the workgroups' partials in rank order, which gives all of them the same
// y bit for bit.  So the matrix is read from memory once per call instead of once
// per iteration, and an iteration costs a few microseconds of exchange instead of
// two kernel launches.
//
// Images with more than 128 pruned tokens take other strips: 144 rows x 576 columns
// (the 1083-token pages of which 560 are kept: four workgroups) or 80 rows x 960
// columns (the 2137-token pages: sixteen workgroups, half an XCD), a wave per row slot
// with its 64 lanes across the columns.  A slot has as many workgroups as the largest
// image of the launch needs (the host knows it under a fixed retention), so that more
// slots share the chip.
//
// The exchange.  The workgroups of all slots are resident together: the kernel is
// launched with one workgroup per compute unit and no more (each needs a CU's whole
// register file), and a slot works through its share of the image list with all its
// workgroups in step.  A slot's workgroups have linear ids of one residue modulo
// eight, so they share an XCD and its L2.  Sums travel as device-scope atomics with
// relaxed ordering, and a sum's place holds a "not yet" pattern until the sum is
// there: a reader polls the places it reads, so an iteration needs neither an arrival
// counter nor a barrier across workgroups (with them it took 3.5 to 4.3 us more per
// iteration; with device-scope fences, whose cache write-backs queue up behind each
// other, 6 to 17 us).  The places are in four buffers used in turn; sinkhorn_cluster_image
// says why the buffer two iterations back can be given its "not yet" again.  Between
// images, and before the first, all of a slot's workgroups put "not yet" into all
// their places and meet at an arrival counter (a workgroup waits until its stores
// have been acknowledged before it arrives: a workgroup-scope release alone does not
// wait for that).  Every wait is bounded: a workgroup that has polled `spin_limit`
// times in vain sets the give-up word, on which all workgroups leave, and
// RTP_DEV_SYNC_TIMEOUT in the status word.
#pragma once
#include "common.hpp"
#include "sinkhorn_team.hpp"
#include "sinkhorn_dual.hpp"

namespace rtp {

constexpr int kClusterMaxGroups = 16;                      // workgroups per cluster slot, at most
constexpr int kClusterDefaultGroups = 8;                   // when the host cannot bound the images' sizes
constexpr int kClusterThreads = 512;
using ClusterShape = TeamWideA;                            // 448 rows x 128 columns per workgroup
using ClusterShapeHalf = TeamShape<8, 4, 7, 8>;            // 224 rows x 128 columns per workgroup
using ClusterShapeWide = TeamStripWide;                    // 144 rows x 576 columns per workgroup
using ClusterShapeWider = TeamStripWider;                  // 80 rows x 960 columns per workgroup
static_assert(8 * ClusterShape::kMaxM == kClusterRows && ClusterShape::kMaxR == kClusterCols &&
              8 * ClusterShapeHalf::kMaxM == kClusterHalfRows && ClusterShapeHalf::kMaxR == kClusterCols &&
              8 * ClusterShapeWide::kMaxM == kClusterWideRows && ClusterShapeWide::kMaxR == kClusterWideCols &&
              16 * ClusterShapeWider::kMaxM == kClusterWiderRows && ClusterShapeWider::kMaxR == kClusterWiderCols,
              "the shapes sinkhorn_variant assumes");
template <typename S> constexpr int cluster_part_of() { return S::TC * (S::CPT + 1); }   // values a workgroup publishes
constexpr int kClusterPart = cluster_part_of<ClusterShapeWider>();         // 1024 (640 and 144 for the others)
static_assert(cluster_part_of<ClusterShape>() <= kClusterPart && cluster_part_of<ClusterShapeWide>() <= kClusterPart &&
                  cluster_part_of<ClusterShapeHalf>() <= kClusterPart,
              "exchange buffers are sized for the widest shape");
// LDS of a cluster workgroup: the waves' partial column sums (reused for the pairing's
// candidates), their totals, the latest x per row, a flag
template <typename S> constexpr int cluster_lds_of() {
  return (S::W * S::TC * (S::CPT + 1) + S::TC * (S::CPT + 1) + S::TR * S::RPT) * 8 + 16;
}
constexpr int cluster_max(int a, int b) { return a > b ? a : b; }
constexpr int kClusterLdsBytes = cluster_max(cluster_lds_of<ClusterShapeWider>(),
                                             cluster_max(cluster_lds_of<ClusterShapeWide>(), cluster_lds_of<ClusterShape>()));
constexpr int kClusterMaxSlots = 64;                       // cluster slots of a launch (8 per XCD)
// synchronisation words, after the work lists: one arrival counter per slot, then the give-up word
constexpr int kClusterSyncWords = kClusterMaxSlots + 1;
static_assert(kClusterSyncWords == kWorkStreamWord, "the list builder zeroes these words (the next one is the sweep kernels')");
// exchange buffers: six per workgroup of the launch (slots x workgroups per slot <= one per compute
// unit: 256 at most, more than that many compute units are not put to use)
constexpr int kClusterMaxBlocks = 256;
constexpr int kClusterSumBufs = 4, kClusterKeyBufs = 2, kClusterBufs = kClusterSumBufs + kClusterKeyBufs;
constexpr size_t kClusterPartDoubles = static_cast<size_t>(kClusterMaxBlocks) * kClusterBufs * kClusterPart;
// what a partial sum's place holds until the sum has been published: no sum has this bit pattern (a NaN)
constexpr long long kClusterNotYet = -1;

struct ClusterArgs {
  SinkhornArgs S;
  const int32_t* work;      // work lists (kVariantCluster)
  int B;
  int32_t* sync;            // [kClusterSyncWords], zeroed by the kernel that built the lists
  double* part;             // [slots][6][groups_per_slot][kClusterPart] exchange buffers: four for the sums
                            // (by the slot's iteration count modulo four), two for the pairing keys (by the
                            // slot's image parity)
  int slots_per_xcd;        // launch: 8 XCDs x slots_per_xcd slots x groups_per_slot workgroups
  int groups_per_slot;      // at most kClusterMaxGroups
  int spin_limit;
  int32_t* status;
};

// Cluster-wide meeting of the `groups` workgroups of a slot.  `arrived` is the count the slot's
// counter must reach (every workgroup keeps the same running total).  False: gave up.
__device__ __forceinline__ bool cluster_meet(int32_t* counter, int32_t* gave_up, int arrived, int spin_limit,
                                             int32_t* status, int* s_flag) {
  // This thread's published values must have reached the L2 before anybody is told that the
  // workgroup has arrived.  A workgroup-scope release does not wait for stores to be acknowledged
  // (waves of a workgroup share their caches), so the store counter is waited for explicitly.
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int ok = 0;
    for (int spin = 0; spin < spin_limit; ++spin) {
      if (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= arrived) { ok = 1; break; }
      if (__hip_atomic_load(gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
      __builtin_amdgcn_s_sleep(2);
    }
    if (!ok) {
      __hip_atomic_store(gave_up, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      atomicOr(status, RTP_DEV_SYNC_TIMEOUT);
    }
    *s_flag = ok;
  }
  __syncthreads();
  return *s_flag != 0;
}

// The same wait without arriving: a workgroup of the slot that has no strip of the current image
// stays here until the image's workgroups have all been through its last meeting.  (If it went on
// to the slot's next image at once, its first arrival there would be counted into a meeting of the
// current image, which would then let a workgroup through before all its partners' sums are out.)
__device__ __forceinline__ bool cluster_wait(int32_t* counter, int32_t* gave_up, int arrived, int spin_limit,
                                             int32_t* status, int* s_flag) {
  __syncthreads();
  if (threadIdx.x == 0) {
    int ok = 0;
    for (int spin = 0; spin < spin_limit; ++spin) {
      if (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= arrived) { ok = 1; break; }
      if (__hip_atomic_load(gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
      __builtin_amdgcn_s_sleep(8);
    }
    if (!ok) {
      __hip_atomic_store(gave_up, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      atomicOr(status, RTP_DEV_SYNC_TIMEOUT);
    }
    *s_flag = ok;
  }
  __syncthreads();
  return *s_flag != 0;
}

// One image on the `groups` workgroups of a slot; this workgroup is `rank` < groups.  Every
// workgroup of the cluster takes the same path through the barriers.  `arrived` carries the
// slot's running arrival count.  False: a wait was given up, leave the kernel.
template <typename S>
__device__ __forceinline__ bool sinkhorn_cluster_image(const ClusterArgs& C, int b, int rank, int groups,
                                                       int32_t* counter, double* part, int& arrived, int seq,
                                                       int& gi, void* lds) {
  constexpr int TC = S::TC, TR = S::TR, RPT = S::RPT, CPT = S::CPT, T = S::T, LOG_TC = S::LOG_TC, W = S::W;
  constexpr int kPart = cluster_part_of<S>();               // (buffers are kClusterPart apart whatever the shape)
  const int per_slot = C.groups_per_slot;
  static_assert(T == kClusterThreads, "workgroup shape");
  const SinkhornArgs& A = C.S;
  const DevParams& p = A.p;
  const int tt = threadIdx.x, tw = tt >> 6, lane = tt & 63;
  const int lo = A.offsets[b];
  const int n = A.offsets[b + 1] - lo;
  const int m = min(max(A.keep[b], 0), n), r = n - m;        // (the list holds images with n > 0, r > 0 only)
  const long long po = A.plan_offsets[b];
  const float* __restrict__ Kg = k32_base(A.kmat, po);        // stored as fp32 (kKernelRowsF32)
  const int pitch = k32_pitch(r);
  float* __restrict__ plan_out = A.plan_out;
  int32_t* __restrict__ pair_out = A.pair_out;
  int32_t* gave_up = C.sync + kClusterMaxSlots;
  const int row_base = rank * S::kMaxM;                      // this workgroup's first row
  const int m_loc = min(max(m - row_base, 0), S::kMaxM);     // rows it holds (>= 1: groups = ceil(m / rows per strip))
  if (pair_out)
    for (int i = tt; i < m_loc; i += T) pair_out[lo + row_base + i] = row_base + i;

  const int cslot = tt & (TC - 1);
  const int rslot = tt >> LOG_TC;

  double (*xw)[TC][CPT + 1] = static_cast<double (*)[TC][CPT + 1]>(lds);                 // [W]
  double (*xtot)[CPT + 1] = reinterpret_cast<double (*)[CPT + 1]>(xw + W);               // [TC]
  double (*xs)[RPT] = reinterpret_cast<double (*)[RPT]>(xtot + TC);                      // [TR]
  int& s_flag = *reinterpret_cast<int*>(xs + TR);
  // the pairing's candidates, once the iterations are over, where the partial sums were
  float (*pv)[TC][CPT] = static_cast<float (*)[TC][CPT]>(lds);                           // [W]
  int (*pi)[TC][CPT] = reinterpret_cast<int (*)[TC][CPT]>(pv + W);                       // [W]
  static_assert(sizeof(float) * 2 * W * TC * CPT <= sizeof(double) * W * TC * (CPT + 1), "candidates fit the sums' area");

  // the matrix: unconditional loads from clamped positions, four rows at a time, narrowed
  // before the next four are requested
  float K[RPT][CPT];
#pragma unroll
  for (int a0 = 0; a0 < RPT; a0 += 4) {
    float v[4][CPT];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = row_base + min(rslot + TR * (a0 + u), m_loc - 1);
#pragma unroll
      for (int c = 0; c < CPT; ++c)
        if (a0 + u < RPT) v[u][c] = Kg[static_cast<long long>(i) * pitch + min(cslot + TC * c, r - 1)];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < CPT; ++c)
        if (a0 + u < RPT) {
          float k = (rslot + TR * (a0 + u) < m_loc && cslot + TC * c < r) ? v[u][c] : 0.f;
          forget_origin(k);
          K[a0 + u][c] = k;
        }
  }

  const double kz = exp((p.z - p.shift) / p.eps);
  double y[CPT];
  const double x_init = exp(p.shift / p.eps);      // T = 0 leaves u = 0
#pragma unroll
  for (int c = 0; c < CPT; ++c) y[c] = (cslot + TC * c < r) ? 1.0 : 0.0;
  double x_dust = x_init, y_dust = 1.0;
  double sum_y = static_cast<double>(r) + 1.0;
  if (cslot == 0) {
#pragma unroll
    for (int a = 0; a < RPT; ++a) xs[rslot][a] = (rslot + TR * a < m_loc) ? x_init : 0.0;   // what T = 0 leaves
  }

  for (int it = 0; it < p.iters; ++it) {
    double t[CPT + 1];
    const double row_dust = kz * y_dust;
#pragma unroll
    for (int c = 0; c <= CPT; ++c) t[c] = 0.0;
#pragma unroll
    for (int a = 0; a < RPT; ++a) {
      if (TR * a >= m_loc) {                 // no row of this pass exists (the same for every thread)
        xs[rslot][a] = 0.0;
        continue;
      }
      // (the widest shape widens a row's entries a second time for the column sums rather than
      // hold 15 widened values across the row's reduction: registers)
      constexpr bool kWidenTwice = CPT > 9;
      double kd[kWidenTwice ? 1 : CPT];
      double acc = 0.0;
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        forget_origin(K[a][c]);
        const double k = static_cast<double>(K[a][c]);
        if constexpr (!kWidenTwice) kd[c] = k;
        acc = fma(k, y[c], acc);
      }
      acc = group_sum<LOG_TC>(acc);
      const double xa = (rslot + TR * a < m_loc) ? rcp64(acc + row_dust) : 0.0;
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        if constexpr (kWidenTwice) {
          forget_origin(K[a][c]);
          t[c] = fma(static_cast<double>(K[a][c]), xa, t[c]);
        } else {
          t[c] = fma(kd[c], xa, t[c]);
        }
      }
      t[CPT] += xa;
      xs[rslot][a] = xa;
      if (a % 2 == 1) __builtin_amdgcn_sched_barrier(0);
    }
    x_dust = static_cast<double>(r) * rcp64(kz * sum_y);
    // this workgroup's column sums: over the row slots of a wave by lane exchanges, over its waves in LDS
#pragma unroll
    for (int c = 0; c <= CPT; ++c) t[c] = cross_sum<LOG_TC>(t[c]);
    if (lane < TC) {
#pragma unroll
      for (int c = 0; c <= CPT; ++c) xw[tw][lane][c] = t[c];
    }
    int& seen_all = (&s_flag)[1 + (it & 1)];           // (two words in turn: the next write of one is a whole iteration away)
    if (tt == 0) seen_all = 1;
    __syncthreads();
    // ... published; every workgroup then adds all the workgroups' sums in rank order.  A sum's
    // place holds kClusterNotYet until the sum is there, so the readers need no word that says
    // "all are out" and no barrier: each polls the places it reads.  Four buffers in turn, by the
    // slot's iteration count: a workgroup that publishes iteration i has seen everybody's sums of
    // iteration i - 1, whose owners had by then finished reading iteration i - 2, so the buffer of
    // i - 2 (= i + 2 modulo four) is free and gets its "not yet" back now; that store is
    // acknowledged (the wait below, one iteration later) before the sums of iteration i + 1 go
    // out, and nobody looks at the buffer of i + 2 before having seen those.
    __builtin_amdgcn_s_waitcnt(0);
    {
      double* mine = part + ((gi & 3) * per_slot + rank) * kClusterPart;
      long long* ahead = reinterpret_cast<long long*>(part + (((gi + 2) & 3) * per_slot + rank) * kClusterPart);
      for (int e = tt; e < kPart; e += T) {
        const int cs = e / (CPT + 1), c = e - cs * (CPT + 1);
        double acc = 0.0;
#pragma unroll
        for (int w = 0; w < W; ++w) acc += xw[w][cs][c];
        __hip_atomic_store(ahead + e, kClusterNotYet, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(mine + e, acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    bool seen = true;
    for (int e = tt; e < kPart; e += T) {
      const int cs = e / (CPT + 1), c = e - cs * (CPT + 1);
      const double* all = part + (gi & 3) * per_slot * kClusterPart + e;
      // all workgroups' values requested together (from a clamped position past the last), added in rank order
      constexpr int kGroups = S::kMaxM >= 144 ? 8 : kClusterMaxGroups;   // as many as the shape's images can have
      double v[kGroups];
      for (int spin = 0;; ++spin) {
        bool ready = true;
#pragma unroll
        for (int g = 0; g < kGroups; ++g)
          v[g] = __hip_atomic_load(all + min(g, groups - 1) * kClusterPart, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int g = 0; g < kGroups; ++g) ready = ready && __double_as_longlong(v[g]) != kClusterNotYet;
        if (ready) break;
        if (spin >= C.spin_limit ||
            ((spin & 63) == 63 && __hip_atomic_load(gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
          seen = false;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
      double acc = 0.0;
#pragma unroll
      for (int g = 0; g < kGroups; ++g) acc += g < groups ? v[g] : 0.0;
      // (the column's reciprocal here, once per workgroup, instead of once per row slot)
      if (c < CPT) acc = (cs + TC * c < r) ? rcp64(acc + kz * x_dust) : 0.0;
      xtot[cs][c] = acc;
    }
    if (!seen) seen_all = 0;
    ++gi;
    __syncthreads();
    if (!seen_all) {                                   // a wait was given up (here or elsewhere): everybody leaves
      if (tt == 0) {
        __hip_atomic_store(gave_up, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        atomicOr(C.status, RTP_DEV_SYNC_TIMEOUT);
      }
      return false;
    }
#pragma unroll
    for (int c = 0; c <= CPT; ++c) t[c] = xtot[cslot][c];
    double ly = 0.0;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      y[c] = t[c];
      ly += y[c];
    }
    y_dust = static_cast<double>(m) * rcp64(kz * (t[CPT] + x_dust));
    ly = group_sum<LOG_TC>(ly);
    sum_y = ly + y_dust;
  }
  __syncthreads();                                     // xs as the last pass left it (or as set up, T = 0)

  // ---- plan and this workgroup's best partner per column ----
  float bv[CPT];
  int bi[CPT];
#pragma unroll
  for (int c = 0; c < CPT; ++c) { bv[c] = -1.f; bi[c] = 0x7fffffff; }
  float* P = plan_out ? plan_out + po : nullptr;
  int rslot_p = rslot, cslot_p = cslot;
  forget_origin(rslot_p);
  forget_origin(cslot_p);
#pragma unroll
  for (int a = 0; a < RPT; ++a) {
    const int il = rslot_p + TR * a;
    const double xa = xs[rslot][a];
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int j = cslot_p + TC * c;
      if (il < m_loc && j < r) {
        const float v = static_cast<float>(xa * static_cast<double>(K[a][c]) * y[c]);
        if (P) P[static_cast<long long>(row_base + il) * r + j] = v;
        if (v > bv[c]) { bv[c] = v; bi[c] = row_base + il; }
      }
    }
  }
  // each workgroup's best per column goes out as a key (value bits, then the lower row), like
  // the sums; after one more meeting the first workgroup picks the cluster's best and sets it
  // against the dustbin row.  (The cluster meets here even when no pairing is asked for: it
  // keeps a fast workgroup's next image out of the buffers a slow one is still reading.)
  long long* mine = reinterpret_cast<long long*>(part + ((kClusterSumBufs + (seq & 1)) * per_slot + rank) * kClusterPart);
  if (pair_out) {
#pragma unroll
    for (int mask = TC; mask < kWave; mask <<= 1)
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const float ov = __shfl_xor(bv[c], mask, kWave);
        const int oi = __shfl_xor(bi[c], mask, kWave);
        if (ov > bv[c] || (ov == bv[c] && oi < bi[c])) { bv[c] = ov; bi[c] = oi; }
      }
    if (lane < TC) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) { pv[tw][lane][c] = bv[c]; pi[tw][lane][c] = bi[c]; }
    }
    __syncthreads();
    if (tt < TC) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
#pragma unroll
        for (int w = 1; w < W; ++w) {
          const float ov = pv[w][tt][c];
          const int oi = pi[w][tt][c];
          if (ov > bv[c] || (ov == bv[c] && oi < bi[c])) { bv[c] = ov; bi[c] = oi; }
        }
        // plan entries are >= 0, so their bit patterns order like their values; "no row" (-1) is below all
        const long long key = (static_cast<long long>(__float_as_int(bv[c])) << 32) | static_cast<unsigned>(0x7fffffff - bi[c]);
        __hip_atomic_store(mine + tt * CPT + c, key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  arrived += groups;
  if (!cluster_meet(counter, gave_up, arrived, C.spin_limit, C.status, &s_flag)) return false;
  if (pair_out && rank == 0 && tt < TC) {
    const long long* all = reinterpret_cast<const long long*>(part + (kClusterSumBufs + (seq & 1)) * per_slot * kClusterPart);
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int j = cslot + TC * c;
      if (j < r) {
        long long best = __hip_atomic_load(all + tt * CPT + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int g = 1; g < groups; ++g) {
          const long long k = __hip_atomic_load(all + g * kClusterPart + tt * CPT + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          best = k > best ? k : best;
        }
        const float v = __int_as_float(static_cast<int>(best >> 32));
        const int i = 0x7fffffff - static_cast<int>(best);
        const float dust = static_cast<float>(x_dust * kz * y[c]);
        pair_out[lo + m + j] = dust > v ? -1 : i;
      }
    }
  }
  return true;
}

// "Not yet" into this workgroup's places of the slot's four buffers of sums, then a meeting of
// all the slot's workgroups: after it no place of the slot holds an old sum.
__device__ __forceinline__ bool cluster_clear(const ClusterArgs& C, int rank, int32_t* counter, double* part,
                                              int& arrived, int* s_flag) {
  const int per_slot = C.groups_per_slot;
  for (int buf = 0; buf < kClusterSumBufs; ++buf) {
    long long* mine = reinterpret_cast<long long*>(part + (buf * per_slot + rank) * kClusterPart);
    for (int e = threadIdx.x; e < kClusterPart; e += kClusterThreads)
      __hip_atomic_store(mine + e, kClusterNotYet, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  arrived += per_slot;
  return cluster_meet(counter, C.sync + kClusterMaxSlots, arrived, C.spin_limit, C.status, s_flag);
}

// Workgroup `block` of the cluster part of the launch: 8 XCDs x slots_per_xcd slots x
// groups_per_slot workgroups; slot s takes images s, s + slots, ... of the list.  The slot's
// arrival counter runs on through all its meetings: one of all its workgroups before the first
// image (the buffers of sums cleared), one of an image's workgroups at the image's end (the
// pairing keys out; the others wait for it without arriving), one of all again before the next
// image (the buffers cleared again, also by those that had no strip: they may have one next).
__device__ __forceinline__ void sinkhorn_cluster_block(const ClusterArgs& C, int block, void* lds) {
  const int x = block & 7, local = block >> 3;
  const int per_slot = C.groups_per_slot;
  const int slot_in_xcd = local / per_slot, rank = local % per_slot;
  if (slot_in_xcd >= C.slots_per_xcd) return;
  const int slots = 8 * C.slots_per_xcd, slot = x * C.slots_per_xcd + slot_in_xcd;
  int32_t* counter = C.sync + slot;
  double* part = C.part + static_cast<size_t>(slot) * kClusterBufs * per_slot * kClusterPart;
  const SinkhornArgs& A = C.S;
  const int count = C.work[kVariantCluster];
  if (slot >= count) return;                           // (the same for all the slot's workgroups)
  int* flag = reinterpret_cast<int*>(static_cast<unsigned char*>(lds) + kClusterLdsBytes - 16);
  int arrived = 0, seq = 0, gi = 0;
  if (!cluster_clear(C, rank, counter, part, arrived, flag)) return;
  for (int k = slot; k < count; k += slots, ++seq) {
    const int b = C.work[kWorkLists + kVariantCluster * C.B + k];
    const int n = A.offsets[b + 1] - A.offsets[b];
    const int m = min(max(A.keep[b], 0), max(n, 0)), r = max(n, 0) - m;
    // (every workgroup of the slot takes the same decisions: they read the same words)
    if (m <= 0 || r <= 0 || sinkhorn_variant(m, r, A.p.mode) != kVariantCluster) continue;
    if (!plan_fits(A.plan_offsets[b], m, r, A.plan_cap)) continue;
    const int groups = cluster_groups(m, r);           // (at most per_slot: sinkhorn_variant has seen to it)
    const bool last = k + slots >= count;
    if (rank < groups) {
      const int shape = cluster_shape(m, r);
      const bool ok = shape == 0   ? sinkhorn_cluster_image<ClusterShapeHalf>(C, b, rank, groups, counter, part, arrived, seq, gi, lds)
                      : shape == 3 ? sinkhorn_cluster_image<ClusterShape>(C, b, rank, groups, counter, part, arrived, seq, gi, lds)
                      : shape == 1 ? sinkhorn_cluster_image<ClusterShapeWide>(C, b, rank, groups, counter, part, arrived, seq, gi, lds)
                                   : sinkhorn_cluster_image<ClusterShapeWider>(C, b, rank, groups, counter, part, arrived, seq, gi, lds);
      if (!ok) return;
    } else {
      arrived += groups;                               // what the image's meeting, which it stays out of, adds to the count
      gi += A.p.iters;
      if (last) return;                                // nothing to wait for: the CU is free for others
      if (!cluster_wait(counter, C.sync + kClusterMaxSlots, arrived, C.spin_limit, C.status, flag)) return;
    }
    if (!last && !cluster_clear(C, rank, counter, part, arrived, flag)) return;
  }
}

// The Sinkhorn work of a batch with large images that one launch can hold beside
// k_sinkhorn_regs: first the cluster workgroups (`cluster_blocks` of them, one per
// compute unit of the slots in use; lowest ids, so they are handed out first and are
// resident together whatever follows), then the tall shapes, one image per
// workgroup.  The two kinds of image are independent, so a few clustered images'
// barrier-bound iterations run beside the tall ones instead of after them.
__global__ __launch_bounds__(kClusterThreads) void k_sinkhorn_large(ClusterArgs C, int cluster_blocks) {
  static_assert(kClusterThreads == kDualThreads, "one workgroup shape for both parts");
  if (C.status[0]) return;
  __shared__ __align__(16) unsigned char cluster_lds[kClusterLdsBytes];
  const int blk = blockIdx.x;
  if (blk < cluster_blocks) sinkhorn_cluster_block(C, blk, cluster_lds);
  else sinkhorn_tall_block(C.S, C.work, C.B, blk - cluster_blocks);
}

}  // namespace rtp
