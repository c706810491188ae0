// C ABI of the RTPrune operator: argument checks, workspace layout and kernel
// launch sequences.  Every entry point only validates on the host and enqueues
// on the caller's stream; see include/rtprune.h for the contract.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <mutex>
#include <string>
#include <type_traits>
#include <vector>

#include "rtprune.h"
#include "common.hpp"
#include "stage1.hpp"
#include "stage2_general.hpp"
#include "sinkhorn_team.hpp"
#include "sinkhorn_dual.hpp"
#include "sinkhorn_sweep.hpp"
#include "sinkhorn_cluster.hpp"
#include "scores_mfma.hpp"
#include "scores_tiled.hpp"
#include "merge_lds.hpp"
#include "merge_tiled.hpp"
#include "merge_mfma.hpp"
#include "density.hpp"
#include "splice.hpp"

using namespace rtp;

namespace {

constexpr size_t kAlign = 256;
constexpr int kNormMinWorkgroups = 1024;   // the norm pass keeps at least this many workgroups when it merges chunks
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Byte offsets of the workspace regions for a batch shape.
struct Layout {
  size_t status, norm64, score, partial, phi, ratio, keep, out_off, plan_off, sel, work, kmat, plan, total;
  size_t sw_x, sw_y, sw_colpart, sw_xpart, sw_ysum, sw_ydust, sw_bestv, sw_besti;   // sweep Sinkhorn state
  size_t cluster_part;   // exchange buffers of the multi-workgroup Sinkhorn kernel
  int chunks_per_image, chunks_per_part, parts_per_image;
  int sweep;            // the batch may hold images beyond the register-resident Sinkhorn shapes
  long long plan_cap;   // entries available in kmat / plan
  long long plan_stride;   // entries per token of an image's slot when the slots are not packed (plan_slot)
  long long strip_cap;  // entries available in the per-strip arrays
};

// `rmax`: an upper bound on any image's pruned set (max_tokens when nothing is known).
Layout make_layout(int B, long long total, int max_tokens, int D, int rmax) {
  Layout L;
  size_t at = 0;
  auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes); return o; };
  L.chunks_per_image = (max_tokens + kNormRowsPerChunk - 1) / kNormRowsPerChunk;
  if (L.chunks_per_image < 1) L.chunks_per_image = 1;
  // A workgroup of the norm pass takes several chunks when the batch has images
  // enough to fill the chip without splitting them: fewer partial vectors to
  // write and to add up afterwards.
  const long long all_chunks = static_cast<long long>(B) * L.chunks_per_image;
  L.chunks_per_part = static_cast<int>(std::min<long long>(L.chunks_per_image, std::max<long long>(1, all_chunks / kNormMinWorkgroups)));
  L.parts_per_image = (L.chunks_per_image + L.chunks_per_part - 1) / L.chunks_per_part;
  // M_b R_b <= N_b^2 / 4 <= N_b ceil(max_tokens / 4), and <= N_b rmax: a slot of N_b * plan_stride entries
  // holds any image's matrix, and total * plan_stride entries hold them all, packed or not
  L.plan_stride = std::min<long long>((max_tokens + 3) / 4, std::max(0, std::min(rmax, max_tokens)));
  L.plan_cap = total * L.plan_stride + 1;
  L.status = take(256);
  L.norm64 = take(sizeof(double) * total);
  L.score = take(sizeof(float) * total);
  L.partial = take(sizeof(double) * static_cast<size_t>(B) * L.chunks_per_image * (D + 1));
  L.phi = take(sizeof(float) * B);
  L.ratio = take(sizeof(float) * B);
  L.keep = take(sizeof(int32_t) * B);
  L.out_off = take(sizeof(int32_t) * (B + 1));
  L.plan_off = take(sizeof(long long) * (B + 1));
  L.sel = take(sizeof(int32_t) * total);
  L.work = take(sizeof(int32_t) * (kWorkLists * (1 + static_cast<size_t>(B)) + kWorkSyncWords));
  L.kmat = take(sizeof(double) * L.plan_cap);
  L.plan = take(sizeof(float) * L.plan_cap);
  // more than 512 tokens: an image can have more kept tokens than any register shape holds
  L.sweep = max_tokens > 512 ? 1 : 0;
  L.strip_cap = L.plan_cap / kSweepRows + total + 1;
  if (L.sweep) {
    L.sw_x = take(sizeof(double) * total);
    L.sw_y = take(sizeof(double) * total);
    L.sw_colpart = take(sizeof(double) * L.strip_cap);
    L.sw_xpart = take(sizeof(double) * total);
    L.sw_ysum = take(sizeof(double) * 2 * total);
    L.sw_ydust = take(sizeof(double) * 2 * B);
    L.sw_bestv = take(sizeof(float) * L.strip_cap);
    L.sw_besti = take(sizeof(int32_t) * L.strip_cap);
    L.cluster_part = take(sizeof(double) * kClusterPartDoubles);
  } else {
    L.sw_x = L.sw_y = L.sw_colpart = L.sw_xpart = L.sw_ysum = L.sw_ydust = L.sw_bestv = L.sw_besti = 0;
    L.cluster_part = 0;
  }
  L.total = at;
  return L;
}

template <typename T>
inline T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

int check_batch(const rtprune_batch* in) {
  if (!in) return RTP_EINVAL;
  if (in->B < 0 || in->total_tokens < 0 || in->max_tokens < 0 || in->D <= 0) return RTP_EINVAL;
  if (in->dtype != RTP_F32 && in->dtype != RTP_BF16) return RTP_EINVAL;
  if (!in->offsets) return RTP_EINVAL;
  if (in->total_tokens > 0 && !in->tokens) return RTP_EINVAL;
  if (reinterpret_cast<uintptr_t>(in->tokens) % 16 != 0) return RTP_EINVAL;
  if (in->D % 4 != 0 || (in->dtype == RTP_BF16 && in->D % 8 != 0)) return RTP_EUNSUPPORTED;
  if (in->D > kMaxD || in->max_tokens > kMaxTokens || in->B > kMaxImages) return RTP_EUNSUPPORTED;
  if (in->total_tokens > 0x7fffffffLL) return RTP_EUNSUPPORTED;
  if (in->total_tokens > static_cast<long long>(in->B) * in->max_tokens) return RTP_EINVAL;
  return RTP_OK;
}

int check_params(const rtprune_params* p, DevParams* d) {
  if (!p) return RTP_EINVAL;
  if (!(p->eps > 0.f) || p->iters < 0) return RTP_EINVAL;
  if (p->metric != RTP_METRIC_L2NORM && p->metric != RTP_METRIC_VARIANCE) return RTP_EINVAL;
  if (p->mid_merge_min_images < 0) return RTP_EINVAL;
  if (!std::isfinite(p->z) || !std::isfinite(p->alpha) || !std::isfinite(p->eps)) return RTP_EINVAL;
  if (p->dynamic) {
    if (!(p->ratio_min > 0.f) || !(p->ratio_max <= 1.f) || !(p->ratio_min <= p->ratio_max)) return RTP_EINVAL;
    if (!(p->phi_hi > p->phi_lo)) return RTP_EINVAL;
  } else {
    if (!(p->ratio > 0.f) || !(p->ratio <= 1.f)) return RTP_EINVAL;
  }
  const double z = p->z, eps = p->eps;
  const double hi = z > 1.0 ? z : 1.0, lo = z < -1.0 ? z : -1.0;
  if ((hi - lo) / eps > 600.0) return RTP_EUNSUPPORTED;
  d->z = z;
  d->alpha = p->alpha;
  d->eps = eps;
  d->shift = hi;
  d->ratio = p->ratio;
  d->ratio_min = p->ratio_min;
  d->ratio_max = p->ratio_max;
  d->phi_lo = p->phi_lo;
  d->phi_hi = p->phi_hi;
  d->iters = p->iters;
  d->dynamic = p->dynamic ? 1 : 0;
  d->metric = p->metric;
  d->mid_min = p->mid_merge_min_images;
  d->mode = 0;                                   // set per batch by launch_ot
  d->k32 = (hi - lo) / eps <= 80.0 ? 1 : 0;      // exp(-80) is a normal fp32 number
  return RTP_OK;
}

// Largest pruned set an image of at most `max_tokens` tokens can have under these
// parameters: R = N - ceil(retention N - 1e-3) <= (1 - retention) N + 1, with the fixed
// retention or the lower clamp of the dynamic one.
int params_pruned_bound(const DevParams& p, int max_tokens) {
  const double keep = p.dynamic ? static_cast<double>(p.ratio_min) : static_cast<double>(p.ratio);
  return std::min(std::max(max_tokens - 1, 0), static_cast<int>((1.0 - keep) * max_tokens) + 1);
}
constexpr int kPrunedAny = 1 << 30;   // make_layout: no bound on the pruned sets

int check_ws(const rtprune_batch* in, int rmax, void* ws, size_t ws_bytes, Layout* L) {
  *L = make_layout(in->B, in->total_tokens, in->max_tokens, in->D, rmax);
  if (!ws || reinterpret_cast<uintptr_t>(ws) % kAlign != 0 || ws_bytes < L->total) return RTP_EWORKSPACE;
  return RTP_OK;
}

inline int launched() { return hipGetLastError() == hipSuccess ? RTP_OK : RTP_EHIP; }

// Compute units of the current device (256 on MI355X; that value if the query fails).
int compute_units() {
  static std::atomic<int> cached{0};   // one kind of device per process; a repeated query gives the same value
  if (cached.load(std::memory_order_relaxed) > 0) return cached.load(std::memory_order_relaxed);
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
    n = 256;
  cached.store(n, std::memory_order_relaxed);
  return n;
}

#define RTP_TRY(expr)            \
  do {                           \
    const int rc_ = (expr);      \
    if (rc_ != RTP_OK) return rc_; \
  } while (0)

// ---- per-kernel timing (measurement aid) ------------------------------------
// When enabled, each kernel launch is bracketed by two HIP events recorded on
// the launch stream; rtprune_profile_summary() turns them into per-kernel totals.

enum KernelId { KID_PREPARE, KID_NORMS, KID_SELECT, KID_SCAN, KID_SCORES, KID_CLASSIFY, KID_SINKHORN_REGS, KID_SINKHORN_C32, KID_SINKHORN_TALL, KID_SINKHORN, KID_MERGE, KID_DENSITY_PREPARE, KID_DENSITY_SOBEL, KID_DENSITY_FINISH, KID_SPLICE, KID_COUNT };
const char* const kKernelNames[KID_COUNT] = {"k_prepare", "k_norms", "k_select", "k_scan",
                                             "k_scores", "k_classify", "k_sinkhorn_regs", "k_sinkhorn_c32", "k_sinkhorn_tall", "k_sinkhorn",
                                             "k_merge", "k_density_prepare", "k_density_sobel",
                                             "k_density_finish", "k_splice"};
struct ProfRec { int kid; hipEvent_t start, stop; };
struct ProfState {
  std::mutex mu;               // guards `recs`
  std::atomic<bool> on{false};
  std::atomic<int> only{-1};   // >= 0: record this kernel id alone (rtprune_profile_only)
  std::vector<ProfRec> recs;
} g_prof;

struct ProfScope {
  int kid;
  hipStream_t s;
  hipEvent_t start = nullptr, stop = nullptr;
  bool live = false;
  ProfScope(int kid_, hipStream_t s_) : kid(kid_), s(s_) {
    const int only = g_prof.only.load(std::memory_order_relaxed);
    if (!g_prof.on.load(std::memory_order_relaxed) || (only >= 0 && only != kid)) return;
    if (hipEventCreate(&start) != hipSuccess || hipEventCreate(&stop) != hipSuccess) return;
    live = hipEventRecord(start, s) == hipSuccess;
  }
  ~ProfScope() {
    if (!live) return;
    (void)hipEventRecord(stop, s);
    std::lock_guard<std::mutex> g(g_prof.mu);
    g_prof.recs.push_back({kid, start, stop});
  }
};

// ---- launch helpers -------------------------------------------------------

int launch_prepare(const rtprune_batch* in, int32_t* status, hipStream_t s) {
  ProfScope prof(KID_PREPARE, s);
  hipLaunchKernelGGL(k_prepare, dim3(1), dim3(256), 0, s, in->offsets, in->B,
                     static_cast<long long>(in->total_tokens), in->max_tokens, status);
  return launched();
}

// `validate`: the kernel's first workgroup validates the ragged layout and writes the
// status word (the fused calls); otherwise k_prepare has written it.
template <typename T>
int launch_norms_t(const rtprune_batch* in, int dynamic, int metric, const Layout& L, void* ws,
                   float* norms_out, bool validate, hipStream_t s) {
  const dim3 grid(L.parts_per_image, in->B), block(kNormThreads);
  const T* tok = static_cast<const T*>(in->tokens);
  double* sq = at<double>(ws, L.norm64);
  float* sc = at<float>(ws, L.score);
  double* part = at<double>(ws, L.partial);
  const NormCheck st{validate ? 1 : 0, in->B, static_cast<long long>(in->total_tokens), in->max_tokens,
                     at<int32_t>(ws, L.status)};
  ProfScope prof(KID_NORMS, s);
  // groups of four elements per row; the lean variants need every k but the last
  // to be fully populated
  const int ngroups = in->D / 4;
#define RTP_LAUNCH_NORMS(KMAX, KFULL)                                                                    \
  do {                                                                                                   \
    if (metric == RTP_METRIC_VARIANCE)                                                                   \
      hipLaunchKernelGGL((k_norms<T, KMAX, KFULL, true>), grid, block, 0, s, tok, in->offsets, in->D,    \
                         dynamic, sq, sc, norms_out, part, L.parts_per_image, L.chunks_per_part, st);    \
    else                                                                                                 \
      hipLaunchKernelGGL((k_norms<T, KMAX, KFULL, false>), grid, block, 0, s, tok, in->offsets, in->D,   \
                         dynamic, sq, sc, norms_out, part, L.parts_per_image, L.chunks_per_part, st);    \
  } while (0)
  if (in->D <= 1280) {
    if (ngroups == 64 * 5) RTP_LAUNCH_NORMS(5, 5);
    else if (ngroups >= 64 * 4) RTP_LAUNCH_NORMS(5, 4);
    else RTP_LAUNCH_NORMS(5, 0);
  } else {
    RTP_LAUNCH_NORMS(16, 0);
  }
#undef RTP_LAUNCH_NORMS
  return launched();
}

int launch_norms(const rtprune_batch* in, int dynamic, int metric, const Layout& L, void* ws,
                 float* norms_out, hipStream_t s, bool validate = false) {
  if (in->B == 0 || in->total_tokens == 0) return RTP_OK;
  return in->dtype == RTP_BF16 ? launch_norms_t<bf16_t>(in, dynamic, metric, L, ws, norms_out, validate, s)
                               : launch_norms_t<float>(in, dynamic, metric, L, ws, norms_out, validate, s);
}

// The norm pass can stand in for k_prepare when it runs at all.
bool norms_validate(const rtprune_batch* in) { return in->B > 0 && in->total_tokens > 0; }

int launch_select(const rtprune_batch* in, const DevParams& p, const float* density,
                  const int32_t* keep_in, int do_select, const Layout& L, void* ws, float* phi,
                  float* ratio, int32_t* keep_out, int32_t* sel, hipStream_t s) {
  if (in->B == 0) return RTP_OK;
  ProfScope prof(KID_SELECT, s);
  const size_t lds = 9 * static_cast<size_t>((in->max_tokens + 1) & ~1);   // 8-byte key + flag per token
  const SelectArgs A{in->offsets, in->D, p, density, keep_in, at<float>(ws, L.score), at<double>(ws, L.partial),
                     L.parts_per_image, L.chunks_per_part * kNormRowsPerChunk, do_select, in->max_tokens,
                     phi, ratio, keep_out, sel};
  const int32_t* st = at<int32_t>(ws, L.status);
  // long images: the rank counting is quadratic in the token count, so the workgroup grows with it
  if (in->max_tokens > 2048)
    hipLaunchKernelGGL(k_select<1024>, dim3(in->B), dim3(1024), lds, s, A, st);
  else
    hipLaunchKernelGGL(k_select<256>, dim3(in->B), dim3(256), lds, s, A, st);
  return launched();
}

// Cluster slots per XCD of the multi-workgroup Sinkhorn kernel on this device: a slot is
// `groups` compute units of one XCD (eight XCDs assumed; 0: too few compute units).
int cluster_slots_per_xcd(int groups) {
  const int per_xcd = std::min(compute_units(), kClusterMaxBlocks) / 8;   // (the exchange buffers are sized for 256 workgroups)
  return std::min(kClusterMaxSlots / 8, per_xcd / std::max(groups, 1));
}

// RTPRUNE_SWEEP_STREAM_16THS = 0 .. 16 fixes the share of strips that the sweep kernels read with
// streaming loads (for tests: a batch whose matrices exceed the memory-side cache takes seconds
// of oracle time); unset, the share follows from the matrices' size.
int sweep_stream_override() {
  if (const char* e = std::getenv("RTPRUNE_SWEEP_STREAM_16THS")) {
    const long v = std::strtol(e, nullptr, 10);
    if (v >= 0 && v <= 16) return static_cast<int>(v);
  }
  return -1;
}

// Polls a workgroup of that kernel spends on one wait before it gives up (each a few hundred
// cycles: the default is seconds).  RTPRUNE_SYNC_SPIN_LIMIT overrides it, for tests of the
// give-up path.
int cluster_spin_limit() {
  if (const char* e = std::getenv("RTPRUNE_SYNC_SPIN_LIMIT")) {
    const long v = std::strtol(e, nullptr, 10);
    if (v > 0 && v < 0x7fffffffL) return static_cast<int>(v);
  }
  return 20 * 1000 * 1000;
}

// Which Sinkhorn kernels a call on this batch launches, and whether the sweep
// kernels' matrices are stored in fp32 (only batches that may hold images beyond
// the 512-row register shapes have any).
void set_sinkhorn_mode(DevParams& p, const Layout& L, const rtprune_batch* in) {
  const int f32 = p.k32 ? kModeF32 : 0;   // exp's range fits fp32: registers may hold the matrix as fp32
  // the multi-workgroup kernel that keeps a matrix on chip runs one workgroup per compute
  // unit, in clusters of eight per XCD
  // Under a fixed retention the largest image the batch can hold bounds the others' kept and
  // pruned counts; when the multi-workgroup kernel can take it, a cluster slot needs no more
  // workgroups than that image does (more slots then share the chip), and no image is beyond the
  // on-chip kernels.
  const int m_top = p.dynamic ? 0 : kept_count(p.ratio, in->max_tokens), r_top = in->max_tokens - m_top;
  const bool top_fits = !p.dynamic && m_top > 0 && cluster_fits(m_top, r_top);
  const int groups = top_fits ? cluster_groups(m_top, std::max(r_top, 1)) : kClusterDefaultGroups;
  const int cluster = (L.sweep && f32 && cluster_slots_per_xcd(groups) > 0) ? (kModeCluster | (groups << kModeGroupsShift)) : 0;
  // The streaming kernels cost two launches per iteration whether or not an image needs them,
  // and only the device knows the sizes, so they are issued when the batch's shape and the
  // parameters say that images beyond the on-chip kernels are to be expected: a fixed
  // retention under which the longest image fits no cluster shape, or images with more kept
  // rows than a cluster holds.  Under a dynamic retention (pages prune 2 to 12 % of their
  // tokens; the clamp at 0.6 is a bound, not the rule) they are not: an image that does end
  // up beyond the on-chip kernels takes the one-workgroup general kernel, which is right and
  // slow.  Only the batch's shape and the parameters enter, so that the staged calls choose
  // the same kernels as the fused ones.
  const bool beyond = p.dynamic ? in->max_tokens - 1 > kClusterRows : !top_fits;
  const int sweep = (L.sweep && (!cluster || beyond)) ? kModeSweep : 0;
  p.k32 = p.k32 && sweep;                 // the sweep kernels' copy in memory is fp32
  p.mode = (L.sweep ? kModeLarge : 0) | f32 | cluster | sweep;
}

// `work` non-null: the same launch also builds the Sinkhorn work lists.
int launch_scan(const rtprune_batch* in, const int32_t* keep, int32_t* out_off, long long* plan_off,
                const int32_t* status, hipStream_t s, int32_t* work = nullptr, int mode = 0) {
  ProfScope prof(KID_SCAN, s);
  if (work)
    hipLaunchKernelGGL(k_scan_classify, dim3(1), dim3(256), 0, s, in->offsets, keep, in->B, out_off, plan_off, work,
                       mode, status);
  else
    hipLaunchKernelGGL(k_scan, dim3(1), dim3(256), 0, s, in->offsets, keep, in->B, out_off, plan_off, status);
  return launched();
}

// Workgroups of the list forms of the tiled kernels: eight per CU, or all tiles if fewer.
unsigned tiled_list_blocks(int tiles, int B) {
  const long long all = static_cast<long long>(tiles) * B;
  return static_cast<unsigned>(std::min<long long>(all, 8LL * compute_units()));
}

// Largest pruned set any image of the call can have.  `hint` >= 0: the caller's
// bound (fixed retention); kPrunedFromClamp: the kept counts come from this
// call's dynamic ratio, whose clamp bounds them; kPrunedUnknown: the kept counts
// are the user's.
constexpr int kPrunedFromClamp = -1, kPrunedUnknown = -2;
int pruned_bound(const rtprune_batch* in, const DevParams& p, int hint) {
  int rmax = in->max_tokens - 1;
  if (hint >= 0) rmax = std::min(rmax, hint);
  else if (hint == kPrunedFromClamp && p.dynamic)
    rmax = std::min(rmax, static_cast<int>((1.0 - static_cast<double>(p.ratio_min)) * in->max_tokens) + 1);
  return rmax;
}

template <typename T>
int launch_scores_t(const rtprune_batch* in, const DevParams& p, const int32_t* sel,
                    const int32_t* keep, const long long* plan_off, const Layout& L, void* ws,
                    double* scores_out, int max_pruned_hint, const int32_t* work, const ScanJob& job,
                    hipStream_t s) {
  const T* tok = static_cast<const T*>(in->tokens);
  const double* sq = at<double>(ws, L.norm64);
  double* kmat = at<double>(ws, L.kmat);
  const int32_t* st = at<int32_t>(ws, L.status);
  ProfScope prof(KID_SCORES, s);
  if constexpr (std::is_same<T, bf16_t>::value) {
    // matrix-core path: its 32-term fp32 partial sums leave an error of about
    // 6e-8 sqrt(32 / D) of the cosine, which the pairing's near-tie band covers from
    // D = 1024 up; narrower tokens take the fp64 vector kernel.
    if (in->D % 128 == 0 && in->D >= kMfmaMinWidth) {
      // matrix-core path (an image's workgroups on one XCD: B rounded up to eight)
      const int tiles_s = (in->max_tokens + kScoreRows - 1) / kScoreRows;
      const unsigned blocks = static_cast<unsigned>(tiles_s) * ((in->B + 7) / 8 * 8) + (job.on ? 1u : 0u);
      hipLaunchKernelGGL(k_scores_mfma, dim3(blocks), dim3(kScoreThreads), 0, s, tok, in->offsets, in->B, in->D, sel,
                         keep, plan_off, sq, p, kmat, L.plan_cap, scores_out, tiles_s, job, st);
      RTP_TRY(launched());
      // images with many pruned tokens: the LDS-tiled kernel.  Largest pruned set
      // the call can produce: the caller's bound, else what the retention clamp allows
      const int rmax = pruned_bound(in, p, max_pruned_hint);
      if (rmax > kTiledMinPruned) {
        // kept rows an image can have: what the fixed retention leaves of the longest one when
        // this call selected under it (then it also passed a bound), else all of its tokens
        const int mmax = (max_pruned_hint >= 0 && !p.dynamic) ? kept_count(p.ratio, in->max_tokens) : in->max_tokens;
        const int tiles_m = (std::max(mmax, 1) + kTileRows - 1) / kTileRows;
        const int tiles_n = (rmax + kTileCols - 1) / kTileCols;
        const int tiles = tiles_m * tiles_n;
        const ScoresTiledArgs TA{tok, in->offsets, in->D, sel, keep, plan_off, sq, p, kmat, L.plan_cap, scores_out,
                                 tiles_n};
        // pruned sets known to be large (fixed retention): a workgroup per tile and
        // image; sizes decided on the device, or barely above the threshold: a fixed
        // number of workgroups over the work list
        if (max_pruned_hint >= 2 * kTiledMinPruned)
          hipLaunchKernelGGL(k_scores_tiled, dim3(tiles, in->B), dim3(kTiledThreads), 0, s, TA, st);
        else
          hipLaunchKernelGGL(k_scores_tiled_list, dim3(tiled_list_blocks(tiles, in->B)), dim3(kTiledThreads), 0, s,
                             TA, tiles, work, in->B, st);
      }
      return launched();
    }
  }
  const int tiles = (in->max_tokens + kScoreRowsPerBlock - 1) / kScoreRowsPerBlock;
  const dim3 grid(tiles, in->B), block(256);
  if (in->D <= 1280)
    hipLaunchKernelGGL((k_scores<T, 5>), grid, block, 0, s, tok, in->offsets, in->D, sel, keep, plan_off,
                       sq, p, kmat, L.plan_cap, scores_out, st);
  else
    hipLaunchKernelGGL((k_scores<T, 16>), grid, block, 0, s, tok, in->offsets, in->D, sel, keep,
                       plan_off, sq, p, kmat, L.plan_cap, scores_out, st);
  return launched();
}

// Whether the score pass of a batch runs on the matrix-core kernel, whose launch can
// carry the fused calls' scan job.
bool scores_on_matrix_cores(const rtprune_batch* in) {
  return in->dtype == RTP_BF16 && in->D % 128 == 0 && in->D >= kMfmaMinWidth && in->B > 0 && in->total_tokens > 0;
}

int launch_ot(const rtprune_batch* in, const DevParams& p_in, const int32_t* sel, const int32_t* keep,
              const long long* plan_off, const Layout& L, void* ws, double* scores_out, float* plan,
              int32_t* pair, int max_pruned_hint, bool classified, hipStream_t s,
              const ScanJob& job = ScanJob{0, nullptr, nullptr, nullptr, 0, 0}) {
  if (in->B == 0 || in->total_tokens == 0) return RTP_OK;
  DevParams p = p_in;
  set_sinkhorn_mode(p, L, in);
  const double* kmat = at<double>(ws, L.kmat);
  const int32_t* st = at<int32_t>(ws, L.status);
  int32_t* work = at<int32_t>(ws, L.work);
  if (!classified) {
    ProfScope prof(KID_CLASSIFY, s);
    hipLaunchKernelGGL(k_classify, dim3(1), dim3(256), 0, s, in->offsets, keep, in->B, work, p.mode, st);
    RTP_TRY(launched());
  }
  RTP_TRY(in->dtype == RTP_BF16
              ? launch_scores_t<bf16_t>(in, p, sel, keep, plan_off, L, ws, scores_out, max_pruned_hint, work, job, s)
              : launch_scores_t<float>(in, p, sel, keep, plan_off, L, ws, scores_out, max_pruned_hint, work, job, s));
  SinkhornArgs A{in->offsets, keep, plan_off, p, kmat, L.plan_cap, plan, pair};
  {
    ProfScope prof(KID_SINKHORN_REGS, s);
    hipLaunchKernelGGL(k_sinkhorn_regs, dim3(in->B), dim3(kDualThreads), 0, s, A, work, in->B, compute_units(), st);
  }
  // (its images have 48 to 64 pruned tokens: smaller sets go to the shapes above, and in
  // batches with large images the sweep kernels take them)
  if ((p.mode & kModeF32) && !(p.mode & kModeLarge) && pruned_bound(in, p, max_pruned_hint) >= 48) {
    ProfScope prof(KID_SINKHORN_C32, s);
    hipLaunchKernelGGL(k_sinkhorn_c32, dim3(std::min(in->B, 2 * compute_units())), dim3(kDualThreads), 0, s, A, work,
                       in->B, st);
  }
  if (p.mode & kModeLarge) {
    // the tall one-workgroup shapes and, before them in the same launch, the clusters of
    // workgroups (one per compute unit of the slots in use: all resident together, which their
    // waits rely on)
    const int groups = std::max(mode_cluster_groups(p.mode), 1);
    const int spx = (p.mode & kModeCluster) ? cluster_slots_per_xcd(groups) : 0;
    const int cluster_blocks = 8 * spx * groups;
    const ClusterArgs CA{A, work, in->B, work + kWorkLists * (1 + static_cast<size_t>(in->B)),
                         at<double>(ws, L.cluster_part), spx, groups, cluster_spin_limit(), at<int32_t>(ws, L.status)};
    ProfScope prof(KID_SINKHORN_TALL, s);
    hipLaunchKernelGGL(k_sinkhorn_large, dim3(cluster_blocks + in->B), dim3(kClusterThreads), 0, s, CA, cluster_blocks);
  }
  RTP_TRY(launched());
  // The general kernel takes what no shape above does.  With the fp32-held shapes
  // in use and at most 512 tokens per image those cover every image with up to 224
  // pruned tokens (64 / 128 / 192 / 224 pruned against 512 / 448 / 384 / 320 kept),
  // so a call that cannot produce a larger pruned set has nothing left for it.
  const bool all_in_registers = (p.mode & kModeF32) && !(p.mode & kModeLarge) &&
                                pruned_bound(in, p, max_pruned_hint) <= TeamWideC::kMaxR;
  ProfScope prof(KID_SINKHORN, s);   // (with the sweep launches below)
  if (!all_in_registers) {
    hipLaunchKernelGGL(k_sinkhorn, dim3(in->B), dim3(1024), 0, s, in->offsets, keep, plan_off, p, kmat,
                       L.plan_cap, plan, pair, 1, p.mode, st);
    RTP_TRY(launched());
  }
  if (p.mode & kModeSweep) {
    // large images: two launches per iteration over all of them, then plan and pairing
    SweepArgs SA{in->offsets, keep, plan_off, work, in->B, p, kmat, L.plan_cap,
                at<double>(ws, L.sw_x), at<double>(ws, L.sw_y), at<void>(ws, L.sw_colpart),
                at<double>(ws, L.sw_xpart), at<double>(ws, L.sw_ysum), at<double>(ws, L.sw_ydust),
                at<float>(ws, L.sw_bestv), at<int32_t>(ws, L.sw_besti), in->total_tokens, plan, pair,
                sweep_stream_override()};
    const int strips = (in->max_tokens + kSweepRows - 1) / kSweepRows;
    const int cols = (std::min(in->max_tokens, kSweepMaxR) + kSweepCols - 1) / kSweepCols;
    const dim3 grows(strips, in->B), gcols(cols, in->B);
    hipLaunchKernelGGL(k_sweep_init, gcols, dim3(kSweepColThreads), 0, s, SA, st);
    // columns per thread: enough for the largest pruned set the batch can hold
    const int rmax = std::min(pruned_bound(in, p, max_pruned_hint), kSweepMaxR);
    const int ch = (std::max(rmax, 1) + kSweepThreads - 1) / kSweepThreads;
    auto rows = [&](auto final_tag, int parity) {
      constexpr bool kFinal = decltype(final_tag)::value;
#define RTP_SWEEP_ROWS(KT, CH) \
  hipLaunchKernelGGL((k_sweep_rows<kFinal, KT, CH>), grows, dim3(kSweepThreads), 0, s, SA, parity, st)
      if (p.k32) {
        if (ch <= 1) RTP_SWEEP_ROWS(float, 1);
        else if (ch == 2) RTP_SWEEP_ROWS(float, 2);
        else if (ch == 3) RTP_SWEEP_ROWS(float, 3);
        else RTP_SWEEP_ROWS(float, 4);
      } else {
        if (ch <= 1) RTP_SWEEP_ROWS(double, 1);
        else if (ch == 2) RTP_SWEEP_ROWS(double, 2);
        else if (ch == 3) RTP_SWEEP_ROWS(double, 3);
        else RTP_SWEEP_ROWS(double, 4);
      }
#undef RTP_SWEEP_ROWS
    };
    for (int it = 0; it < p.iters; ++it) {
      rows(std::false_type{}, it & 1);
      if (p.k32) hipLaunchKernelGGL((k_sweep_cols<false, float>), gcols, dim3(kSweepColThreads), 0, s, SA, it & 1, 0, st);
      else hipLaunchKernelGGL((k_sweep_cols<false, double>), gcols, dim3(kSweepColThreads), 0, s, SA, it & 1, 0, st);
    }
    rows(std::true_type{}, 0);
    hipLaunchKernelGGL((k_sweep_cols<true, double>), gcols, dim3(kSweepColThreads), 0, s, SA,
                       p.iters > 0 ? (p.iters - 1) & 1 : 0, p.iters == 0 ? 1 : 0, st);
  }
  return launched();
}

template <typename T>
int launch_merge_t(const rtprune_batch* in, const DevParams& p, const int32_t* sel,
                   const int32_t* keep, const int32_t* out_off, const float* plan,
                   const long long* plan_off, void* out, int max_pruned_hint, const int32_t* status,
                   const int32_t* work, hipStream_t s) {
  const int tiles = (in->max_tokens + kMergeRowsPerBlock - 1) / kMergeRowsPerBlock;
  const dim3 grid(tiles, in->B), block(256);
  const T* tok = static_cast<const T*>(in->tokens);
  const float alpha = static_cast<float>(p.alpha);
  // images with many pruned tokens go to the matrix-core kernel (bf16, width a
  // multiple of 128) when the call can produce any
  const int rmax = pruned_bound(in, p, max_pruned_hint);
  const bool tiled = std::is_same<T, bf16_t>::value && in->D % 128 == 0 && rmax > kTiledMinPruned;
  // and those with a middling number to the one that streams the kept rows, when the
  // call has the work lists (a workspace)
  const bool mid = std::is_same<T, bf16_t>::value && in->D % kMergeMidFeatures == 0 && rmax > kMergeMidMin && work && status;
  // (when the device counts enough of them to fill the chip: four row tiles per compute unit)
  const int tiles_mid = (in->max_tokens + kMergeMidBlockRows - 1) / kMergeMidBlockRows;
  const int mid_min = p.mid_min > 0 ? p.mid_min : std::max(1, (4 * compute_units() + tiles_mid - 1) / tiles_mid);
  const MergeSkip skip{(tiled ? kSkipTiled : 0) | (mid ? kSkipMid : 0), mid ? work + kListMid : nullptr, mid_min};
  ProfScope prof(KID_MERGE, s);
  if (in->D <= 1280) {
    const dim3 g2((in->max_tokens + kMergeBlockRows - 1) / kMergeBlockRows, in->B);
    if (in->D == 1280)
      hipLaunchKernelGGL((k_merge_lds<T, 5, true>), g2, block, 0, s, tok, in->offsets, in->D, sel, keep,
                         out_off, plan, plan_off, alpha, in->max_tokens, skip, static_cast<T*>(out), status);
    else
      hipLaunchKernelGGL((k_merge_lds<T, 5, false>), g2, block, 0, s, tok, in->offsets, in->D, sel, keep,
                         out_off, plan, plan_off, alpha, in->max_tokens, skip, static_cast<T*>(out), status);
  } else if (in->D <= 1024) {
    hipLaunchKernelGGL((k_merge<T, 1>), grid, block, 0, s, tok, in->offsets, in->D, sel, keep, out_off,
                       plan, plan_off, alpha, in->max_tokens, skip, static_cast<T*>(out), status);
  } else if (in->D <= 2048) {
    hipLaunchKernelGGL((k_merge<T, 2>), grid, block, 0, s, tok, in->offsets, in->D, sel, keep, out_off,
                       plan, plan_off, alpha, in->max_tokens, skip, static_cast<T*>(out), status);
  } else {
    hipLaunchKernelGGL((k_merge<T, 4>), grid, block, 0, s, tok, in->offsets, in->D, sel, keep, out_off,
                       plan, plan_off, alpha, in->max_tokens, skip, static_cast<T*>(out), status);
  }
  RTP_TRY(launched());
  if constexpr (std::is_same<T, bf16_t>::value) {
    const int tiles_ti = (in->max_tokens + kMergeTileRows - 1) / kMergeTileRows;
    const int tiles_td = in->D / kMergeTileCols;
    const MergeTiledArgs TA{tok, in->offsets, in->D, sel, keep, out_off, plan, plan_off, alpha, in->max_tokens,
                            tiles_td, static_cast<bf16_t*>(out)};
    // pruned sets known to be large (fixed retention), or no work list: a workgroup per
    // tile and image for the tiled kernel; else its list form shares a launch with the
    // middling sets' kernel
    const bool tiled_grid = tiled && (max_pruned_hint >= 2 * kTiledMinPruned || !work || !status);
    if (tiled_grid)
      hipLaunchKernelGGL(k_merge_tiled, dim3(tiles_ti * tiles_td, in->B), dim3(kMergeTiledThreads), 0, s, TA, status);
    const bool tiled_list = tiled && !tiled_grid;
    if (tiled_list || mid) {
      const MergeMidArgs MA{tok, in->offsets, in->D, sel, keep, out_off, plan, plan_off, alpha, in->max_tokens,
                            static_cast<bf16_t*>(out)};
      const int tiles_t = tiled_list ? tiles_ti * tiles_td : 0, tiles_m = mid ? tiles_mid : 0;
      const dim3 gl((tiled_list_blocks(std::max(tiles_t, tiles_m), in->B) + 7) / 8 * 8);
      if (in->D % (2 * kMergeMidFeatures) == 0)
        hipLaunchKernelGGL(k_merge_lists<2>, gl, dim3(kMergeMidThreads), 0, s, TA, tiles_t, MA, tiles_m, work, in->B,
                           mid_min, status);
      else
        hipLaunchKernelGGL(k_merge_lists<1>, gl, dim3(kMergeMidThreads), 0, s, TA, tiles_t, MA, tiles_m, work, in->B,
                           mid_min, status);
    }
  }
  return launched();
}

int launch_merge(const rtprune_batch* in, const DevParams& p, const int32_t* sel, const int32_t* keep,
                 const int32_t* out_off, const float* plan, const long long* plan_off, void* out,
                 int max_pruned_hint, const int32_t* status, const int32_t* work, hipStream_t s) {
  if (in->B == 0 || in->total_tokens == 0) return RTP_OK;
  return in->dtype == RTP_BF16
             ? launch_merge_t<bf16_t>(in, p, sel, keep, out_off, plan, plan_off, out, max_pruned_hint, status, work, s)
             : launch_merge_t<float>(in, p, sel, keep, out_off, plan, plan_off, out, max_pruned_hint, status, work, s);
}

// Stage 1 of the fused calls: [layout check ->] norms (+ phi sums) -> ratio, kept count,
// selection [-> prefix sums and work lists].  Two launches in the common case (the
// norm pass checks the layout; the sums and lists are left to the score pass as `job`);
// the separate kernels otherwise.  `text`: the splice call's text spans, checked
// between the norm pass and the selection.
int launch_stage1(const rtprune_batch* in, const DevParams& p, int mode, const float* density, float* ratio,
                  int32_t* keep, int32_t* sel, int32_t* out_offsets, long long* plan_off, const Layout& L,
                  void* ws, hipStream_t s, ScanJob* job, const TextSpans* text = nullptr) {
  int32_t* status = at<int32_t>(ws, L.status);
  int32_t* work = at<int32_t>(ws, L.work);
  const bool validate = norms_validate(in);
  if (!validate) RTP_TRY(launch_prepare(in, status, s));
  RTP_TRY(launch_norms(in, p.dynamic, p.metric, L, ws, nullptr, s, validate));
  if (text && in->B > 0) {
    hipLaunchKernelGGL(k_splice_check, dim3(1), dim3(256), 0, s, *text, in->B, status);
    RTP_TRY(launched());
  }
  RTP_TRY(launch_select(in, p, density, nullptr, 1, L, ws, nullptr, ratio, keep, sel, s));
  // the prefix sums and work lists: by an extra workgroup of the score pass when that runs
  // on the matrix-core kernel (`job`), else by a launch of their own
  if (scores_on_matrix_cores(in)) {
    *job = ScanJob{1, out_offsets, plan_off, work, mode, L.plan_stride};
    return RTP_OK;
  }
  return launch_scan(in, keep, out_offsets, plan_off, status, s, work, mode);
}

}  // namespace

// ---- exported entry points --------------------------------------------------

extern "C" const char* rtprune_status_string(int status) {
  switch (status) {
    case RTP_OK: return "RTP_OK";
    case RTP_EINVAL: return "RTP_EINVAL: invalid argument";
    case RTP_EUNSUPPORTED: return "RTP_EUNSUPPORTED: outside the supported limits";
    case RTP_EWORKSPACE: return "RTP_EWORKSPACE: workspace missing, unaligned or too small";
    case RTP_EHIP: return "RTP_EHIP: kernel launch failed";
    default: return "unknown status";
  }
}

// Plain 16-byte-per-lane copy: the reference point hardware counters are scaled by.
__global__ __launch_bounds__(256) void k_copy(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                              size_t n16) {
  for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n16;
       i += static_cast<size_t>(gridDim.x) * blockDim.x)
    dst[i] = src[i];
}

extern "C" int rtprune_copy_bytes(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes % 16 != 0) return RTP_EINVAL;
  if (reinterpret_cast<uintptr_t>(dst) % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0) return RTP_EINVAL;
  if (bytes == 0) return RTP_OK;
  const size_t n16 = bytes / 16;
  const size_t want = (n16 + 255) / 256;
  const unsigned grid = static_cast<unsigned>(want < 16384 ? want : 16384);
  hipLaunchKernelGGL(k_copy, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16);
  return launched();
}

extern "C" int rtprune_profile_enable(int on) {
  std::lock_guard<std::mutex> g(g_prof.mu);
  for (ProfRec& r : g_prof.recs) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_prof.recs.clear();
  g_prof.on = on != 0;
  return RTP_OK;
}

extern "C" int rtprune_profile_only(const char* kernel) {
  int kid = -1;
  if (kernel && kernel[0]) {
    for (int k = 0; k < KID_COUNT; ++k)
      if (std::strcmp(kernel, kKernelNames[k]) == 0) kid = k;
    if (kid < 0) return RTP_EINVAL;
  }
  std::lock_guard<std::mutex> g(g_prof.mu);
  g_prof.only = kid;
  return RTP_OK;
}

extern "C" int rtprune_profile_summary(char* buf, size_t cap) {
  if (!buf || cap == 0) return RTP_EINVAL;
  std::lock_guard<std::mutex> g(g_prof.mu);
  double total_ms[KID_COUNT] = {0};
  long long launches[KID_COUNT] = {0};
  for (ProfRec& r : g_prof.recs) {
    if (hipEventSynchronize(r.stop) != hipSuccess) return RTP_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return RTP_EHIP;
    total_ms[r.kid] += ms;
    launches[r.kid] += 1;
  }
  std::string out = "[";
  bool first = true;
  for (int k = 0; k < KID_COUNT; ++k) {
    if (!launches[k]) continue;
    char line[160];
    std::snprintf(line, sizeof(line), "%s{\"kernel\": \"%s\", \"launches\": %lld, \"total_ms\": %.6f}",
                  first ? "" : ", ", kKernelNames[k], launches[k], total_ms[k]);
    out += line;
    first = false;
  }
  out += "]";
  if (out.size() + 1 > cap) return RTP_EINVAL;
  std::memcpy(buf, out.c_str(), out.size() + 1);
  return RTP_OK;
}

extern "C" int rtprune_workspace_bytes(int32_t B, int64_t total_tokens, int32_t max_tokens, int32_t D,
                                       int32_t dtype, const rtprune_params* params, size_t* bytes) {
  if (!bytes) return RTP_EINVAL;
  int rmax = kPrunedAny;
  if (params) {
    DevParams p;
    RTP_TRY(check_params(params, &p));
    rmax = params_pruned_bound(p, max_tokens);
  }
  rtprune_batch in;
  std::memset(&in, 0, sizeof(in));
  int32_t dummy = 0;
  in.tokens = nullptr;
  in.offsets = &dummy;
  in.total_tokens = 0;
  in.B = B;
  in.D = D;
  in.max_tokens = max_tokens;
  in.dtype = dtype;
  RTP_TRY(check_batch(&in));
  if (total_tokens < 0 || total_tokens > 0x7fffffffLL) return RTP_EINVAL;
  if (total_tokens > static_cast<long long>(B) * max_tokens) return RTP_EINVAL;
  *bytes = make_layout(B, total_tokens, max_tokens, D, rmax).total;
  return RTP_OK;
}

namespace {
struct DensityLayout { size_t status, counts, total; int patches_max; long long ncounts; };
DensityLayout make_density_layout(int B, int max_h, int max_w, int patch_h, int patch_w) {
  DensityLayout L;
  L.patches_max = (max_h / patch_h) * (max_w / patch_w);
  L.ncounts = static_cast<long long>(B) * L.patches_max;
  L.status = 0;
  L.counts = 256;
  L.total = align_up(256 + sizeof(int32_t) * static_cast<size_t>(L.ncounts));
  return L;
}
int check_density_shape(int B, int max_h, int max_w, int patch_h, int patch_w) {
  if (B < 0 || max_h < 0 || max_w < 0 || patch_h <= 0 || patch_w <= 0) return RTP_EINVAL;
  if (max_h > 65536 || max_w > 65536) return RTP_EUNSUPPORTED;
  if (max_w > 0 && density_strip_rows(patch_h, max_w) == 0) return RTP_EUNSUPPORTED;
  return RTP_OK;
}
}  // namespace

extern "C" int rtprune_text_density_workspace_bytes(int32_t B, int32_t max_height, int32_t max_width,
                                                    int32_t patch_h, int32_t patch_w, size_t* bytes) {
  if (!bytes) return RTP_EINVAL;
  RTP_TRY(check_density_shape(B, max_height, max_width, patch_h, patch_w));
  *bytes = make_density_layout(B, max_height, max_width, patch_h, patch_w).total;
  return RTP_OK;
}

extern "C" int rtprune_text_density(const uint8_t* pixels, const int64_t* pixel_offsets,
                                    const int32_t* heights, const int32_t* widths, int32_t B,
                                    int32_t max_height, int32_t max_width, int32_t patch_h,
                                    int32_t patch_w, float tau, float* density, float* patch_density,
                                    const int32_t* patch_offsets, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  RTP_TRY(check_density_shape(B, max_height, max_width, patch_h, patch_w));
  if (!pixel_offsets || !heights || !widths || !density) return RTP_EINVAL;
  if (patch_density && !patch_offsets) return RTP_EINVAL;
  if (!(tau == tau)) return RTP_EINVAL;
  const DensityLayout L = make_density_layout(B, max_height, max_width, patch_h, patch_w);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 || workspace_bytes < L.total)
    return RTP_EWORKSPACE;
  if (B == 0) return RTP_OK;
  if (!pixels && max_height > 0 && max_width > 0) return RTP_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* status = at<int32_t>(workspace, L.status);
  int32_t* counts = at<int32_t>(workspace, L.counts);
  const long long* poff = reinterpret_cast<const long long*>(pixel_offsets);
  {
    ProfScope prof(KID_DENSITY_PREPARE, s);
    const long long want = (L.ncounts + 255) / 256;
    const unsigned grid = static_cast<unsigned>(want < 1 ? 1 : (want > 4096 ? 4096 : want));
    hipLaunchKernelGGL(k_density_prepare, dim3(grid), dim3(256), 0, s, poff, heights, widths, B, max_height,
                       max_width, patch_h, patch_w, counts, L.ncounts, status);
  }
  RTP_TRY(launched());
  if (max_height > 0 && max_width > 0) {
    const int strip = density_strip_rows(patch_h, max_width);
    const size_t lds = sizeof(int) * (static_cast<size_t>(strip + 2) * (max_width + 2) + max_width / patch_w + 1);
    // G >= tau on [0, 1] intensities <=> G_x^2 + G_y^2 >= (tau * 255 * 1000)^2 in luma units of 1/1000
    const double t = static_cast<double>(tau) * 255000.0;
    const double thr2 = t * t;
    const float lo = static_cast<float>(thr2 * (1.0 - 2e-6)), hi = static_cast<float>(thr2 * (1.0 + 2e-6));
    ProfScope prof(KID_DENSITY_SOBEL, s);
    if (patch_w % 4 == 0) {
      // register-window kernel: a wave per 248-column band and patch row
      const int bands = ((max_width / 4) + kDensityBand - 1) / kDensityBand;
      hipLaunchKernelGGL(k_density_rows, dim3((bands + 3) / 4, (max_height + patch_h - 1) / patch_h, B), dim3(256), 0,
                         s, pixels, poff, heights, widths, patch_h, patch_w, L.patches_max, lo, hi, thr2, counts,
                         status);
    } else {
      hipLaunchKernelGGL(k_density_sobel, dim3((max_height + strip - 1) / strip, B), dim3(kDensityThreads), lds, s,
                         pixels, poff, heights, widths, strip, patch_h, patch_w, L.patches_max, lo, hi, thr2,
                         counts, status);
    }
    RTP_TRY(launched());
  }
  ProfScope prof(KID_DENSITY_FINISH, s);
  hipLaunchKernelGGL(k_density_finish, dim3(B), dim3(256), 0, s, heights, widths, patch_h, patch_w,
                     L.patches_max, counts, density, patch_density, patch_offsets, status);
  return launched();
}

extern "C" int rtprune_dynamic_ratio(const rtprune_batch* in, const float* density,
                                     const rtprune_params* params, float* phi, float* ratio,
                                     int32_t* keep_counts, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  RTP_TRY(check_batch(in));
  DevParams p;
  RTP_TRY(check_params(params, &p));
  if (!params->dynamic) {
    // the dynamic formula is what this call computes; the clamp fields must be valid
    rtprune_params q = *params;
    q.dynamic = 1;
    RTP_TRY(check_params(&q, &p));
  }
  if (!density || !keep_counts) return RTP_EINVAL;
  Layout L;
  RTP_TRY(check_ws(in, 0 /* no kernel matrix or plan */, workspace, workspace_bytes, &L));
  hipStream_t s = static_cast<hipStream_t>(stream);
  RTP_TRY(launch_prepare(in, at<int32_t>(workspace, L.status), s));
  RTP_TRY(launch_norms(in, 1, p.metric, L, workspace, nullptr, s));
  return launch_select(in, p, density, nullptr, 0, L, workspace, phi, ratio, keep_counts, nullptr, s);
}

extern "C" int rtprune_norms_topk(const rtprune_batch* in, const int32_t* keep_counts_in,
                                  const rtprune_params* params, float* norms, int32_t* sel_idx,
                                  int32_t* keep_counts, int32_t* out_offsets, int64_t* plan_offsets,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  RTP_TRY(check_batch(in));
  DevParams p;
  rtprune_params q;
  if (!params) return RTP_EINVAL;
  q = *params;
  q.dynamic = 0;
  if (keep_counts_in) q.ratio = 1.f;   // unused
  RTP_TRY(check_params(&q, &p));
  if (!sel_idx || !keep_counts || !out_offsets || !plan_offsets) return RTP_EINVAL;
  Layout L;
  RTP_TRY(check_ws(in, 0 /* no kernel matrix or plan */, workspace, workspace_bytes, &L));
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* status = at<int32_t>(workspace, L.status);
  RTP_TRY(launch_prepare(in, status, s));
  RTP_TRY(launch_norms(in, 0, p.metric, L, workspace, norms, s));
  RTP_TRY(launch_select(in, p, nullptr, keep_counts_in, 1, L, workspace, nullptr, nullptr, keep_counts,
                        sel_idx, s));
  return launch_scan(in, keep_counts, out_offsets, reinterpret_cast<long long*>(plan_offsets), status, s);
}

extern "C" int rtprune_ot_pair(const rtprune_batch* in, const int32_t* sel_idx,
                               const int32_t* keep_counts, const int64_t* plan_offsets,
                               const rtprune_params* params, double* scores, float* plan,
                               int32_t* pair, void* workspace, size_t workspace_bytes, void* stream) {
  RTP_TRY(check_batch(in));
  DevParams p;
  RTP_TRY(check_params(params, &p));
  if (!sel_idx || !keep_counts || !plan_offsets) return RTP_EINVAL;
  Layout L;
  RTP_TRY(check_ws(in, kPrunedAny, workspace, workspace_bytes, &L));
  hipStream_t s = static_cast<hipStream_t>(stream);
  RTP_TRY(launch_prepare(in, at<int32_t>(workspace, L.status), s));
  // exact squared norms of every row (fp32 norms from stage 1 would cost 1e-7 on S)
  RTP_TRY(launch_norms(in, 0, RTP_METRIC_L2NORM, L, workspace, nullptr, s));
  // the kept counts live on the device: no host-side bound on the pruned sets
  return launch_ot(in, p, sel_idx, keep_counts, reinterpret_cast<const long long*>(plan_offsets), L,
                   workspace, scores, plan, pair, kPrunedUnknown, false, s);
}

extern "C" int rtprune_merge(const rtprune_batch* in, const int32_t* sel_idx,
                             const int32_t* keep_counts, const int32_t* out_offsets, const float* plan,
                             const int64_t* plan_offsets, const rtprune_params* params, void* out,
                             void* workspace, size_t workspace_bytes, void* stream) {
  RTP_TRY(check_batch(in));
  DevParams p;
  RTP_TRY(check_params(params, &p));
  if (!sel_idx || !keep_counts || !out_offsets || !plan || !plan_offsets || !out) return RTP_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const long long* plan_off = reinterpret_cast<const long long*>(plan_offsets);
  if (!workspace)   // the vector kernel, and the tiled one over a worst-case grid
    return launch_merge(in, p, sel_idx, keep_counts, out_offsets, plan, plan_off, out, kPrunedUnknown, nullptr,
                        nullptr, s);
  // with a workspace the images are sorted by pruned count first, as in the fused calls
  Layout L;
  RTP_TRY(check_ws(in, kPrunedAny, workspace, workspace_bytes, &L));
  int32_t* status = at<int32_t>(workspace, L.status);
  int32_t* work = at<int32_t>(workspace, L.work);
  RTP_TRY(launch_prepare(in, status, s));
  if (in->B > 0) {
    ProfScope prof(KID_CLASSIFY, s);
    hipLaunchKernelGGL(k_classify, dim3(1), dim3(256), 0, s, in->offsets, keep_counts, in->B, work, 0, status);
    RTP_TRY(launched());
  }
  return launch_merge(in, p, sel_idx, keep_counts, out_offsets, plan, plan_off, out, kPrunedUnknown, status, work, s);
}

extern "C" int rtprune_prune(const rtprune_batch* in, const float* density,
                             const rtprune_params* params, void* out, int32_t* out_offsets,
                             int32_t* keep_counts, int32_t* sel_idx, int32_t* pair, float* ratio,
                             void* workspace, size_t workspace_bytes, void* stream) {
  RTP_TRY(check_batch(in));
  DevParams p;
  RTP_TRY(check_params(params, &p));
  if (!out || !out_offsets) return RTP_EINVAL;
  if (p.dynamic && !density) return RTP_EINVAL;
  Layout L;
  RTP_TRY(check_ws(in, params_pruned_bound(p, in->max_tokens), workspace, workspace_bytes, &L));
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* status = at<int32_t>(workspace, L.status);
  int32_t* keep = keep_counts ? keep_counts : at<int32_t>(workspace, L.keep);
  int32_t* sel = sel_idx ? sel_idx : at<int32_t>(workspace, L.sel);
  long long* plan_off = at<long long>(workspace, L.plan_off);
  float* plan = at<float>(workspace, L.plan);
  DevParams pm = p;
  set_sinkhorn_mode(pm, L, in);
  ScanJob job{0, nullptr, nullptr, nullptr, 0, 0};
  RTP_TRY(launch_stage1(in, p, pm.mode, density, ratio, keep, sel, out_offsets, plan_off, L, workspace, s, &job));
  // fixed retention: R <= N - ceil(ratio N - 1e-3) <= (1 - ratio) N + 1 for every image
  const int max_pruned = p.dynamic ? kPrunedFromClamp
                                   : static_cast<int>((1.0 - static_cast<double>(p.ratio)) * in->max_tokens) + 1;
  RTP_TRY(launch_ot(in, p, sel, keep, plan_off, L, workspace, nullptr, plan, pair, max_pruned, true, s, job));
  return launch_merge(in, p, sel, keep, out_offsets, plan, plan_off, out, max_pruned, status,
                      at<int32_t>(workspace, L.work), s);
}

// ---- rtprune_prune without a caller's workspace --------------------------------
// The workspace of this variant is a fixed array in the library's device image (one
// copy per GPU, held until the process ends).  In host code the array's name only
// stands for the symbol; its device address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[RTPRUNE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once known

// The current device's copy of `scratch`.
int static_scratch(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RTP_EHIP;
  std::lock_guard<std::mutex> g(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RTP_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return RTP_OK;
}
}  // namespace

extern "C" int rtprune_prune_static(const rtprune_batch* in, const float* density,
                                    const rtprune_params* params, void* out, int32_t* out_offsets,
                                    int32_t* keep_counts, int32_t* sel_idx, int32_t* pair, float* ratio,
                                    void* stream) {
  // sizes first: a batch beyond the array is refused before anything touches the device
  RTP_TRY(check_batch(in));
  DevParams p;
  RTP_TRY(check_params(params, &p));
  const Layout L = make_layout(in->B, in->total_tokens, in->max_tokens, in->D, params_pruned_bound(p, in->max_tokens));
  if (L.total > static_cast<size_t>(RTPRUNE_STATIC_SCRATCH_BYTES)) return RTP_EWORKSPACE;
  void* ws = nullptr;
  RTP_TRY(static_scratch(&ws));
  // every kernel of the call writes what it later reads, so the array's old content
  // (the previous call's) needs no clearing
  return rtprune_prune(in, density, params, out, out_offsets, keep_counts, sel_idx, pair, ratio, ws,
                       static_cast<size_t>(RTPRUNE_STATIC_SCRATCH_BYTES), stream);
}

extern "C" int rtprune_prune_splice(const rtprune_batch* in, const float* density,
                                    const rtprune_params* params, const rtprune_text_spans* text,
                                    int32_t position_mode, void* seq, int64_t seq_capacity_rows,
                                    int32_t* seq_offsets, int32_t* position_ids, int32_t* keep_counts,
                                    int32_t* sel_idx, int32_t* pair, float* ratio, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  RTP_TRY(check_batch(in));
  DevParams p;
  RTP_TRY(check_params(params, &p));
  if (!seq || !seq_offsets || !text) return RTP_EINVAL;
  if (p.dynamic && !density) return RTP_EINVAL;
  if (position_mode != RTP_POSITIONS_CONSECUTIVE && position_mode != RTP_POSITIONS_ORIGINAL) return RTP_EINVAL;
  if (text->prefix_rows < 0 || text->suffix_rows < 0) return RTP_EINVAL;
  if ((text->prefix_rows > 0 && (!text->prefix || !text->prefix_offsets)) ||
      (text->suffix_rows > 0 && (!text->suffix || !text->suffix_offsets)))
    return RTP_EINVAL;
  if (reinterpret_cast<uintptr_t>(text->prefix) % 16 != 0 || reinterpret_cast<uintptr_t>(text->suffix) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(seq) % 16 != 0)
    return RTP_EINVAL;
  // every image keeps at most all of its tokens
  const long long need = text->prefix_rows + text->suffix_rows + in->total_tokens;
  if (seq_capacity_rows < need) return RTP_EINVAL;
  if (need > 0x7fffffffLL) return RTP_EUNSUPPORTED;
  if (static_cast<long long>(in->D) * (in->dtype == RTP_BF16 ? 2 : 4) % 16 != 0) return RTP_EUNSUPPORTED;
  Layout L;
  RTP_TRY(check_ws(in, params_pruned_bound(p, in->max_tokens), workspace, workspace_bytes, &L));
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* status = at<int32_t>(workspace, L.status);
  int32_t* keep = keep_counts ? keep_counts : at<int32_t>(workspace, L.keep);
  int32_t* sel = sel_idx ? sel_idx : at<int32_t>(workspace, L.sel);
  int32_t* visual_start = at<int32_t>(workspace, L.out_off);
  long long* plan_off = at<long long>(workspace, L.plan_off);
  float* plan = at<float>(workspace, L.plan);
  const TextSpans t{text->prefix, text->prefix_offsets, text->prefix_rows,
                    text->suffix, text->suffix_offsets, text->suffix_rows};
  // (the text offsets are checked after the norm pass has written the status word and
  // before the first kernel that writes to the caller's arrays)
  DevParams pm = p;
  set_sinkhorn_mode(pm, L, in);
  ScanJob job{0, nullptr, nullptr, nullptr, 0, 0};
  RTP_TRY(launch_stage1(in, p, pm.mode, density, ratio, keep, sel, nullptr, plan_off, L, workspace, s, &job, &t));
  hipLaunchKernelGGL(k_splice_scan, dim3(1), dim3(256), 0, s, t, keep, in->B, seq_offsets, visual_start, status);
  RTP_TRY(launched());
  const int max_pruned = p.dynamic ? kPrunedFromClamp
                                   : static_cast<int>((1.0 - static_cast<double>(p.ratio)) * in->max_tokens) + 1;
  RTP_TRY(launch_ot(in, p, sel, keep, plan_off, L, workspace, nullptr, plan, pair, max_pruned, true, s, job));
  // the merge writes image b's kept rows at visual_start[b], between its text spans
  RTP_TRY(launch_merge(in, p, sel, keep, visual_start, plan, plan_off, seq, max_pruned, status,
                       at<int32_t>(workspace, L.work), s));
  if (in->B == 0) return RTP_OK;
  ProfScope prof(KID_SPLICE, s);
  const dim3 grid(64, in->B);
  if (in->dtype == RTP_BF16)
    hipLaunchKernelGGL((k_splice_text<bf16_t>), grid, dim3(256), 0, s, t, in->offsets, keep, sel, in->D,
                       position_mode, seq_offsets, static_cast<bf16_t*>(seq), position_ids, status);
  else
    hipLaunchKernelGGL((k_splice_text<float>), grid, dim3(256), 0, s, t, in->offsets, keep, sel, in->D,
                       position_mode, seq_offsets, static_cast<float*>(seq), position_ids, status);
  return launched();
}
