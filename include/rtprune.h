/*
 * rtprune.h - C ABI of the RTPrune batched visual-token reduction operator
 * for AMD MI355X (gfx950).
 *
 * The operator is the training-free step RTPrune places between DeepSeek-OCR's
 * vision encoder and the language model's prefill (paper: Sec. 3.3, Algorithm 1):
 *
 *   stage 1  keep the M tokens of largest l2 norm (Eq. 1, M = N(1-r));
 *   stage 2  score kept x pruned pairs by cosine similarity (Eq. 3), add a
 *            dustbin row and column of score z (Eq. 4-5), run T log-domain
 *            Sinkhorn iterations (Appendix C) to get the transport plan P;
 *   merge    T_i <- T_i + alpha * sum_j P_ij T_j for every kept token (Eq. 6);
 *   ratio    optionally choose r per image from the mean pairwise cosine phi
 *            (Eq. 7) and a textual-density scalar rho: r = f(phi)(1-rho) (Eq. 9).
 *
 * Conventions common to every call
 * --------------------------------
 * - Every array pointer is a DEVICE pointer owned by the caller, unless marked
 *   "host".  The library never allocates, frees or synchronises; each call
 *   enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = the
 *   default stream) and returns at once.  Results are valid once the stream
 *   has reached the end of the call's work.
 * - A batch is ragged: image b owns token rows offsets[b] .. offsets[b+1]-1 of
 *   the packed row-major token matrix (row length D).  `offsets` is an int32
 *   exclusive prefix sum with B+1 entries, offsets[0] = 0,
 *   offsets[B] = total_tokens.  `total_tokens` and `max_tokens` (an upper
 *   bound on any image's token count) are host scalars the caller knows.
 * - Token indices in outputs are LOCAL to their image (0 .. N_b-1).
 * - "Retention" is 1 - r, the fraction of tokens kept.
 * - Return value: RTP_OK, or an error found on the host (bad pointer, size,
 *   dtype or parameter; workspace too small), in which case NOTHING has been
 *   enqueued.  Errors that only the device can see (offsets not monotone, an
 *   image longer than max_tokens, offsets[B] != total_tokens) make every kernel
 *   of the call skip its work, touch no output, and set a nonzero int32 at
 *   byte 0 of the workspace (see RTP_DEV_*).  No call crashes on bad data.
 * - Limits: 1 <= D <= 4096 and D % 4 == 0 (D % 8 == 0 for bf16);
 *   max_tokens <= 8192; B <= 65535 (an image is a row of the launch grids);
 *   (max(1,z) - min(-1,z)) / eps <= 600 (else RTP_EUNSUPPORTED).
 * - The operator's calls keep no state between calls and are thread-safe as long
 *   as concurrent calls use distinct workspaces (the measurement aids at the end
 *   of this header are process-wide switches; see there).
 */
#ifndef RTPRUNE_H
#define RTPRUNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rtp_status {
  RTP_OK = 0,
  RTP_EINVAL = 1,       /* NULL pointer, negative size, bad dtype or parameter */
  RTP_EUNSUPPORTED = 2, /* valid request outside the documented limits */
  RTP_EWORKSPACE = 3,   /* workspace pointer NULL/unaligned or too small */
  RTP_EHIP = 4          /* a kernel launch was rejected by the runtime */
} rtp_status;

typedef enum rtp_dtype {
  RTP_F32 = 0,          /* IEEE binary32 tokens in, binary32 merged tokens out */
  RTP_BF16 = 1          /* bfloat16 in and out (merge accumulates in fp32, one RNE) */
} rtp_dtype;

/* Device-side status word (int32 at byte 0 of the workspace), bit flags. */
enum {
  RTP_DEV_OK = 0,
  RTP_DEV_BAD_OFFSETS = 1,   /* offsets not monotone / offsets[0] != 0 / offsets[B] != total_tokens */
  RTP_DEV_IMAGE_TOO_LONG = 2, /* some image has more than max_tokens tokens */
  RTP_DEV_BAD_IMAGE = 4,      /* rtprune_text_density: a page's size is negative, above the stated
                                 maximum, not a multiple of the patch size, or overruns its pixel span */
  RTP_DEV_SYNC_TIMEOUT = 8    /* the Sinkhorn kernel that spreads a tall image over several workgroups gave
                                 up waiting for one of them (they must all be resident at once: only a GPU
                                 kept busy for seconds by other work can cause it); the images it serves
                                 - in batches with images above 512 tokens, those that no one-workgroup
                                 shape holds, with up to 128 pruned tokens and 3584 kept ones, up to
                                 576 and 1152, or up to 960 and 1280 - have no valid plan, pairing or
                                 merged rows in this call's outputs */
};

/* Two environment variables are read at each call, for tests only (they change no result):
 *   RTPRUNE_SYNC_SPIN_LIMIT      polls a workgroup of that kernel spends on one wait before it gives
 *                                up (default: 20 000 000, seconds); a value of 1 forces the give-up path
 *   RTPRUNE_SWEEP_STREAM_16THS   0 .. 16: how many of every 16 strips the streaming Sinkhorn kernels
 *                                read with non-temporal loads (default: worked out on the device from
 *                                the size of their matrices against the memory-side cache) */

/* Importance score of stage 1.  The method uses the l2 norm (Eq. 1); the
 * variance of a token's D feature values is the alternative the paper's
 * selection-metric ablation measures (Sec. 4.4, Table 7), taken here in its
 * population form sum_d (x_d - mean)^2 / D and accumulated in fp64 (mean first,
 * then the squared deviations).  Stage 2 is the same for both: cosines always
 * use the l2 norms. */
typedef enum rtp_metric { RTP_METRIC_L2NORM = 0, RTP_METRIC_VARIANCE = 1 } rtp_metric;

/* Hyper-parameters.  Defaults in the paper: z = 0.2, alpha = 0.1 (Algorithm 1,
 * input line), iters = 100 (Appendix C).  eps, the clamp and the form of
 * f_normalize are not given by the paper (see each field). */
typedef struct rtprune_params {
  float z;         /* dustbin score of Eq. 4 */
  float alpha;     /* merge strength of Eq. 6 */
  float eps;       /* entropic temperature: the Sinkhorn log-kernel is S_bar / eps;
                      eps = 1 uses the scores directly as Appendix C's Z. > 0 */
  int32_t iters;   /* T, number of Sinkhorn iterations (u then v each). >= 0 */
  int32_t dynamic; /* 0: fixed retention `ratio`; 1: retention from Eq. 9 */
  float ratio;     /* fixed retention 1 - r, in (0, 1] */
  float ratio_min; /* dynamic retention is clamped to [ratio_min, ratio_max] */
  float ratio_max;
  float phi_lo;    /* f_normalize(phi) = clamp((phi - phi_lo) / (phi_hi - phi_lo), 0, 1) */
  float phi_hi;    /* phi_hi > phi_lo */
  int32_t metric;  /* rtp_metric: the importance score stage 1 ranks tokens by */
  int32_t mid_merge_min_images; /* kernel choice only, no effect on what is computed beyond the
                      order of fp32 additions in the merge: images with 17 to 64 pruned tokens have
                      a merge kernel of their own (kept rows streamed past the matrix cores), which
                      the calls with a workspace run only when the batch holds at least this many
                      such images (a few cost less inside the vector kernel's launch).  0: decide by
                      the size of the chip (four 128-row tiles per compute unit: 256 images of 400
                      tokens on MI355X); n > 0: from n such images on.  >= 0 */
} rtprune_params;

/* One packed ragged batch of visual tokens. */
typedef struct rtprune_batch {
  const void* tokens;     /* device, [total_tokens, D] row-major, dtype below */
  const int32_t* offsets; /* device, [B + 1] */
  int64_t total_tokens;   /* host scalar, = offsets[B] */
  int32_t B;              /* images */
  int32_t D;              /* token width */
  int32_t max_tokens;     /* host scalar, >= every image's token count */
  int32_t dtype;          /* rtp_dtype */
} rtprune_batch;

/* Name of a status code (host string, static storage). */
const char* rtprune_status_string(int status);

/* Bytes of device workspace for a batch of this shape.  `bytes` is a host
 * pointer.  The workspace must be 256-byte aligned.  Its content is scratch:
 * nothing is carried from one call to the next, and it need not be cleared.
 *   params = NULL  the worst case over all parameters: enough for every call
 *                  below, whatever kept counts the staged calls are given
 *                  (the kernel matrix and the plan take
 *                  12 * total_tokens * max_tokens / 4 bytes of it);
 *   params given   what rtprune_prune, rtprune_prune_splice,
 *                  rtprune_dynamic_ratio and rtprune_norms_topk need with
 *                  these parameters: the fixed retention, or the clamp of the
 *                  dynamic one, bounds every pruned set by
 *                  (1 - retention) * max_tokens + 1 tokens, and the kernel
 *                  matrix and the plan are sized from that bound.
 *                  rtprune_ot_pair and rtprune_merge take their kept counts
 *                  from the caller and always ask for the worst case. */
int rtprune_workspace_bytes(int32_t B, int64_t total_tokens, int32_t max_tokens,
                            int32_t D, int32_t dtype, const rtprune_params* params,
                            size_t* bytes);

/* Dynamic pruning ratio (Sec. 3.3.3).  For each image: phi = mean pairwise
 * cosine over all its tokens (Eq. 7; 0 when N < 2; a zero-norm token has cosine
 * 0 with everything), retention = clamp(1 - f_normalize(phi) (1 - density[b]),
 * ratio_min, ratio_max) (Eq. 9), keep_counts[b] = ceil(retention * N_b - 1e-3)
 * clamped to [1, N_b] (0 when N_b = 0).
 *   density      [B] fp32 in, textual density rho of Eq. 8 per image, in [0, 1]
 *   phi          [B] fp32 out (may be NULL)
 *   ratio        [B] fp32 out, the retention (may be NULL)
 *   keep_counts  [B] int32 out */
int rtprune_dynamic_ratio(const rtprune_batch* in, const float* density,
                          const rtprune_params* params, float* phi, float* ratio,
                          int32_t* keep_counts, void* workspace,
                          size_t workspace_bytes, void* stream);

/* Stage 1, dominant-token selection (Sec. 3.3.1, Eq. 1).  Tokens are ranked by
 * the fp32 rounding of their exactly accumulated squared norm (or, with
 * params->metric = RTP_METRIC_VARIANCE, of their variance), larger first,
 * lower index first among equals; the first M_b are kept.
 *   keep_counts_in  [B] int32 in, M_b per image (clamped to [min(1,N_b), N_b]);
 *                   NULL: M_b = ceil(params->ratio * N_b - 1e-3), same clamp
 *   norms           [total_tokens] fp32 out, ||T_k||_2 (may be NULL)
 *   sel_idx         [total_tokens] int32 out; image b's segment starts at
 *                   offsets[b]: first its M_b kept token indices, ascending,
 *                   then its N_b - M_b pruned ("proposed-to-prune") indices,
 *                   ascending
 *   keep_counts     [B] int32 out, M_b (may alias keep_counts_in)
 *   out_offsets     [B + 1] int32 out, exclusive prefix sum of M_b
 *   plan_offsets    [B + 1] int64 out, exclusive prefix sum of M_b * (N_b - M_b) */
int rtprune_norms_topk(const rtprune_batch* in, const int32_t* keep_counts_in,
                       const rtprune_params* params, float* norms,
                       int32_t* sel_idx, int32_t* keep_counts,
                       int32_t* out_offsets, int64_t* plan_offsets,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Stage 2, optimal token matching (Sec. 3.3.2, Eq. 2-5; Appendix C).
 * For each image with R_b = N_b - M_b > 0: S = cosine(kept_i, pruned_j)
 * (Eq. 3), S_bar = S plus a dustbin row and column of score z (Eq. 4),
 * Z = S_bar / eps, log mu = [0_M, log R], log nu = [0_R, log M], duals start
 * at 0, `iters` iterations of (u from v, then v from u), and
 * P = exp(Z + u 1^T + 1 v^T) without its dustbin row and column.  The device
 * iterates the same map in multiplicative form in fp64.
 *   sel_idx, keep_counts, plan_offsets   as written by rtprune_norms_topk
 *   scores  [sum M_b R_b] fp64 out, S packed row-major (M_b x R_b) at
 *           plan_offsets[b] (may be NULL)
 *   plan    [sum M_b R_b] fp32 out, P packed the same way (may be NULL)
 *   pair    [total_tokens] int32 out, aligned with sel_idx: at a kept token's
 *           position its own rank i in 0..M_b-1; at a pruned token's position
 *           the rank of the kept token with the largest fp32 P_bar[i][j] in
 *           its column (lowest rank wins ties), or -1 when the dustbin row
 *           holds the column's maximum (may be NULL) */
int rtprune_ot_pair(const rtprune_batch* in, const int32_t* sel_idx,
                    const int32_t* keep_counts, const int64_t* plan_offsets,
                    const rtprune_params* params, double* scores, float* plan,
                    int32_t* pair, void* workspace, size_t workspace_bytes,
                    void* stream);

/* Merge and compaction (Eq. 6).  Row out_offsets[b] + i of `out` receives
 * T[kept_i] + alpha * sum_j plan[i][j] * T[pruned_j] for image b (fp32
 * accumulation, one rounding to the token dtype); an image with R_b = 0 is
 * copied through.
 *   out        [sum M_b, D] same dtype as the tokens
 *   workspace  as for the other calls, or NULL (then workspace_bytes is
 *              ignored).  With a workspace the call sorts the images by their
 *              pruned count first and runs the same kernels as the fused calls,
 *              so its output equals theirs bit for bit; without one, images
 *              with 17 to 64 pruned tokens take the slower vector kernel, whose
 *              fp32 sums are ordered differently. */
int rtprune_merge(const rtprune_batch* in, const int32_t* sel_idx,
                  const int32_t* keep_counts, const int32_t* out_offsets,
                  const float* plan, const int64_t* plan_offsets,
                  const rtprune_params* params, void* out, void* workspace,
                  size_t workspace_bytes, void* stream);

/* The whole operator (Algorithm 1) on a ragged batch, one enqueue, no host
 * synchronisation: [ratio ->] stage 1 -> stage 2 -> merge.
 *   density      [B] fp32 in; read only when params->dynamic (else may be NULL)
 *   out          device buffer with room for total_tokens rows of D; the first
 *                out_offsets[B] rows are written
 *   out_offsets  [B + 1] int32 out
 *   keep_counts  [B] int32 out (may be NULL)
 *   sel_idx      [total_tokens] int32 out (may be NULL)
 *   pair         [total_tokens] int32 out (may be NULL)
 *   ratio        [B] fp32 out, retention used per image (may be NULL) */
int rtprune_prune(const rtprune_batch* in, const float* density,
                  const rtprune_params* params, void* out, int32_t* out_offsets,
                  int32_t* keep_counts, int32_t* sel_idx, int32_t* pair,
                  float* ratio, void* workspace, size_t workspace_bytes,
                  void* stream);

/* rtprune_prune for callers that cannot allocate device memory or carry a
 * workspace with them: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  It is rtprune_prune with the workspace
 * taken from a fixed array of RTPRUNE_STATIC_SCRATCH_BYTES inside the
 * library's device image (each GPU the library runs on holds one copy until
 * the process ends); same kernels, same results, bit for bit.  The call
 * allocates and frees nothing (with the measurement aid below switched off);
 * the first call on a device looks up the array's address on that device and
 * is best made before a capture starts.
 *   - A batch fits when rtprune_workspace_bytes(..., params, &n) gives
 *     n <= RTPRUNE_STATIC_SCRATCH_BYTES (e.g. 64 images of 400 tokens, width
 *     1280, at any retention); a larger one is refused with RTP_EWORKSPACE and
 *     nothing is enqueued.
 *   - The status word of device-visible errors lives in the array, where the
 *     caller cannot read it: after such an error out_offsets (and every other
 *     output) is left untouched, so a caller that wants to detect one presets
 *     out_offsets[B] to -1.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap in time
 *     on the same GPU (different streams, different threads) race and give
 *     wrong results; calls on one stream, or ordered by events, are fine. */
#define RTPRUNE_STATIC_SCRATCH_BYTES (64u << 20)
int rtprune_prune_static(const rtprune_batch* in, const float* density,
                         const rtprune_params* params, void* out, int32_t* out_offsets,
                         int32_t* keep_counts, int32_t* sel_idx, int32_t* pair,
                         float* ratio, void* stream);

/* Text embeddings around each image of a batch, for rtprune_prune_splice.  All
 * rows have the batch's dtype and width D.  A side with no rows anywhere may
 * have NULL pointers and 0 rows. */
typedef struct rtprune_text_spans {
  const void* prefix;            /* device, [prefix_rows, D]: the rows before each image, packed */
  const int32_t* prefix_offsets; /* device, [B + 1] exclusive prefix sum of per-image row counts */
  int64_t prefix_rows;           /* host scalar, = prefix_offsets[B] */
  const void* suffix;            /* device, [suffix_rows, D]: the rows after each image */
  const int32_t* suffix_offsets; /* device, [B + 1] */
  int64_t suffix_rows;           /* host scalar, = suffix_offsets[B] */
} rtprune_text_spans;

/* Position convention of rtprune_prune_splice (the paper does not fix one). */
typedef enum rtp_positions {
  RTP_POSITIONS_CONSECUTIVE = 0, /* 0 .. L'-1 over each shortened sequence */
  RTP_POSITIONS_ORIGINAL = 1     /* the position each token had before pruning: prefix k -> k, kept
                                    visual token with original index i -> P + i, suffix k -> P + N + k */
} rtp_positions;

/* rtprune_prune with its output spliced into the language model's prefill input
 * (Sec. 4.3: the pruning runs before the prefill stage; Algorithm 1's output is
 * what replaces the N visual tokens).  Sequence b is written at row
 * seq_offsets[b] of `seq`: its P_b prefix rows, its M_b merged kept tokens in
 * ascending original index (the rows rtprune_prune would write), its S_b suffix
 * rows; sequences are packed in image order.
 *   seq                [seq_capacity_rows, D] out, dtype of the batch, 16-byte aligned;
 *                      seq_capacity_rows >= prefix_rows + suffix_rows + total_tokens
 *                      (else RTP_EINVAL); rows beyond seq_offsets[B] are untouched
 *   seq_offsets        [B + 1] int32 out
 *   position_ids       [seq_capacity_rows] int32 out, one per written row (may be NULL)
 *   keep_counts, sel_idx, pair, ratio   as in rtprune_prune (each may be NULL)
 * Text offsets that decrease or do not end at the stated row counts set
 * RTP_DEV_BAD_OFFSETS in the status word and nothing is written. */
int rtprune_prune_splice(const rtprune_batch* in, const float* density,
                         const rtprune_params* params, const rtprune_text_spans* text,
                         int32_t position_mode, void* seq, int64_t seq_capacity_rows,
                         int32_t* seq_offsets, int32_t* position_ids, int32_t* keep_counts,
                         int32_t* sel_idx, int32_t* pair, float* ratio, void* workspace,
                         size_t workspace_bytes, void* stream);

/* Textual density (Sec. 3.3.3, Eq. 8; Appendix B): for each page image,
 * grayscale I = (0.299 R + 0.587 G + 0.114 B) / 255, the two 3x3 Sobel responses
 * G_x, G_y (border pixels see their nearest neighbour repeated), an edge pixel
 * where sqrt(G_x^2 + G_y^2) >= tau, rho_k = fraction of edge pixels in token
 * patch k, rho = average of rho_k over the page's patches.  The arithmetic is
 * exact (integers; tau enters as (double)tau * 255000), so results do not
 * depend on rounding.  rho is what rtprune_dynamic_ratio / rtprune_prune take
 * as `density`.
 *   pixels         device, uint8, pages packed back to back; page b is
 *                  heights[b] x widths[b] x 3 (RGB interleaved, row-major) and
 *                  starts at byte pixel_offsets[b]
 *   pixel_offsets  [B + 1] int64 (device), heights / widths [B] int32 (device)
 *   max_height, max_width   host upper bounds on the page sizes
 *   patch_h, patch_w        pixels per token patch (64 x 64 for DeepSeek-OCR's
 *                  native modes); every page size must be a multiple of them
 *   density        [B] fp32 out
 *   patch_density  fp32 out, rho_k in raster order, page b's patches starting
 *                  at patch_offsets[b] (may be NULL; then patch_offsets may be)
 *   patch_offsets  [B + 1] int32 (device)
 * Device-visible errors set RTP_DEV_BAD_IMAGE in the workspace status word and
 * leave the outputs untouched.  Limits: page sides <= 65536, and at least three
 * luma rows of max_width + 2 ints must fit 60 KB of LDS (width <= 5118). */
int rtprune_text_density_workspace_bytes(int32_t B, int32_t max_height, int32_t max_width,
                                         int32_t patch_h, int32_t patch_w, size_t* bytes);
int rtprune_text_density(const uint8_t* pixels, const int64_t* pixel_offsets,
                         const int32_t* heights, const int32_t* widths, int32_t B,
                         int32_t max_height, int32_t max_width, int32_t patch_h,
                         int32_t patch_w, float tau, float* density, float* patch_density,
                         const int32_t* patch_offsets, void* workspace,
                         size_t workspace_bytes, void* stream);

/* Measurement aid (not part of the operator).  The switches are process-wide:
 * they may be flipped from any thread, and they apply to every call that starts
 * after the flip, on whichever thread; a program that prunes from several
 * threads while recording gets all of their launches in one summary.
 * While enabled, every kernel the calls above launch is bracketed by two HIP
 * events recorded on the launch stream (events are created per launch: with the
 * aid on, calls allocate).  rtprune_profile_enable(1) discards
 * earlier records and starts recording, (0) stops.  rtprune_profile_summary
 * waits for the recorded events and writes a JSON array
 *   [{"kernel": name, "launches": n, "total_ms": t}, ...]
 * into the host buffer `buf` of `cap` bytes (RTP_EINVAL if it does not fit). */
int rtprune_profile_enable(int on);
int rtprune_profile_summary(char* buf, size_t cap);
/* Restricts the recording to the launches reported under one name (as in the
 * summary, e.g. "k_merge"); NULL or "" records all again.  An event pair takes a
 * few microseconds of stream time, so a timed region that wants one kernel's
 * duration records that kernel alone.  RTP_EINVAL for an unknown name. */
int rtprune_profile_only(const char* kernel);

/* Measurement aid: a plain device-to-device copy kernel (`k_copy`) of `bytes`
 * bytes (a multiple of 16; both pointers 16-byte aligned, non-overlapping).
 * It moves exactly `bytes` in and `bytes` out, which is what hardware traffic
 * counters read for the operator's kernels are scaled against. */
int rtprune_copy_bytes(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RTPRUNE_H */
