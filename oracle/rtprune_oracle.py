"""CPU oracle for the RTPrune visual-token reduction operator.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, double-precision restatement
of what the operator computes, written from the paper's definitions so that it
can be checked against them by eye.  Only ``tests/``, the repository's smoke
check and the benchmark's ``cpu_baseline`` leg may import it; the product
path (the HIP library and its binding) never does, and shares no code, table or
helper with it.

Every function cites the passage it follows:

* stage 1, dominant-token selection: Sec. 3.3.1, Eq. 1, and ``M = N(1-r)``;
* stage 2, score matrix, dustbin augmentation, transport constraints:
  Sec. 3.3.2, Eq. 2-5;
* log-space Sinkhorn iterations and the final plan: Appendix C;
* merge: Eq. 6 (also the last equation of Appendix C);
* inter-token similarity and the dynamic pruning ratio: Sec. 3.3.3, Eq. 7, 9;
* textual density from Sobel edges: Sec. 3.3.3, Eq. 8, and Appendix B (exact
  integer arithmetic on 8-bit pixels; the only real number is the threshold);
* order of the steps: Algorithm 1.

Arithmetic is float64 throughout.  Inputs are the exact values the device sees
(bf16 bit patterns are widened exactly).  The few places where a real number
decides an integer take that decision on a float32 rounding of the float64
value, the precision in which the device kernels publish the same quantity:

* the selection score of a token is ``float32(sum of squares)``; ordering is by
  (score descending, index ascending);
* the similarity statistic enters the ratio formula as ``float32(phi)``, the
  retention leaves it as a float32, and the kept count is
  ``ceil(float64(retention32) * N - 1e-3)`` clamped to [1, N];
* the partner of a pruned token is the arg-max over ``float32(P_bar[:, j])``
  with the lowest row index winning ties (the dustbin row is the last row).

Readings of points the paper leaves open (each is restated where it is used):
retention = 1 - r; ``f_normalize`` is an affine map clamped to [0, 1];
``Z = S_bar / eps`` with eps = 1 giving the literal text; duals start at zero
and u is updated before v; marginals are the unnormalised ones printed in
Appendix C; a zero-norm token has cosine 0 with everything; if nothing is
pruned (R = 0) the image passes through unchanged.

Parity status: every function below is pinned by ``tests/test_oracle_*.py``
against closed forms, invariants, library routines, an exact LP solver and
brute force; what cannot be pinned offline is OCR accuracy on real pages
("parity unpinned": it needs model weights and benchmark data).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np

TINY_NORM = 1e-12          # floor on a token norm before dividing by it
COUNT_SLACK = 1e-3         # tokens; absorbs float32 representation error of the retention


# ---------------------------------------------------------------------------
# parameters
# ---------------------------------------------------------------------------
@dataclass
class Params:
    """Hyper-parameters; every real is held as the float32 the C struct carries."""
    z: float = 0.2          # dustbin score (Algorithm 1 input line)
    alpha: float = 0.1      # merge strength (Algorithm 1 input line)
    eps: float = 0.05       # entropic temperature (not in the paper; 1.0 = literal text)
    iters: int = 100        # T (Appendix C)
    dynamic: int = 0        # 0: fixed retention `ratio`; 1: Eq. 9
    ratio: float = 0.84     # retention 1 - r when not dynamic
    ratio_min: float = 0.6  # clamp on the dynamic retention
    ratio_max: float = 1.0
    phi_lo: float = 0.0     # f_normalize(phi) = clamp((phi - lo) / (hi - lo), 0, 1)
    phi_hi: float = 1.0
    metric: int = 0         # importance score: 0 = l2 norm (Eq. 1), 1 = variance (Table 7 ablation)

    @staticmethod
    def from_dict(d: Dict[str, float]) -> "Params":
        return Params(**{k: d[k] for k in Params.__dataclass_fields__ if k in d})

    def f32(self, name: str) -> float:
        """The parameter as float32, widened back to a Python float."""
        return float(np.float32(getattr(self, name)))


# ---------------------------------------------------------------------------
# input widening and output rounding
# ---------------------------------------------------------------------------
def widen(tokens: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 values of a token array (float32, or uint16 bf16 patterns)."""
    if dtype == "bf16":
        bits = np.ascontiguousarray(tokens, dtype=np.uint16).astype(np.uint32) << 16
        return bits.view(np.float32).astype(np.float64)
    if dtype == "f32":
        return np.asarray(tokens, dtype=np.float32).astype(np.float64)
    raise ValueError(dtype)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (ties to even), as float64.

    One rounding straight from float64: 8 significant bits, float32's exponent
    range (subnormals below 2**-126 keep that fixed spacing).
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros_like(x)
    nz = (x != 0) & np.isfinite(x)
    _, e = np.frexp(x[nz])                     # |x| = m * 2**e, m in [0.5, 1)
    e = np.maximum(e - 1, -126)                # exponent of the leading bit
    q = np.ldexp(1.0, e - 7)                   # spacing of bf16 at that exponent
    out[nz] = np.rint(x[nz] / q) * q           # rint: ties to even
    out[~np.isfinite(x)] = x[~np.isfinite(x)]
    return out


def round_to_f32(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


# ---------------------------------------------------------------------------
# stage 1: norm criterion and top-M selection (Sec. 3.3.1, Eq. 1)
# ---------------------------------------------------------------------------
def token_sqnorms(X: np.ndarray) -> np.ndarray:
    """q_k = sum_d X[k, d]**2 in float64 (Eq. 1 squared)."""
    return np.einsum("kd,kd->k", X, X)


def token_norms(X: np.ndarray) -> np.ndarray:
    """C_k = ||T_v^k||_2 (Eq. 1)."""
    return np.sqrt(token_sqnorms(X))


METRIC_L2NORM, METRIC_VARIANCE = 0, 1


def token_variances(X: np.ndarray) -> np.ndarray:
    """Variance of each token's D feature values (selection-metric ablation,
    Sec. 4.4 / Table 7), by the two-pass definition in float64.

    The paper names the metric without a formula; the population form (divide
    by D) is taken - the sample form differs by the constant D/(D-1) and ranks
    tokens identically.
    """
    X = np.asarray(X, dtype=np.float64)
    if X.shape[1] == 0:
        return np.zeros(X.shape[0])
    mean = np.sum(X, axis=1, keepdims=True) / X.shape[1]
    dev = X - mean
    return np.sum(dev * dev, axis=1) / X.shape[1]


def selection_scores(X: np.ndarray, metric: int = METRIC_L2NORM) -> np.ndarray:
    """The float32 score tokens are ranked by.

    l2 norm (Eq. 1): float32 of the squared norm - ranking by the squared norm
    equals ranking by the norm (sqrt is monotone), and the squared form is what
    both sides round to float32.  Variance: float32 of the variance.
    """
    if metric == METRIC_VARIANCE:
        return token_variances(X).astype(np.float32)
    if metric != METRIC_L2NORM:
        raise ValueError("unknown selection metric")
    return token_sqnorms(X).astype(np.float32)


def kept_count(retention32: float, n: int) -> int:
    """M = N(1 - r) (Sec. 3.3.1) with the rounding the paper leaves open.

    Reading: M = ceil(retention * N), evaluated as
    ceil(float64(retention32) * N - 1e-3) and clamped to [1, N], so that a
    retention whose float32 form sits a hair above k/N still gives k (all
    counts the paper prints are exact products: 48, 75, 192, 300, 128, 200).
    """
    if n <= 0:
        return 0
    m = math.ceil(float(np.float32(retention32)) * n - COUNT_SLACK)
    return min(n, max(1, m))


def select_topk(scores32: np.ndarray, m: int):
    """Top-M tokens by score (Sec. 3.3.1): returns (kept, prop), both ascending.

    Order is (score descending, index ascending): among equal scores the lower
    index is kept first.  Output order is original (raster) order, which is what
    the language model's positions encode.
    """
    n = len(scores32)
    order = sorted(range(n), key=lambda k: (-float(scores32[k]), k))
    kept = np.array(sorted(order[:m]), dtype=np.int32)
    prop = np.array(sorted(order[m:]), dtype=np.int32)
    return kept, prop


# ---------------------------------------------------------------------------
# dynamic pruning ratio (Sec. 3.3.3, Eq. 7 and 9)
# ---------------------------------------------------------------------------
def unit_rows(X: np.ndarray) -> np.ndarray:
    n = token_norms(X)
    return X / np.maximum(n, TINY_NORM)[:, None]


def inter_token_similarity(X: np.ndarray) -> float:
    """phi = 2 / (N (N-1)) * sum_{i<j} cos(T_i, T_j) over all N tokens (Eq. 7).

    Written as the definition: the full cosine matrix, then the sum of its
    strict upper triangle.  N < 2 has no pairs; phi is taken as 0.
    """
    n = X.shape[0]
    if n < 2:
        return 0.0
    U = unit_rows(X)
    C = U @ U.T
    iu = np.triu_indices(n, k=1)
    return float(2.0 / (n * (n - 1)) * C[iu].sum())


def dynamic_retention(phi: float, density32: float, p: Params) -> np.float32:
    """Retention 1 - r_dyn with r_dyn = f_normalize(phi) (1 - rho) (Eq. 9).

    ``f_normalize`` is not defined in the paper; reading: the affine map
    (phi - lo) / (hi - lo) clamped to [0, 1] (defaults lo = 0, hi = 1).  The
    retention is then clamped to [ratio_min, ratio_max] (benchmark definition)
    and published as float32.  phi enters as float32(phi).
    """
    phi32 = float(np.float32(phi))
    lo, hi = p.f32("phi_lo"), p.f32("phi_hi")
    f = min(1.0, max(0.0, (phi32 - lo) / (hi - lo)))
    r = f * (1.0 - float(np.float32(density32)))
    ret = min(p.f32("ratio_max"), max(p.f32("ratio_min"), 1.0 - r))
    return np.float32(ret)


# ---------------------------------------------------------------------------
# stage 2: scores, dustbins, Sinkhorn, pairing (Sec. 3.3.2, Appendix C)
# ---------------------------------------------------------------------------
def cosine_scores(X: np.ndarray, kept: np.ndarray, prop: np.ndarray) -> np.ndarray:
    """S_ij = T_i . T_j / (||T_i|| ||T_j||) for (i, j) in kept x prop (Eq. 3)."""
    n = token_norms(X)
    dots = X[kept] @ X[prop].T
    den = np.maximum(n[kept][:, None] * n[prop][None, :], TINY_NORM * TINY_NORM)
    return dots / den


def augment(S: np.ndarray, z: float) -> np.ndarray:
    """S_bar: S with one more row and column, all new entries equal z (Eq. 4)."""
    m, r = S.shape
    Sb = np.full((m + 1, r + 1), float(z), dtype=np.float64)
    Sb[:m, :r] = S
    return Sb


def logsumexp(A: np.ndarray, axis: int) -> np.ndarray:
    """log sum exp along an axis, with the maximum taken out first."""
    mx = np.max(A, axis=axis, keepdims=True)
    return (mx + np.log(np.sum(np.exp(A - mx), axis=axis, keepdims=True))).squeeze(axis)


def sinkhorn_log(S: np.ndarray, z: float, eps: float, iters: int):
    """Appendix C: T log-space Sinkhorn iterations on the augmented scores.

    Z = S_bar / eps (the paper's "log-augmented score matrix"; eps = 1 is the
    literal text).  log mu = [0_M, log(N-M)], log nu = [0_{N-M}, log M].
    Duals start at zero; each iteration updates u from the current v, then v
    from the new u.  Returns (P_bar, u, v) with
    P_bar = exp(Z + u 1^T + 1 v^T), shape (M+1) x (N-M+1).
    """
    m, r = S.shape
    Z = augment(S, z) / float(eps)
    log_mu = np.zeros(m + 1)
    log_mu[m] = math.log(r)
    log_nu = np.zeros(r + 1)
    log_nu[r] = math.log(m)
    u = np.zeros(m + 1)
    v = np.zeros(r + 1)
    for _ in range(int(iters)):
        u = log_mu - logsumexp(Z + v[None, :], axis=1)
        v = log_nu - logsumexp(Z + u[:, None], axis=0)
    P_bar = np.exp(Z + u[:, None] + v[None, :])
    return P_bar, u, v


def pairing(P_bar: np.ndarray) -> np.ndarray:
    """Partner of each pruned token: arg-max of its column of P_bar.

    The paper merges softly (Eq. 6) and only says that a pruned token goes "to
    some selected tokens or the dustbin"; the hard pairing reported here is the
    column arg-max over the M kept rows and the dustbin row, taken on the
    float32 rounding of P_bar, lowest row index winning ties.  The dustbin
    (row M) is reported as -1.  The map need not be injective.
    """
    m = P_bar.shape[0] - 1
    r = P_bar.shape[1] - 1
    P32 = P_bar[:, :r].astype(np.float32)
    best = np.argmax(P32, axis=0).astype(np.int32)      # first maximum = lowest index
    best[best == m] = -1
    return best


def merge(X: np.ndarray, kept: np.ndarray, prop: np.ndarray, P: np.ndarray,
          alpha: float) -> np.ndarray:
    """T_i <- T_i + alpha * sum_j P_ij T_j for kept i, pruned j (Eq. 6)."""
    return X[kept] + float(alpha) * (P @ X[prop])


# ---------------------------------------------------------------------------
# whole operator (Algorithm 1)
# ---------------------------------------------------------------------------
@dataclass
class ImageResult:
    n: int
    sqnorm: np.ndarray            # float64 [N]
    score: np.ndarray             # float32 [N]
    phi: float                    # float64 (0 when not computed)
    retention: np.float32
    m: int
    kept: np.ndarray              # int32 [M] ascending
    prop: np.ndarray              # int32 [R] ascending
    S: Optional[np.ndarray]       # float64 [M, R]
    P_bar: Optional[np.ndarray]   # float64 [M+1, R+1]
    pair: np.ndarray              # int32 [R]
    merged: np.ndarray            # float64 [M, D], unrounded

    @property
    def r(self) -> int:
        return self.n - self.m

    @property
    def P(self) -> Optional[np.ndarray]:
        return None if self.P_bar is None else self.P_bar[:-1, :-1]


def prune_image(X: np.ndarray, density32: float, p: Params,
                keep_count: Optional[int] = None) -> ImageResult:
    """Algorithm 1 on one image's float64 tokens ``X`` ([N, D]).

    ``keep_count`` overrides the kept count (used to re-run an image at the
    device's M when the two retentions straddle a ceil boundary).
    """
    n = X.shape[0]
    q = token_sqnorms(X)
    score = selection_scores(X, p.metric)
    phi = 0.0
    if p.dynamic:
        phi = inter_token_similarity(X)
        ret = dynamic_retention(phi, density32, p)
    else:
        ret = np.float32(p.ratio)
    m = kept_count(ret, n) if keep_count is None else int(keep_count)
    kept, prop = select_topk(score, m)
    r = n - m
    if n == 0 or r == 0:
        return ImageResult(n, q, score, phi, ret, m, kept, prop, None, None,
                           np.zeros(0, dtype=np.int32), X[kept].copy())
    S = cosine_scores(X, kept, prop)
    P_bar, _, _ = sinkhorn_log(S, p.f32("z"), p.f32("eps"), p.iters)
    pr = pairing(P_bar)
    out = merge(X, kept, prop, P_bar[:m, :r], p.f32("alpha"))
    return ImageResult(n, q, score, phi, ret, m, kept, prop, S, P_bar, pr, out)


def prune_batch(tokens: np.ndarray, dtype: str, offsets: Sequence[int],
                density: Sequence[float], p: Params,
                keep_counts: Optional[Sequence[Optional[int]]] = None) -> List[ImageResult]:
    """Algorithm 1 on a packed ragged batch, one image at a time."""
    res = []
    for b in range(len(offsets) - 1):
        lo, hi = int(offsets[b]), int(offsets[b + 1])
        X = widen(tokens[lo:hi], dtype)
        kc = None if keep_counts is None else keep_counts[b]
        res.append(prune_image(X, float(density[b]) if len(density) else 0.0, p, kc))
    return res


# ---------------------------------------------------------------------------
# near-tie bookkeeping (used by parity tests to classify index mismatches)
# ---------------------------------------------------------------------------
def selection_gap(score32: np.ndarray, m: int) -> float:
    """Relative gap between the M-th and (M+1)-th largest scores (inf if none)."""
    n = len(score32)
    if m <= 0 or m >= n:
        return math.inf
    s = np.sort(score32.astype(np.float64))[::-1]
    a, b = s[m - 1], s[m]
    return float((a - b) / max(abs(a), 1e-300))


def pairing_gaps(P_bar: np.ndarray) -> np.ndarray:
    """Per pruned token: relative gap between the two largest float32 entries of its column."""
    r = P_bar.shape[1] - 1
    P32 = P_bar[:, :r].astype(np.float32).astype(np.float64)
    if P32.shape[0] < 2:
        return np.full(r, np.inf)
    top = np.sort(P32, axis=0)[::-1]
    return (top[0] - top[1]) / np.maximum(np.abs(top[0]), 1e-300)


# ---------------------------------------------------------------------------
# textual density (Sec. 3.3.3, Eq. 8; Appendix B)
# ---------------------------------------------------------------------------
GRAY_MILLI = (299, 587, 114)     # ITU-R BT.601 weights x 1000 (Appendix B)


def gray_milli(rgb_u8: np.ndarray) -> np.ndarray:
    """1000 x 255 x I(i, j): the BT.601 grayscale of Appendix B in exact integers.

    With 8-bit channels and intensities scaled to [0, 1] (the scale on which the
    default threshold tau = 0.2 is meaningful), I = (0.299 R + 0.587 G + 0.114 B) / 255.
    """
    c = np.asarray(rgb_u8).astype(np.int64)
    return GRAY_MILLI[0] * c[..., 0] + GRAY_MILLI[1] * c[..., 1] + GRAY_MILLI[2] * c[..., 2]


def sobel_xy(gray: np.ndarray):
    """G_x and G_y of Appendix B (the printed 3x3 kernels) on an integer image.

    Border pixels see their nearest neighbour repeated (reading: the paper does
    not say; zero padding would turn every border pixel of a white page into an
    edge).  Convolution versus correlation only flips signs, which the magnitude
    does not see.
    """
    p = np.pad(gray, 1, mode="edge")
    gx = (p[:-2, 2:] + 2 * p[1:-1, 2:] + p[2:, 2:]) - (p[:-2, :-2] + 2 * p[1:-1, :-2] + p[2:, :-2])
    gy = (p[:-2, :-2] + 2 * p[:-2, 1:-1] + p[:-2, 2:]) - (p[2:, :-2] + 2 * p[2:, 1:-1] + p[2:, 2:])
    return gx, gy


def edge_map(rgb_u8: np.ndarray, tau: float) -> np.ndarray:
    """E(i, j) = [G(i, j) >= tau], G = sqrt(G_x^2 + G_y^2) on intensities in [0, 1].

    Evaluated without a square root and without rounding: in units of
    1/(255 * 1000) the squared magnitude is an integer, compared with
    (float32(tau) * 255000)^2.
    """
    gx, gy = sobel_xy(gray_milli(rgb_u8))
    mag2 = (gx * gx + gy * gy).astype(np.float64)          # exact: below 2**53
    t = float(np.float32(tau)) * 255000.0
    return mag2 >= t * t


def text_density(rgb_u8: np.ndarray, patch_h: int, patch_w: int, tau: float):
    """rho_k per token patch (Eq. 8) and their average rho, both float32.

    The image (H x W x 3, uint8) is cut into (H / patch_h) x (W / patch_w)
    patches in raster order, one per visual token.
    """
    h, w = rgb_u8.shape[:2]
    assert h % patch_h == 0 and w % patch_w == 0
    e = edge_map(rgb_u8, tau)
    counts = e.reshape(h // patch_h, patch_h, w // patch_w, patch_w).sum(axis=(1, 3)).astype(np.int64)
    area = patch_h * patch_w
    rho_k = (counts.astype(np.float64) / area).astype(np.float32).ravel()
    rho = np.float32(float(counts.sum()) / float(counts.size * area))
    return rho, rho_k


# ---------------------------------------------------------------------------
# sequence splice: pruned visual tokens into the language model's input
# ---------------------------------------------------------------------------
POSITIONS_CONSECUTIVE, POSITIONS_ORIGINAL = 0, 1


def splice_sequence(prefix: np.ndarray, visual: np.ndarray, suffix: np.ndarray,
                    kept: np.ndarray, n_visual: int, mode: int = POSITIONS_CONSECUTIVE):
    """Input sequence of the language model's prefill after pruning (Sec. 4.3: the
    pruning runs before the prefill stage): text embeddings before the image, the
    merged kept visual tokens in ascending original index, text embeddings after it.

    The paper does not say which position each token takes; both natural choices
    are offered:
      POSITIONS_CONSECUTIVE  0, 1, ..., L'-1 over the shortened sequence;
      POSITIONS_ORIGINAL     the position the token had in the unpruned sequence:
                             prefix k -> k, kept token with original index i ->
                             P + i, suffix k -> P + N + k.
    Returns (rows [P + M + S, D], position ids int32 [P + M + S]).
    """
    P, M, S = prefix.shape[0], visual.shape[0], suffix.shape[0]
    assert len(kept) == M
    rows = np.concatenate([prefix, visual, suffix], axis=0)
    if mode == POSITIONS_CONSECUTIVE:
        pos = np.arange(P + M + S, dtype=np.int32)
    elif mode == POSITIONS_ORIGINAL:
        pos = np.concatenate([np.arange(P), P + np.asarray(kept, dtype=np.int64),
                              P + n_visual + np.arange(S)]).astype(np.int32)
    else:
        raise ValueError("unknown position mode")
    return rows, pos
