"""Pins for the oracle's stage 2: scores (Eq. 3), dustbins (Eq. 4-5), Sinkhorn
(Appendix C), pairing, merge (Eq. 6) and the whole operator (Algorithm 1)."""
import itertools
import math

import numpy as np
import pytest

from oracle import rtprune_oracle as orc


def _converged(S, z, eps, tol=1e-11, cap=200000):
    """Run the oracle's own iteration until the row marginals settle."""
    m, r = S.shape
    it = 64
    while True:
        P, u, v = orc.sinkhorn_log(S, z, eps, it)
        a = np.ones(m + 1)
        a[m] = r
        if np.abs(P.sum(axis=1) - a).max() < tol or it >= cap:
            return P, it
        it *= 2


# -------------------------------------------------------------------- scores
def test_scores_are_the_normalised_gram_block():
    rng = np.random.default_rng(10)
    X = rng.standard_normal((12, 7))
    kept = np.array([0, 3, 4, 8, 11])
    prop = np.array([1, 2, 5, 6, 7, 9, 10])
    S = orc.cosine_scores(X, kept, prop)
    for a, i in enumerate(kept):
        for b, j in enumerate(prop):
            want = sum(X[i] * X[j]) / math.sqrt(sum(X[i] ** 2) * sum(X[j] ** 2))
            assert abs(S[a, b] - want) < 1e-14
    np.testing.assert_allclose(S, orc.cosine_scores(X, prop, kept).T, rtol=0, atol=1e-15)
    assert np.abs(S).max() <= 1 + 1e-12
    # a token against a positive multiple of itself scores 1, against its negative -1
    Y = np.array([[1.0, 2.0, 3.0], [2.0, 4.0, 6.0], [-0.5, -1.0, -1.5], [0.0, 0.0, 0.0]])
    S = orc.cosine_scores(Y, np.array([0]), np.array([1, 2, 3]))
    np.testing.assert_allclose(S, [[1.0, -1.0, 0.0]], atol=1e-15)


def test_augment_layout():
    S = np.arange(6.0).reshape(2, 3)
    Sb = orc.augment(S, 0.2)
    assert Sb.shape == (3, 4)
    np.testing.assert_array_equal(Sb[:2, :3], S)
    assert (Sb[2, :] == 0.2).all() and (Sb[:, 3] == 0.2).all()


# ------------------------------------------------------------------ Sinkhorn
def test_column_marginals_and_total_mass_after_any_number_of_iterations():
    rng = np.random.default_rng(11)
    for (m, r), eps, T in (((5, 3), 0.05, 1), ((20, 9), 0.05, 7), ((54, 10), 0.05, 50), ((7, 12), 1.0, 3)):
        S = rng.uniform(-1, 1, size=(m, r))
        P, u, v = orc.sinkhorn_log(S, 0.2, eps, T)
        b = np.ones(r + 1)
        b[r] = m
        np.testing.assert_allclose(P.sum(axis=0), b, rtol=1e-12)       # the v-update came last
        assert abs(P.sum() - (m + r)) < 1e-10
        assert (P >= 0).all()
        # row mass of the kept x pruned block never exceeds the kept token's unit mass by much
        assert u.shape == (m + 1,) and v.shape == (r + 1,)


def test_row_marginals_at_convergence():
    rng = np.random.default_rng(12)
    S = rng.uniform(-1, 1, size=(9, 6))
    P, it = _converged(S, 0.2, 0.5)
    a = np.ones(10)
    a[9] = 6
    np.testing.assert_allclose(P.sum(axis=1), a, atol=1e-10)
    b = np.ones(7)
    b[6] = 9
    np.testing.assert_allclose(P.sum(axis=0), b, atol=1e-10)
    assert (P[:-1, :-1].sum(axis=1) <= 1 + 1e-9).all()


def test_one_kept_one_pruned_closed_form():
    # M = R = 1: the 2x2 plan [[p, 1-p], [1-p, p]] has p = sqrt(k) / (1 + sqrt(k)),
    # k = exp((s - z) / eps)   (from p^2 / (1-p)^2 = k)
    for s, z, eps in ((0.9, 0.2, 1.0), (-0.3, 0.2, 1.0), (0.2, 0.2, 1.0), (0.6, 0.1, 0.5)):
        P, _ = _converged(np.array([[s]]), z, eps)
        k = math.exp((s - z) / eps)
        want = math.sqrt(k) / (1 + math.sqrt(k))
        assert abs(P[0, 0] - want) < 1e-9, (s, z, eps)
        assert abs(P[1, 1] - want) < 1e-9
        assert abs(P[0, 1] - (1 - want)) < 1e-9


def test_constant_scores_closed_form():
    # S == c: by symmetry every kept x pruned cell equals x, the dustbin cells are
    # 1 - R x (rows) and 1 - M x (columns), the corner is R M x, and
    # x * corner / (row_dustbin * col_dustbin) = k = exp((c - z) / eps), i.e.
    # (k - 1) R M x^2 - k (R + M) x + k = 0, root in [0, 1 / max(M, R)].
    for m, r, c, z, eps in ((5, 3, 1.0, 0.2, 0.05), (5, 3, 0.5, 0.2, 0.1), (5, 3, 0.2, 0.2, 0.3), (2, 6, -0.4, 0.2, 0.5)):
        k = math.exp((c - z) / eps)
        if abs(k - 1) < 1e-12:
            x = 1.0 / (m + r)
        else:
            A, B, C = (k - 1) * r * m, -k * (r + m), k
            roots = [(-B - math.sqrt(B * B - 4 * A * C)) / (2 * A), (-B + math.sqrt(B * B - 4 * A * C)) / (2 * A)]
            x = [t for t in roots if -1e-12 <= t <= 1.0 / max(m, r) + 1e-12][0]
        P, _ = _converged(np.full((m, r), c), z, eps, tol=1e-12)
        np.testing.assert_allclose(P[:m, :r], x, rtol=1e-7, atol=1e-12)
        assert abs(P[m, r] - r * m * x) < 1e-7


def test_matches_textbook_scaling_form_iteration_for_iteration():
    # Cuturi's matrix-scaling iteration on K = exp(S_bar / eps) with the same
    # marginals and update order is the same map written multiplicatively.
    rng = np.random.default_rng(13)
    m, r, z, eps, T = 11, 5, 0.2, 0.1, 17
    S = rng.uniform(-1, 1, size=(m, r))
    Sb = np.full((m + 1, r + 1), z)
    Sb[:m, :r] = S
    K = np.exp(Sb / eps)
    a = np.ones(m + 1)
    a[m] = r
    b = np.ones(r + 1)
    b[r] = m
    y = np.ones(r + 1)
    for _ in range(T):
        x = a / (K @ y)
        y = b / (K.T @ x)
    want = x[:, None] * K * y[None, :]
    got, u, v = orc.sinkhorn_log(S, z, eps, T)
    np.testing.assert_allclose(got, want, rtol=1e-11)
    np.testing.assert_allclose(np.exp(u), x, rtol=1e-11)


def test_logsumexp_against_scipy():
    sp = pytest.importorskip("scipy.special")
    rng = np.random.default_rng(14)
    A = rng.uniform(-800, 800, size=(6, 9))
    np.testing.assert_allclose(orc.logsumexp(A, 1), sp.logsumexp(A, axis=1), rtol=1e-14)
    np.testing.assert_allclose(orc.logsumexp(A, 0), sp.logsumexp(A, axis=0), rtol=1e-14)


def test_small_eps_plan_reaches_the_exact_transport_optimum():
    # Eq. 2 with the dustbin constraints (Eq. 5) is a linear programme; solve it
    # exactly and check that the converged entropic plan is feasible and within
    # eps * (entropy range) of the optimum, and never above it.
    opt = pytest.importorskip("scipy.optimize")
    rng = np.random.default_rng(15)
    m, r, z, eps = 6, 4, 0.2, 0.02
    S = rng.uniform(-1, 1, size=(m, r))
    Sb = orc.augment(S, z)
    rows, cols = m + 1, r + 1
    A_eq, b_eq = [], []
    for i in range(rows):
        row = np.zeros((rows, cols))
        row[i, :] = 1
        A_eq.append(row.ravel())
        b_eq.append(1.0 if i < m else float(r))
    for j in range(cols):
        col = np.zeros((rows, cols))
        col[:, j] = 1
        A_eq.append(col.ravel())
        b_eq.append(1.0 if j < r else float(m))
    lp = opt.linprog(-Sb.ravel(), A_eq=np.array(A_eq), b_eq=np.array(b_eq), bounds=(0, None), method="highs")
    assert lp.status == 0
    best = -lp.fun
    P, _ = _converged(S, z, eps, tol=1e-10)
    val = float((Sb * P).sum())
    n = m + r
    assert val <= best + 1e-8
    assert val >= best - eps * n * (1 + math.log(rows * cols))
    # and the LP optimum is the max-weight partial matching with weights S - z, plus z N
    assert abs(best - (_best_matching(S, z)[0] + z * n)) < 1e-9


# ------------------------------------------------------------------- pairing
def _best_matching(S, z):
    """Brute force: best and second-best value of sum (S_ij - z) over injective partial maps pruned -> kept."""
    m, r = S.shape
    vals = []
    choices = [list(range(m)) + [None]] * r
    for assign in itertools.product(*choices):
        used = [a for a in assign if a is not None]
        if len(used) != len(set(used)):
            continue
        vals.append((sum(S[a, j] - z for j, a in enumerate(assign) if a is not None), assign))
    vals.sort(key=lambda t: -t[0])
    return vals[0][0], vals[0][1], vals[1][0]


def test_pairing_equals_brute_force_matching_when_the_optimum_is_clear():
    rng = np.random.default_rng(16)
    z, eps = 0.2, 0.05
    checked = 0
    for trial in range(60):
        n = int(rng.integers(3, 9))
        m = int(rng.integers(1, n))
        r = n - m
        if r > m + 3:
            continue
        X = rng.standard_normal((n, 3))
        kept = np.arange(m)
        prop = np.arange(m, n)
        S = orc.cosine_scores(X, kept, prop)
        best, assign, second = _best_matching(S, z)
        if best - second < 2 * eps:
            continue
        P, _ = _converged(S, z, eps, tol=1e-9, cap=1 << 16)
        pr = orc.pairing(P)
        want = [-1 if a is None else a for a in assign]
        assert list(pr) == want, (trial, S)
        checked += 1
    assert checked >= 15


def test_pairing_planted_near_copies_and_outlier():
    rng = np.random.default_rng(17)
    d = 32
    kept_tok = rng.standard_normal((5, d)) * 3.0                 # large norm -> kept
    copies = kept_tok[[3, 0, 3]] / 3.0 + 0.01 * rng.standard_normal((3, d))
    loner = rng.standard_normal((1, d)) * 0.5                   # similar to nothing
    X = np.concatenate([kept_tok, copies, loner])
    res = orc.prune_image(X, 0.5, orc.Params(ratio=5 / 9, iters=300))
    assert list(res.kept) == [0, 1, 2, 3, 4] and list(res.prop) == [5, 6, 7, 8]
    assert list(res.pair) == [3, 0, 3, -1]                      # not injective, dustbin for the loner


def test_pairing_tie_goes_to_lowest_index_and_dustbin_loses_ties():
    P_bar = np.array([[0.2, 0.1, 0.0], [0.2, 0.3, 0.0], [0.2, 0.3, 0.0]])
    # last row is the dustbin row, last column the dustbin column
    assert list(orc.pairing(P_bar)) == [0, 1]
    P_bar = np.array([[0.1, 0.0], [0.4, 0.0]])
    assert list(orc.pairing(P_bar)) == [-1]


# --------------------------------------------------------------------- merge
def test_merge_equals_triple_loop():
    rng = np.random.default_rng(18)
    X = rng.standard_normal((9, 4))
    kept = np.array([0, 2, 5, 8])
    prop = np.array([1, 3, 4, 6, 7])
    P = rng.uniform(0, 0.3, size=(4, 5))
    out = orc.merge(X, kept, prop, P, 0.1)
    for a, i in enumerate(kept):
        for d in range(4):
            acc = X[i, d]
            for b, j in enumerate(prop):
                acc += 0.1 * P[a, b] * X[j, d]
            assert abs(out[a, d] - acc) < 1e-15


def test_merge_limits():
    rng = np.random.default_rng(19)
    X = rng.standard_normal((40, 16)) * rng.lognormal(0, 0.5, size=(40, 1))
    base = orc.Params(ratio=0.75, iters=50)
    r0 = orc.prune_image(X, 0.5, orc.Params(ratio=0.75, iters=50, alpha=0.0))
    np.testing.assert_array_equal(r0.merged, X[r0.kept])               # alpha = 0: pure pruning
    r1 = orc.prune_image(X, 0.5, base)
    delta = np.linalg.norm(r1.merged - X[r1.kept], axis=1)
    bound = base.f32("alpha") * np.linalg.norm(X[r1.prop], axis=1).max()
    row_mass = r1.P.sum(axis=1)
    assert (delta <= bound * np.maximum(row_mass, 1e-300) + 1e-12).all()
    # a dustbin score far above every cosine sends all mass to the dustbins
    r2 = orc.prune_image(X, 0.5, orc.Params(ratio=0.75, iters=50, z=3.0))
    assert np.abs(r2.merged - X[r2.kept]).max() < 1e-12
    assert (r2.pair == -1).all()


# ------------------------------------------------------------ whole operator
def test_ragged_batch_equals_each_image_alone():
    rng = np.random.default_rng(20)
    counts = [5, 0, 1, 12, 7]
    imgs = [rng.standard_normal((c, 8)).astype(np.float32) for c in counts]
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    tokens = np.concatenate(imgs)
    dens = rng.uniform(0.1, 0.9, len(counts)).astype(np.float32)
    p = orc.Params(dynamic=1, phi_lo=0.0, phi_hi=0.2, iters=20)
    batch = orc.prune_batch(tokens, "f32", offsets, dens, p)
    for b, x in enumerate(imgs):
        alone = orc.prune_image(x.astype(np.float64), float(dens[b]), p)
        assert alone.m == batch[b].m
        np.testing.assert_array_equal(alone.kept, batch[b].kept)
        np.testing.assert_array_equal(alone.merged, batch[b].merged)
    assert batch[1].m == 0 and batch[1].merged.shape == (0, 8)
    assert batch[2].m == 1 and batch[2].r == 0


def test_whole_operator_counts_and_pass_through():
    rng = np.random.default_rng(21)
    X = rng.standard_normal((64, 24))
    res = orc.prune_image(X, 0.5, orc.Params(ratio=0.84, iters=10))
    assert res.m == 54 and res.merged.shape == (54, 24) and res.P.shape == (54, 10)
    full = orc.prune_image(X, 0.5, orc.Params(ratio=1.0))
    assert full.m == 64 and full.P_bar is None
    np.testing.assert_array_equal(full.merged, X)


def test_near_tie_bookkeeping():
    s = np.array([4.0, 3.0, 3.0 * (1 + 2.0 ** -22), 1.0], dtype=np.float32)
    assert orc.selection_gap(s, 1) > 0.2
    assert orc.selection_gap(s, 2) < 1e-6
    assert orc.selection_gap(s, 4) == math.inf
    P_bar = np.array([[0.5, 0.1, 0.0], [0.5 * (1 - 1e-7), 0.4, 0.0], [0.0, 0.5, 0.0]])
    g = orc.pairing_gaps(P_bar)
    assert g[0] < 1e-6 and 0.19 < g[1] < 0.21
