"""Pins for the oracle's stage 1 (Eq. 1, M = N(1-r)) and dynamic ratio (Eq. 7, 9)."""
import math
import os

import numpy as np
import pytest

from oracle import rtprune_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                out.append(line.split())
    return out


# ---------------------------------------------------------------- kept count
def test_kept_count_matches_counts_printed_in_the_paper():
    for mode, n, r, m, *_ in _rows("paper_token_counts.txt"):
        n, m, r = int(n), int(m), float(r)
        retention32 = np.float32(1.0 - r)
        assert orc.kept_count(retention32, n) == m, (mode, n, r)


def test_kept_count_benchmark_retention():
    for n, ret, m in _rows("benchmark_kept_counts.txt"):
        assert orc.kept_count(np.float32(float(ret)), int(n)) == int(m)


def test_kept_count_is_ceil_in_exact_decimal_arithmetic():
    from fractions import Fraction
    # retention given to two decimals; exact ceil via rationals
    for pct in range(1, 101):
        for n in (1, 2, 7, 64, 100, 256, 400, 456, 1083, 1156):
            exact = math.ceil(Fraction(pct, 100) * n)
            got = orc.kept_count(np.float32(pct / 100.0), n)
            assert got == max(1, exact), (pct, n)


def test_kept_count_float32_hair_above_integer():
    # float32(0.85) * 400 = 340.0000095...: must still be 340, not 341
    assert float(np.float32(0.85)) * 400 > 340.0
    assert orc.kept_count(np.float32(0.85), 400) == 340
    assert orc.kept_count(np.float32(1.0), 400) == 400
    assert orc.kept_count(np.float32(1e-6), 400) == 1
    assert orc.kept_count(np.float32(0.5), 0) == 0


# --------------------------------------------------------------------- norms
def test_norms_equal_library_norm():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((37, 129))
    np.testing.assert_allclose(orc.token_norms(X), np.linalg.norm(X, axis=1), rtol=1e-14)
    # hand value: (3, 4, 12) has norm 13
    assert orc.token_norms(np.array([[3.0, 4.0, 12.0]]))[0] == 13.0
    assert orc.selection_scores(np.array([[3.0, 4.0, 12.0]]))[0] == np.float32(169.0)


def test_selection_keeps_the_m_largest_and_sorts_ascending():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((50, 16)) * rng.lognormal(0, 0.5, size=(50, 1))
    s = orc.selection_scores(X)
    kept, prop = orc.select_topk(s, 20)
    assert len(kept) == 20 and len(prop) == 30
    assert list(kept) == sorted(kept) and list(prop) == sorted(prop)
    assert set(kept) | set(prop) == set(range(50)) and not (set(kept) & set(prop))
    assert s[kept].min() >= s[prop].max()
    # against numpy's sort of the norms themselves
    top = set(np.argsort(-np.linalg.norm(X, axis=1), kind="stable")[:20])
    assert set(kept) == top


def test_selection_tie_break_lowest_index():
    s = np.array([1, 5, 5, 5, 0, 5], dtype=np.float32)
    kept, prop = orc.select_topk(s, 2)
    assert list(kept) == [1, 2] and list(prop) == [0, 3, 4, 5]
    kept, _ = orc.select_topk(np.ones(7, dtype=np.float32), 3)
    assert list(kept) == [0, 1, 2]


def test_selection_permutation_invariance():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((64, 32)) * rng.lognormal(0, 0.5, size=(64, 1))
    kept, _ = orc.select_topk(orc.selection_scores(X), 40)
    perm = rng.permutation(64)
    keptp, _ = orc.select_topk(orc.selection_scores(X[perm]), 40)
    # token perm[k] of X sits at position k of X[perm]
    assert set(perm[keptp]) == set(kept)


def test_scaling_a_token_up_can_only_move_it_into_kept():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((30, 8))
    kept, prop = orc.select_topk(orc.selection_scores(X), 10)
    j = int(prop[0])
    X2 = X.copy()
    X2[j] *= 100.0
    kept2, _ = orc.select_topk(orc.selection_scores(X2), 10)
    assert j in kept2
    for k in kept:
        X3 = X.copy()
        X3[k] *= 3.0
        assert k in orc.select_topk(orc.selection_scores(X3), 10)[0]


# ----------------------------------------------------------------------- phi
def _phi_loops(X):
    n = len(X)
    tot = 0.0
    for i in range(n):
        for j in range(i + 1, n):
            ni = math.sqrt(sum(a * a for a in X[i]))
            nj = math.sqrt(sum(a * a for a in X[j]))
            tot += sum(a * b for a, b in zip(X[i], X[j])) / (ni * nj)
    return 2.0 * tot / (n * (n - 1))


def test_phi_equals_plain_double_loop():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((9, 5))
    assert abs(orc.inter_token_similarity(X) - _phi_loops(X.tolist())) < 1e-14


def test_phi_equals_closed_form_of_the_unit_vector_sum():
    rng = np.random.default_rng(6)
    for n, d in ((2, 3), (17, 40), (256, 64)):
        X = rng.standard_normal((n, d)) + 0.3
        U = X / np.linalg.norm(X, axis=1, keepdims=True)
        closed = (np.linalg.norm(U.sum(axis=0)) ** 2 - n) / (n * (n - 1))
        assert abs(orc.inter_token_similarity(X) - closed) < 1e-12


def test_phi_special_cases():
    t = np.array([0.3, -1.2, 2.0, 0.1])
    same = np.tile(t, (7, 1)) * np.arange(1, 8)[:, None]       # same direction
    assert abs(orc.inter_token_similarity(same) - 1.0) < 1e-14
    assert abs(orc.inter_token_similarity(np.eye(6) * 3.0)) < 1e-15        # orthogonal
    n = 8
    anti = np.concatenate([np.eye(n // 2), -np.eye(n // 2)])               # antipodal pairs
    assert abs(orc.inter_token_similarity(anti) + 1.0 / (n - 1)) < 1e-15
    assert orc.inter_token_similarity(np.ones((1, 4))) == 0.0
    # a zero token has cosine 0 with everything: 3 identical + 1 zero -> 3 of 6 pairs
    X = np.array([[1.0, 1.0], [2.0, 2.0], [3.0, 3.0], [0.0, 0.0]])
    assert abs(orc.inter_token_similarity(X) - 0.5) < 1e-14


# --------------------------------------------------------------------- ratio
def test_dynamic_retention_hand_values():
    p = orc.Params(dynamic=1)
    # phi = 0.3, rho = 0.4 -> r = 0.3 * 0.6 = 0.18 -> retention 0.82
    assert abs(float(orc.dynamic_retention(0.3, 0.4, p)) - 0.82) < 1e-6
    # dense text (rho = 1) or dissimilar tokens (phi <= 0) prune nothing
    assert float(orc.dynamic_retention(0.9, 1.0, p)) == 1.0
    assert float(orc.dynamic_retention(-0.2, 0.0, p)) == 1.0
    # homogeneous blank page: r = 1 -> clamp at ratio_min
    assert float(orc.dynamic_retention(1.0, 0.0, p)) == float(np.float32(0.6))
    # affine normalisation with (lo, hi) = (0, 0.2): phi = 0.05 -> f = 0.25
    q = orc.Params(dynamic=1, phi_lo=0.0, phi_hi=0.2)
    assert abs(float(orc.dynamic_retention(0.05, 0.2, q)) - (1 - 0.25 * 0.8)) < 1e-6
    assert float(orc.dynamic_retention(0.5, 0.0, q)) == float(np.float32(0.6))
    # monotone: more similar -> keep fewer; denser text -> keep more
    a = [float(orc.dynamic_retention(x, 0.3, p)) for x in np.linspace(0, 0.5, 11)]
    assert all(x >= y for x, y in zip(a, a[1:]))
    b = [float(orc.dynamic_retention(0.3, x, p)) for x in np.linspace(0, 1, 11)]
    assert all(x <= y for x, y in zip(b, b[1:]))


def test_dynamic_ratio_range_printed_in_the_paper_is_reachable():
    # Table 8 prints average r_dyn of 0.17 .. 0.30; with f_normalize = clamp01
    # those need phi (1 - rho) in that range, e.g. phi = 0.4, rho = 0.5.
    p = orc.Params(dynamic=1)
    r = 1.0 - float(orc.dynamic_retention(0.4, 0.5, p))
    assert 0.17 <= r <= 0.30


# ----------------------------------------------------------- bf16 round-trip
def test_round_to_bf16_against_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    x[:8] = [0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e38, 1e-30, -0.0]
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.round_to_bf16(x.astype(np.float64))
    np.testing.assert_array_equal(got, want)
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert orc.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert orc.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # a float64 just above the tie rounds up (no double rounding through float32)
    assert orc.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7


def test_widen_bf16_is_exact():
    torch = pytest.importorskip("torch")
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    bits = bits[(bits & 0x7F80) != 0x7F80]                     # skip inf / nan
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(orc.widen(bits, "bf16"), want)


# ------------------------------------------------- variance metric (Table 7 ablation)
def test_variance_hand_values_and_library():
    # (1, 2, 3, 4): mean 2.5, squared deviations 2.25 .25 .25 2.25 -> 5/4
    assert orc.token_variances(np.array([[1.0, 2.0, 3.0, 4.0]]))[0] == 1.25
    assert orc.token_variances(np.array([[7.0, 7.0, 7.0]]))[0] == 0.0
    rng = np.random.default_rng(11)
    X = rng.standard_normal((23, 77)) * 3 + 5
    np.testing.assert_allclose(orc.token_variances(X), np.var(X, axis=1), rtol=1e-13)
    # identity E[x^2] - E[x]^2, evaluated in exact rational arithmetic on small integers
    from fractions import Fraction
    Xi = rng.integers(-9, 10, size=(5, 12))
    for row, v in zip(Xi, orc.token_variances(Xi.astype(np.float64))):
        ex2 = Fraction(int((row * row).sum()), 12)
        ex = Fraction(int(row.sum()), 12)
        assert abs(v - float(ex2 - ex * ex)) < 1e-13


def test_variance_shift_and_scale():
    rng = np.random.default_rng(12)
    X = rng.standard_normal((9, 64))
    v = orc.token_variances(X)
    np.testing.assert_allclose(orc.token_variances(X + 3.5), v, rtol=1e-12)      # a feature shift leaves it
    np.testing.assert_allclose(orc.token_variances(-2.0 * X), 4.0 * v, rtol=1e-12)
    # squared norm = D (variance + mean^2): the two metrics differ exactly by the mean term
    np.testing.assert_allclose(orc.token_sqnorms(X), 64 * (v + X.mean(axis=1) ** 2), rtol=1e-12)


def test_variance_misses_a_token_whose_norm_comes_from_a_feature_shift():
    # what Sec. 4.4 says of the variance metric: a token that is large because all
    # features moved together has a large norm and an ordinary variance
    rng = np.random.default_rng(13)
    X = rng.standard_normal((20, 256))
    X[7] = 0.5 * X[7] + 4.0                     # norm ~ 64, variance ~ 0.25
    l2_kept, _ = orc.select_topk(orc.selection_scores(X, orc.METRIC_L2NORM), 5)
    var_kept, _ = orc.select_topk(orc.selection_scores(X, orc.METRIC_VARIANCE), 5)
    assert 7 in l2_kept and 7 not in var_kept
    assert int(np.argmin(orc.selection_scores(X, orc.METRIC_VARIANCE))) == 7
    with pytest.raises(ValueError):
        orc.selection_scores(X, 2)


def test_metric_only_changes_the_selection_step():
    rng = np.random.default_rng(14)
    X = rng.standard_normal((30, 48)) + rng.standard_normal((30, 1))
    p0 = orc.Params(iters=5, ratio=0.7)
    p1 = orc.Params(iters=5, ratio=0.7, metric=orc.METRIC_VARIANCE)
    a, b = orc.prune_image(X, 0.0, p0), orc.prune_image(X, 0.0, p1)
    assert a.m == b.m == 21
    exp_kept, _ = orc.select_topk(orc.token_variances(X).astype(np.float32), 21)
    np.testing.assert_array_equal(b.kept, exp_kept)
    assert not np.array_equal(a.kept, b.kept)
    # stage 2 of the variance run is the l2 run's stage 2 on the other split: cosines
    # still use the l2 norms
    np.testing.assert_allclose(b.S, orc.cosine_scores(X, b.kept, b.prop), rtol=0, atol=0)
    G = (X / np.linalg.norm(X, axis=1, keepdims=True))
    np.testing.assert_allclose(b.S, (G @ G.T)[np.ix_(b.kept, b.prop)], atol=1e-14)
