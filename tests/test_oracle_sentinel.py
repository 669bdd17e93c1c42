"""Pins for oracle/sentinel_oracle.py: sliced Wasserstein distance, Tukey fences, the adaptive
multiplier of Alg. adaptive_iqr and the violation / ban bookkeeping of Alg. activation_verification.
Every expected value here comes from a closed form, a brute force over permutations, a library
routine that works differently (CDF integration), or a hand-worked example."""
import itertools

import numpy as np
import pytest
from scipy.stats import wasserstein_distance

from oracle import sentinel_oracle as so


def _dirs(L, D, seed):
    u = np.random.default_rng(seed).standard_normal((L, D))
    return u / np.linalg.norm(u, axis=1, keepdims=True)


# ------------------------------------------------------------------ sliced Wasserstein
def test_sw_one_dimension_matches_cdf_integration():
    rng = np.random.default_rng(0)
    a, b = rng.standard_normal(37), 0.5 + 1.7 * rng.standard_normal(37)
    want = wasserstein_distance(a, b)                      # integrates |F_a - F_b|
    got = so.sliced_wasserstein(a[:, None], b[:, None], np.ones((1, 1)))
    assert got == pytest.approx(want, rel=1e-12)


def test_sw_equals_optimal_matching_cost_by_brute_force():
    rng = np.random.default_rng(1)
    T, D, L = 6, 3, 4
    a, b, u = rng.standard_normal((T, D)), rng.standard_normal((T, D)) * 2 + 0.3, _dirs(L, D, 2)
    total = 0.0
    for l in range(L):
        pa, pb = a @ u[l], b @ u[l]
        total += min(np.mean(np.abs(pa - pb[list(p)])) for p in itertools.permutations(range(T)))
    assert so.sliced_wasserstein(a, b, u) == pytest.approx(total / L, rel=1e-12)


def test_sw_closed_forms_and_invariances():
    rng = np.random.default_rng(3)
    T, D, L = 50, 8, 16
    r, u = rng.standard_normal((T, D)), _dirs(L, D, 4)
    assert so.sliced_wasserstein(r, r, u) == 0.0
    # translation of every sample by v: each projection shifts by v.u
    v = rng.standard_normal(D)
    assert so.sliced_wasserstein(r + v, r, u) == pytest.approx(np.mean(np.abs(u @ v)), rel=1e-12)
    # positive scaling keeps the order of the projected samples
    assert so.sliced_wasserstein(1.5 * r, r, u) == pytest.approx(0.5 * np.mean(np.abs(r @ u.T)), rel=1e-12)
    # a distance between sample SETS: permuting the tokens of one side changes nothing
    c = r + 0.1 * rng.standard_normal((T, D))
    base = so.sliced_wasserstein(c, r, u)
    assert so.sliced_wasserstein(c[rng.permutation(T)], r, u) == pytest.approx(base, rel=1e-12)
    assert so.sliced_wasserstein(r, c, u) == pytest.approx(base, rel=1e-12)            # symmetric
    # ... while negating the samples of a symmetric-looking cloud is NOT seen as an element-wise change
    assert so.sliced_wasserstein(-r, r, u) < np.mean(np.abs(r @ u.T))
    # triangle inequality per direction carries over to the mean
    d2 = r + rng.standard_normal((T, D))
    assert so.sliced_wasserstein(c, d2, u) <= so.sliced_wasserstein(c, r, u) + so.sliced_wasserstein(r, d2, u) + 1e-12
    # leading dimensions are flattened into samples
    assert so.sliced_wasserstein(c.reshape(5, 10, D), r.reshape(5, 10, D), u) == pytest.approx(base, rel=1e-15)


def test_sw_direction_axis_is_the_feature_axis():
    # two samples in R^2, one direction e_x: only the x coordinates matter
    a = np.array([[0.0, 100.0], [1.0, -100.0]])
    b = np.array([[3.0, 0.0], [2.0, 0.0]])
    assert so.sliced_wasserstein(a, b, np.array([[1.0, 0.0]])) == pytest.approx(2.0)     # sorted x: (0,1) vs (2,3)
    assert so.sliced_wasserstein(a, b, np.array([[0.0, 1.0]])) == pytest.approx(100.0)   # sorted y: (-100,100) vs (0,0)


# ------------------------------------------------------------------ percentiles / fences
def test_percentiles_textbook_cases():
    assert so.percentiles(range(1, 10)) == (3.0, 5.0, 7.0)
    assert so.percentiles([4, 1, 3, 2]) == pytest.approx((1.75, 2.5, 3.25))
    assert so.percentiles([7.0]) == (7.0, 7.0, 7.0)
    h = np.random.default_rng(5).standard_normal(101)
    assert so.percentiles(h) == pytest.approx(tuple(np.percentile(h, [25, 50, 75])))
    hs = np.sort(h)
    assert so.percentiles(h) == (hs[25], hs[50], hs[75])         # n = 101: exact order statistics


def test_tukey_fence_is_inclusive_and_centred_on_the_median():
    q1, q2, q3 = 3.0, 5.0, 7.0
    assert so.tukey_flag(11.0, q1, q2, q3, 1.5)                    # |11 - 5| = 6 = 1.5 * 4
    assert so.tukey_flag(-1.0, q1, q2, q3, 1.5)
    assert not so.tukey_flag(10.999, q1, q2, q3, 1.5)
    assert not so.tukey_flag(5.0, q1, q2, q3, 1.5)


# ------------------------------------------------------------------ Alg. adaptive_iqr
def test_adaptive_iqr_hand_worked_example():
    """history 0..100: q1, q2, q3 = 25, 50, 75, IQR 50.  k0 = 0.5 -> fences [25, 75], 50 of 101
    outside (0.495 > 0.2) -> k = 0.75 -> [12.5, 87.5], 26 outside (0.257 > 0.2) -> k = 1.125 ->
    nothing outside.  Then 0 < 0.02: shrink by 0.8 -> k = 0.9 -> [5, 95], 10 outside (0.099), stop."""
    lo, up, k = so.adaptive_iqr(np.arange(101.0), 0.5, alpha=0.2, grow=1.5, shrink=0.8, n_max=10,
                                min_dist_mult=0.0, eps=1e-3)
    assert k == pytest.approx(0.9) and lo == pytest.approx(5.0) and up == pytest.approx(95.0)


def test_adaptive_iqr_keeps_k_inside_the_band():
    # 1 of 21 values outside the fences: 0.0476 lies in [alpha/10, alpha] for alpha = 0.1: k stays
    h = np.concatenate([np.linspace(-1, 1, 20), [50.0]])
    lo, up, k = so.adaptive_iqr(h, 1.5, alpha=0.1, grow=1.1, shrink=0.9, n_max=10, min_dist_mult=0.0, eps=1e-6)
    q1, q2, q3 = so.percentiles(h)
    assert k == 1.5 and lo == pytest.approx(q2 - 1.5 * (q3 - q1)) and up == pytest.approx(q2 + 1.5 * (q3 - q1))


def test_adaptive_iqr_widening_is_minimal_and_bounded():
    h = np.random.default_rng(6).standard_normal(400)
    q1, q2, q3 = so.percentiles(h)
    iqr = q3 - q1
    alpha, grow = 0.01, 1.1
    lo, up, k = so.adaptive_iqr(h, 0.5, alpha, grow, 1.0 - 1e-12, n_max=50, min_dist_mult=0.0, eps=1e-9)
    # shrink factor ~1 makes the narrowing phase a no-op: k is k0 * grow^j for the smallest j that works
    j = round(np.log(k / 0.5) / np.log(grow))
    assert k == pytest.approx(0.5 * grow ** j, rel=1e-9) and j >= 1
    outside = lambda kk: np.mean(np.abs(h - q2) > kk * iqr)
    assert outside(0.5 * grow ** j) <= alpha < outside(0.5 * grow ** (j - 1))
    # the iteration cap binds
    _, _, k3 = so.adaptive_iqr(h, 0.5, alpha, grow, 1.0 - 1e-12, n_max=3, min_dist_mult=0.0, eps=1e-9)
    assert k3 == pytest.approx(0.5 * grow ** 3, rel=1e-9)


def test_adaptive_iqr_degenerate_history_and_minimum_distance():
    # constant history: IQR = eps, nothing ever outside, the narrowing loop runs n_max times
    lo, up, k = so.adaptive_iqr(np.full(30, 10.0), 3.0, alpha=0.01, grow=1.1, shrink=0.9, n_max=10,
                                min_dist_mult=0.0, eps=0.01)
    assert k == pytest.approx(3.0 * 0.9 ** 10)
    assert lo == pytest.approx(10.0 - k * 0.01) and up == pytest.approx(10.0 + k * 0.01)
    # minimum distance |q2| * Lambda from the median overrides tighter fences, never looser ones
    lo, up, _ = so.adaptive_iqr(np.full(30, 10.0), 3.0, 0.01, 1.1, 0.9, 10, min_dist_mult=0.35, eps=0.01)
    assert lo == pytest.approx(6.5) and up == pytest.approx(13.5)
    lo, up, k = so.adaptive_iqr(np.full(30, -10.0), 3.0, 0.01, 1.1, 0.9, 0, min_dist_mult=0.001, eps=1.0)
    assert (lo, up, k) == pytest.approx((-13.0, -7.0, 3.0))


# ------------------------------------------------------------------ violation counters, bans, taint
def _policy(**kw):
    # eps = 1000 pins IQR to 1000; n_max = 0 freezes k = 1: the fences are median -/+ 1000
    args = dict(c=5, t_forgive=100, window=10_000, k0=1.0, alpha=0.01, grow=1.1, shrink=0.9, n_max=0,
                min_dist_mult=0.0, eps=1000.0)
    args.update(kw)
    p = so.StagePolicy(4, 2, **args)
    p.warmup(np.full((4, 2), 50.0))
    return p


def test_policy_nothing_flagged_before_history_exists():
    p = so.StagePolicy(3, 1)
    assert p.step(np.array([[1e9], [0.0], [-1e9]])) == []
    assert p.v == [0, 0, 0] and len(p.hist[0]) == 3


def test_policy_ban_after_c_violations_and_fence_is_inclusive():
    p = _policy()
    g = np.full((4, 2), 50.0)
    g[2, 1] = 1050.0                                   # exactly on the upper fence: flagged
    for it in range(5):
        assert p.step(g) == [2]
        assert p.v[2] == it + 1 and p.banned[2] == (it == 4)
    assert p.step(g) == []                             # a banned worker is no longer examined
    g[1, 0] = 1049.0                                   # inside
    assert p.step(g) == [] and p.v[1] == 0


def test_policy_severe_deviation_bans_at_once():
    p = _policy()
    g = np.full((4, 2), 50.0)
    g[0, 0] = 50.0 - 100.0 * 1000.0                    # 100 x the fence half-width below the median
    assert p.step(g) == [0] and p.banned[0] and p.v[0] == 1
    g[1, 0] = 50.0 + 99_999.0
    assert p.step(g) == [1] and not p.banned[1]


def test_policy_forgiveness_after_consecutive_clean_steps():
    p = _policy(t_forgive=3)
    bad, good = np.full((4, 2), 50.0), np.full((4, 2), 50.0)
    bad[3, 0] = 5000.0
    p.step(bad); p.step(bad)
    assert p.v[3] == 2
    p.step(good); p.step(good)
    assert p.v[3] == 2                                 # two clean steps: not yet
    p.step(bad)                                        # streak broken
    assert p.v[3] == 3
    p.step(good); p.step(good); p.step(good)
    assert p.v[3] == 2
    p.step(good); p.step(good); p.step(good)
    assert p.v[3] == 1 and p.v[0] == 0                 # counters never go below zero


def test_policy_history_takes_clean_values_only_and_majority_flag_clears_taint():
    p = _policy()
    n0 = len(p.hist[0])
    g = np.full((4, 2), 60.0)
    g[1, 0] = 9999.0
    assert p.step(g) == [1]
    assert len(p.hist[0]) == n0 + 3 and 9999.0 not in p.hist[0]
    # three of four flagged: read as a natural shift, the tainted set is dropped (counters stay)
    g = np.full((4, 2), 9999.0)
    g[0] = 60.0
    assert p.step(g) == []
    assert p.v == [0, 2, 1, 1]
    # skip mask: worker 2 is tainted upstream, not examined, its value does not enter the history
    g = np.full((4, 2), 61.0)
    g[2] = 9999.0
    n1 = len(p.hist[1])
    assert p.step(g, skip=[False, False, True, False]) == []
    assert p.v[2] == 1 and len(p.hist[1]) == n1 + 3


def test_policy_history_is_cut_at_the_start_of_a_call_not_before_the_fences_are_adapted():
    """Alg. activation_verification cuts the history to its last l values in its second line, then appends this call's
    clean values, then runs Alg. adaptive_iqr: the quartiles at the end of a call come from up to l + d values.
    Hand-worked with l = 4, d = 4, k frozen at 100 (n_max = 0) so that nothing is flagged:
      warm-up (1, 2, 3, 4)              -> q2 = 2.5, IQR = 1.5, fences 2.5 -/+ 150
      call 1 adds (10, 11, 12, 13)      -> the EIGHT values 1, 2, 3, 4, 10, 11, 12, 13: positions 1.75 / 3.5 / 5.25 give
                                           q1 = 2.75, q2 = 7, q3 = 11.25, IQR = 8.5, fences 7 -/+ 850
                                           (cutting before adapting would leave 10..13: q2 = 11.5, IQR = 1.5)
      call 2 cuts to (10, 11, 12, 13), adds (20, 21, 22, 23) -> q1 = 11.75, q2 = 16.5, q3 = 21.25, IQR = 9.5."""
    p = so.StagePolicy(4, 1, window=4, k0=100.0, n_max=0, eps=1e-9, min_dist_mult=0.0)
    p.warmup(np.array([[1.0], [2.0], [3.0], [4.0]]))
    assert (p.q2[0], p.iqr[0]) == (2.5, 1.5) and (p.lower[0], p.upper[0]) == (-147.5, 152.5)
    assert p.step(np.array([[10.0], [11.0], [12.0], [13.0]])) == []
    assert p.hist[0] == [1.0, 2.0, 3.0, 4.0, 10.0, 11.0, 12.0, 13.0]
    assert (p.q2[0], p.iqr[0]) == (7.0, 8.5) and (p.lower[0], p.upper[0]) == (-843.0, 857.0)
    assert p.step(np.array([[20.0], [21.0], [22.0], [23.0]])) == []
    assert p.hist[0] == [10.0, 11.0, 12.0, 13.0, 20.0, 21.0, 22.0, 23.0]
    assert (p.q2[0], p.iqr[0]) == (16.5, 9.5)
    # a warm-up iteration keeps at most l values (it has no later call to cut for it)
    w = so.StagePolicy(4, 1, window=4, k0=100.0, n_max=0, eps=1e-9)
    w.warmup(np.array([[1.0], [2.0], [3.0], [4.0]]))
    w.warmup(np.array([[5.0], [6.0], [7.0], [8.0]]))
    assert w.hist[0] == [5.0, 6.0, 7.0, 8.0] and w.q2[0] == 6.5


def test_policy_window_and_adaptation_track_a_drifting_statistic():
    # the minimum-distance multiplier (0.15 |median|, as in the paper's configuration table) keeps the
    # fences from collapsing onto a history that only ever receives un-flagged values
    p = so.StagePolicy(8, 1, window=100, k0=1.5, alpha=0.01, grow=1.1, shrink=0.9, n_max=10, eps=1e-4,
                       min_dist_mult=0.15)
    rng = np.random.default_rng(7)
    for t in range(20):
        p.warmup(1.0 + 0.01 * rng.standard_normal((8, 1)))
    flagged = 0
    for t in range(200):                               # slow benign drift of the statistic
        flagged += len(p.step(1.0 + 0.002 * t + 0.01 * rng.standard_normal((8, 1))))
    assert len(p.hist[0]) <= 100 + 8
    assert flagged == 0 and not any(p.banned)
    assert 1.3 < p.q2[0] < 1.45 and p.lower[0] < 1.4 < p.upper[0]      # the fences followed the drift
    assert p.upper[0] - p.q2[0] == pytest.approx(0.15 * p.q2[0])         # ... at the minimum distance
    g = 1.4 + 0.01 * rng.standard_normal((8, 1))
    g[5] = 3.0
    assert p.step(g) == [5]


# ------------------------------------------------------------------ the whole-signal statistics of the loop
def test_global_scores_closed_forms_for_every_column():
    """Paragraph "Choice of Distance Measure": each column of global_scores against a value that follows from the
    definition for a constructed pair, so that a slip in any one column (a missing square root, the wrong
    denominator, a sample instead of a population deviation, a sign convention) fails here."""
    rng = np.random.default_rng(21)
    r = rng.standard_normal((7, 33)) + 0.4                 # a reference with a mean, so centring matters
    n = r.size
    # the signal itself: every statistic is 0
    assert so.global_scores(r, r) == {"rel_l2": 0.0, "l1": 0.0, "zl2": 0.0, "sfr": 0.0}
    # claim = alpha r: relative L2 |alpha - 1|, mean absolute difference |alpha - 1| mean|r|; the z-scores coincide
    # for alpha > 0 and are mirrored for alpha < 0 (mean of (2 z)^2 = 4); every sign kept / flipped
    for alpha in (1.5, 0.25, -1.0, -3.0):
        sc = so.global_scores(alpha * r, r)
        assert sc["rel_l2"] == pytest.approx(abs(alpha - 1.0), rel=1e-12)
        assert sc["l1"] == pytest.approx(abs(alpha - 1.0) * np.mean(np.abs(r)), rel=1e-12)
        assert sc["zl2"] == pytest.approx(0.0 if alpha > 0 else 4.0, abs=1e-12)
        assert sc["sfr"] == (0.0 if alpha > 0 else 1.0)
    # a zeroed claim: relative L2 exactly 1, and sign(0) = 0 differs from every non-zero sign
    z = so.global_scores(np.zeros_like(r), r)
    assert z["rel_l2"] == pytest.approx(1.0, rel=1e-15) and z["sfr"] == 1.0 and z["l1"] == pytest.approx(np.mean(np.abs(r)))
    # a perturbation orthogonal to r with a chosen norm: relative L2 is the ratio of the two norms (Pythagoras does
    # not enter: the numerator is the difference alone)
    d = rng.standard_normal(r.shape)
    d -= r * np.sum(d * r) / np.sum(r * r)
    d *= 0.3 * np.linalg.norm(r) / np.linalg.norm(d)
    assert so.global_scores(r + d, r)["rel_l2"] == pytest.approx(0.3, rel=1e-12)
    # the relative L2 is NOT symmetric: the denominator is the reference's norm
    assert so.global_scores(r, 2.0 * r)["rel_l2"] == pytest.approx(0.5, rel=1e-12)
    assert so.global_scores(2.0 * r, r)["rel_l2"] == pytest.approx(1.0, rel=1e-12)


def test_global_scores_zscore_column_is_two_minus_two_rho():
    """Both signals whitened by their own scalar mean and POPULATION deviation over the flattened tensor: the mean
    squared difference is 2 (1 - rho) with Pearson's rho, here from numpy's corrcoef (a covariance-matrix routine)
    and from a scalar loop; with sample deviations (n - 1) the value would be (n - 1) / n times that, which the
    last-but-one group of assertions separates from the exact identity at these sizes."""
    rng = np.random.default_rng(22)
    for shape in ((4, 5), (3, 11, 6)):
        r = 2.0 + rng.standard_normal(shape)
        c = 0.7 * r + 0.6 * rng.standard_normal(shape) - 1.0
        rho = np.corrcoef(c.ravel(), r.ravel())[0, 1]
        got = so.global_scores(c, r)["zl2"]
        assert got == pytest.approx(2.0 * (1.0 - rho), rel=1e-12)
        # scalar loop of the definition
        cf, rf = c.ravel().tolist(), r.ravel().tolist()
        n = len(cf)
        mc, mr = sum(cf) / n, sum(rf) / n
        sc_, sr_ = (sum((x - mc) ** 2 for x in cf) / n) ** 0.5, (sum((x - mr) ** 2 for x in rf) / n) ** 0.5
        loop = sum(((x - mc) / sc_ - (y - mr) / sr_) ** 2 for x, y in zip(cf, rf)) / n
        assert got == pytest.approx(loop, rel=1e-12)
        # with sample deviations the value would be smaller by (n - 1) / n: the pin tells the two apart
        assert abs(got - loop * (n - 1) / n) > 1e-3 * got
        # whitening removes any positive affine map of either side; a negative scale mirrors the z-scores
        assert so.global_scores(3.0 * c + 7.0, r)["zl2"] == pytest.approx(got, rel=1e-12)
        assert so.global_scores(c, 0.1 * r - 2.0)["zl2"] == pytest.approx(got, rel=1e-12)
        assert so.global_scores(-c, r)["zl2"] == pytest.approx(2.0 * (1.0 + rho), rel=1e-12)
        # uncorrelated by construction: exactly 2
        e = rng.standard_normal(shape)
        e -= e.mean()
        rc = r - r.mean()
        e -= rc * np.sum(e * rc) / np.sum(rc * rc)
        assert so.global_scores(e, r)["zl2"] == pytest.approx(2.0, rel=1e-12)


def test_global_scores_constant_signals_have_no_zscore():
    """A constant tensor has deviation 0 and no z-score: both constant -> 0 (nothing to tell apart), exactly one
    constant -> 2 (the value of an uncorrelated pair); the other columns keep their plain definitions."""
    r = np.random.default_rng(23).standard_normal((5, 8))
    k3, k5 = np.full((5, 8), 3.0), np.full((5, 8), 5.0)
    assert so.global_scores(k3, k5)["zl2"] == 0.0 and so.global_scores(k3, k3)["zl2"] == 0.0
    assert so.global_scores(k3, r)["zl2"] == 2.0 and so.global_scores(r, k3)["zl2"] == 2.0
    sc = so.global_scores(k3, k5)
    assert sc["rel_l2"] == pytest.approx(2.0 / 5.0) and sc["l1"] == pytest.approx(2.0) and sc["sfr"] == 0.0
    # the first warm-up step compares against m_0 = 0: the guarded denominator, every sign differs from sign(0)
    sc0 = so.global_scores(r, np.zeros_like(r))
    assert sc0["rel_l2"] == pytest.approx(np.linalg.norm(r) / 1e-30) and sc0["sfr"] == 1.0 and sc0["zl2"] == 2.0


# ------------------------------------------------------------------ Alg. momentum_verification end to end
import stage_inputs as si

P, DW, T, D = 3, 6, 32, 64
POLICY = dict(c=5, t_forgive=100, window=100, k0=1.5, alpha=0.01, grow=1.1, shrink=0.9, n_max=10, min_dist_mult=0.35, eps=1e-4)


def _stream(metrics=("rel_l2", "l1", "zl2", "sfr", "sw")):
    return so.SentinelStream(P, DW, (T, D), metrics, si.make_directions(D, 32, 0), 0.9, 0.8, POLICY, POLICY)


def _signals(kind, s, t, attack=None):
    """attack = (stage, worker, kind): that worker's signal is corrupted; in the forward pass the same
    pipe's later stages carry a contaminated (noisy) signal as well."""
    out = [si.stream_signal(kind, s, r, t, T, D, "f32") for r in range(DW)]
    if attack is not None:
        a_s, a_r, a_kind = attack
        if s == a_s:
            out[a_r] = si.make_claim(a_kind, out[a_r], "f32", seed=t)
        elif kind == "h" and s > a_s:
            out[a_r] = si.make_claim("noise", out[a_r] * 1.2, "f32", seed=t)
    return out


def _run(st, t, warm, attack_h=None, attack_g=None):
    st.begin_iteration(warm)
    rec = {"h": [], "g": [None] * P, "out": [None] * P, "m_g_before": [m.copy() for m in st.m["g"]]}
    for s in range(P):
        rec["h"].append(st.forward(s, _signals("h", s, t, attack_h))[0])
    for s in reversed(range(P)):
        g = _signals("g", s, t, attack_g)
        here, _, out = st.backward(s, g)
        rec["g"][s], rec["out"][s], rec.setdefault("g_in", {})[s] = here, out, g
    return rec


def test_stream_warmup_ema_closed_form_and_nothing_flagged():
    st = _stream(metrics=("l1", "sfr"))
    x = si.stream_signal("h", 0, 0, 0, T, D, "f32").astype(np.float64)
    for t in range(6):
        st.begin_iteration(True)
        here, gam = st.forward(0, [x] * DW)
        assert here == [] and gam.shape == (DW, 2)
        np.testing.assert_allclose(st.m["h"][0], (1 - 0.9 ** (t + 1)) * x, rtol=1e-12)
        # the statistic of x against (1 - beta^t) x: mean |x| beta^t and no sign flips (first step: reference 0)
        assert gam[0, 0] == pytest.approx(0.9 ** t * np.mean(np.abs(x)), rel=1e-12)
        assert gam[0, 1] == (1.0 if t == 0 else 0.0)
    assert len(st.pol["h"][0].hist[0]) == 6 * DW and st.pol["h"][0].v == [0] * DW


WARM = 40      # iterations until the EMAs (beta 0.9 / 0.8, m_0 = 0) have converged and the 100-value windows hold settled values


def _warm(st):
    for t in range(WARM):
        _run(st, t, True)


def test_stream_activation_attack_is_caught_and_does_not_cascade():
    st = _stream()
    _warm(st)
    for t in range(WARM, WARM + 2):
        rec = _run(st, t, False)
        assert rec["h"] == [[], [], []] and rec["g"] == [[], [], []]
    m_h1 = st.m["h"][1].copy()
    attack = (1, 2, "sign")
    for n_att, t in enumerate(range(WARM + 2, WARM + 7), start=1):
        rec = _run(st, t, False, attack_h=attack)
        # caught where it happens; the contaminated later stage of the same pipe is neither examined nor blamed
        assert rec["h"] == [[], [2], []]
        assert st.pol["h"][1].v[2] == n_att and st.pol["h"][2].v[2] == 0
        # the EMA of stage 1 is the mean of the five other workers
        sig = _signals("h", 1, t, attack)
        m_h1 = 0.9 * m_h1 + 0.1 * np.mean([np.float64(sig[r]) for r in range(DW) if r != 2], axis=0)
        np.testing.assert_allclose(st.m["h"][1], m_h1, rtol=1e-12, atol=1e-15)
        # backward: stage 2 examines the pipe as usual (its gradient is honest here); stage 1 holds the forward
        # taint and stage 0 sees it as tainted downstream: both hand on the gradient EMA of before this iteration
        assert rec["g"] == [[2], [], []]
        for s in (0, 1):
            assert np.array_equal(rec["out"][s][2], rec["m_g_before"][s])
            assert all(rec["out"][s][r] is rec["g_in"][s][r] for r in range(DW) if r != 2)
        assert all(rec["out"][2][r] is rec["g_in"][2][r] for r in range(DW))
    assert st.pol["h"][1].banned[2]                       # fifth violation
    assert not st.pol["g"][0].banned[2] and st.pol["g"][0].v[2] == 0    # marked, never examined, never blamed
    rec = _run(st, WARM + 7, False, attack_h=attack)
    assert rec["h"][1] == []                              # a banned worker is no longer collected


def test_stream_gradient_attack_taints_upstream_stages_only():
    st = _stream()
    _warm(st)
    rec = _run(st, WARM, False, attack_g=(1, 4, "scale"))
    assert rec["h"] == [[], [], []]
    assert rec["g"][2] == [] and rec["g"][1] == [4] and rec["g"][0] == [4]
    assert np.array_equal(rec["out"][1][4], rec["m_g_before"][1]) and np.array_equal(rec["out"][0][4], rec["m_g_before"][0])
    assert st.pol["g"][1].v[4] == 1 and st.pol["g"][0].v[4] == 0
    # severe deviation: banned at once
    rec = _run(st, WARM + 1, False, attack_g=(2, 0, "zero"))
    big = [x.copy() for x in _signals("g", 2, WARM + 2)]
    big[3] = big[3] * 1e6
    st.begin_iteration(False)
    for s in range(P):
        st.forward(s, _signals("h", s, WARM + 2))
    here, gam, out = st.backward(2, big)
    assert here == [3] and st.pol["g"][2].banned[3] and st.pol["g"][2].v[3] == 1


def test_stream_majority_deviation_is_a_distribution_shift():
    st = _stream(metrics=("l1", "zl2"))
    _warm(st)
    st.begin_iteration(False)
    h = _signals("h", 0, WARM)
    for r in range(4):                                    # four of six shift together
        h[r] = h[r] * 1.5
    m0 = st.m["h"][0].copy()
    here, _ = st.forward(0, h)
    assert here == [] and st.tainted == set()
    assert st.pol["h"][0].v == [1, 1, 1, 1, 0, 0]         # the listing clears the set, not the counters
    # ... and the listing's clean set then lets nobody in that was flagged: only the two un-flagged enter the EMA? No:
    # the set was emptied, so every worker of the stage is clean again.
    np.testing.assert_allclose(st.m["h"][0], 0.9 * m0 + 0.1 * np.mean([np.float64(x) for x in h], axis=0), rtol=1e-12, atol=1e-15)


# ------------------------------------------------------------------ the remaining attack generators
def test_attack_generators_have_the_stated_statistics():
    x = si.stream_signal("h", 0, 0, 0, 512, 64, "f32")
    assert si.invisible_noise_zmax(0.99) == pytest.approx(2.3263478740, rel=1e-9)      # 99 % quantile of N(0, 1)
    assert si.invisible_noise_zmax(0.5) == pytest.approx(0.0, abs=1e-12)
    y = si.attack_invisible_noise(x, 0.99, 1, "f32").astype(np.float64)
    np.testing.assert_allclose(y.mean(axis=0), x.mean(axis=0), atol=0.4)
    assert np.mean(y.std(axis=0) / x.std(axis=0)) == pytest.approx(2.3263, rel=0.03)
    s = si.attack_sign_elements(x, 0.25, 2, "f32")
    assert np.all(np.abs(s) == np.abs(x)) and np.mean(s != x) == pytest.approx(0.25, abs=0.02)
    assert np.all(si.attack_constant(x, -1.0, "bf16") == -1.0)
    r = si.attack_random_value(x, 3, "f32")
    assert abs(r.mean()) < 0.02 and r.std() == pytest.approx(1.0, rel=0.02)
    m, tgt = x.astype(np.float64), np.ones_like(x, dtype=np.float64)
    d = si.attack_drift(m, tgt, alpha=0.5, sigma=0.0, seed=0, dtype="f32")
    np.testing.assert_allclose(d, m + 0.5 * (tgt - m) / np.linalg.norm(m), rtol=1e-6, atol=1e-7)
    assert si.drift_delay(0.9) == 22 and si.drift_delay(0.8) == 11


def test_stream_detects_value_replacing_attacks_and_not_the_delay_attack():
    """Against the EMA reference: constant, random-value and invisible-noise submissions move every statistic far out
    of the fences; a delayed (stale but honest) signal of this slowly drifting stream is statistically a clean one."""
    st = _stream()
    _warm(st)
    t = WARM
    for w, kind in enumerate(("constant", "random", "invisible")):      # one worker each: a gross deviation bans at once
        st.begin_iteration(False)
        h = _signals("h", 0, t)
        if kind == "constant":
            h[w] = si.attack_constant(h[w], -1.0, "f32")
        elif kind == "random":
            h[w] = si.attack_random_value(h[w], t, "f32")
        else:
            h[w] = si.attack_invisible_noise(h[w], 0.99, t, "f32")
        here, _ = st.forward(0, h)
        assert here == [w], kind
        t += 1
    st.begin_iteration(False)
    h = _signals("h", 0, t)
    h[3] = si.stream_signal("h", 0, 3, t - 20, T, D, "f32")          # delay attack, k = 20
    here, _ = st.forward(0, h)
    assert here == []


# ------------------------------------------------------------------ identities the device loop's arrangement rests on
def test_ema_from_the_sum_and_projections_by_linearity():
    """Two rearrangements the library makes of Alg. momentum_verification's arithmetic, pinned on the oracle's own
    routines: (i) Eq. momentum_def from the SUM over the clean set equals the update from the clean set itself;
    (ii) the projections <u_l, m_t> of the updated EMA equal the same recurrence applied to the projections, so
    Omega_SW against the EMA can be formed from projections that were never recomputed from the EMA."""
    from oracle import stage_oracle as st
    rng = np.random.default_rng(11)
    T, D, L, n, beta = 40, 24, 8, 7, 0.9
    u = _dirs(L, D, 5)
    m = rng.standard_normal((T, D))
    pm = m @ u.T                                              # [T, L]
    for it in range(4):
        x = [m + 0.3 * rng.standard_normal((T, D)) for _ in range(n)]
        flags = [int(rng.random() < 0.3) for _ in range(n)]
        if it == 3:
            flags = [1] * n                                   # nobody clean: everything stays
        clean = [xi for xi, f in zip(x, flags) if not f]
        want = st.ema_update(m, x, flags, beta)
        if clean:
            total = np.sum(clean, axis=0)
            np.testing.assert_allclose(beta * m + (1 - beta) * total / len(clean), want, rtol=1e-13, atol=1e-13)
            pm = beta * pm + (1 - beta) * np.mean([xi @ u.T for xi in clean], axis=0)
        else:
            assert np.array_equal(want, m)
        m = want
        np.testing.assert_allclose(pm, m @ u.T, rtol=1e-12, atol=1e-12)
        # the statistic from the carried projections is the oracle's statistic against the EMA
        probe = m + 0.5 * rng.standard_normal((T, D))
        from_proj = float(np.mean(np.mean(np.abs(np.sort(probe @ u.T, axis=0) - np.sort(pm, axis=0)), axis=0)))
        assert from_proj == pytest.approx(so.sliced_wasserstein(probe, m, u), rel=1e-12)
