"""Pins for the oracle's check statistics, flag rule and EMA update (CPU only).

Closed forms of the paper's attack variants (Problem Statement, "Attack Variants"),
the [0,1] bound of the sign flip ratio, the strict '>' of Eq. test_statistic, the EMA
recurrence solution used in the proof of Lemma momentum_dev and the lemma's bound.
"""
import math

import numpy as np
import pytest

from oracle import stage_oracle as so
import stage_inputs as si


def ref_signal(T=96, D=64, seed=0):
    return np.random.default_rng(seed).standard_normal((T, D)) * 1.7 + 0.05


def test_identical_submission_scores_zero():
    r = ref_signal()
    for red in ("max_token", "global"):
        s = so.scores(r, r, red)
        assert s == {"rel_l2": 0.0, "l1": 0.0, "zl2": 0.0, "sfr": 0.0}


@pytest.mark.parametrize("alpha", [1.5, 0.25, -1.0, -0.5])
def test_scaling_attack_closed_forms(alpha):
    r = ref_signal()
    c = alpha * r
    for red in ("max_token", "global"):
        s = so.scores(c, r, red)
        assert s["rel_l2"] == pytest.approx(abs(alpha - 1.0), rel=1e-12)
    np.testing.assert_allclose(so.token_rel_l2(c, r), abs(alpha - 1.0), rtol=1e-12)
    assert s["l1"] == pytest.approx(abs(alpha - 1.0) * np.mean(np.abs(r)), rel=1e-12)
    assert s["sfr"] == (0.0 if alpha > 0 else 1.0)
    assert s["zl2"] == pytest.approx(0.0 if alpha > 0 else 4.0, abs=1e-12)


def test_zero_attack_closed_forms():
    r = ref_signal()
    s = so.scores(np.zeros_like(r), r)
    assert s["rel_l2"] == pytest.approx(1.0, rel=1e-14)
    assert s["sfr"] == 1.0                       # sign(0) = 0 differs from every non-zero sign
    assert s["l1"] == pytest.approx(np.mean(np.abs(r)), rel=1e-13)
    assert s["zl2"] == 2.0                       # a constant signal has no z-score
    assert so.scores(np.zeros_like(r), np.zeros_like(r))["zl2"] == 0.0


def test_sign_flip_on_channel_set_closed_forms():
    r = ref_signal(T=50, D=40)
    c, ch = si.attack_sign_channels(r, 0.05, seed=3, dtype="f32")
    r = r.astype(np.float32)                      # the attack helper works in fp32
    assert len(ch) == 2
    s = so.scores(c, r)
    want_tok = 2.0 * np.sqrt(np.sum(r[:, ch].astype(np.float64) ** 2, axis=1) / np.sum(r.astype(np.float64) ** 2, axis=1))
    np.testing.assert_allclose(so.token_rel_l2(c, r), want_tok, rtol=1e-12)
    assert s["rel_l2"] == pytest.approx(want_tok.max(), rel=1e-12)
    assert s["sfr"] == pytest.approx(len(ch) / 40.0, rel=1e-14)


def test_additive_noise_concentrates_at_relative_std():
    r = ref_signal(T=512, D=256)
    c = si.attack_noise(r, 0.1, seed=1, dtype="f32")
    n = r.size
    s = so.scores(c, r.astype(np.float32), "global")
    # ||eps||^2 / n ~ chi2_n / n: relative std sqrt(2/n); the mean offset of r (0.05) is inside RMS
    assert s["rel_l2"] == pytest.approx(0.1, rel=4.0 / math.sqrt(2 * n) + 1e-3)


def test_zl2_equals_two_minus_two_rho_and_sfr_in_unit_interval():
    g = np.random.default_rng(5)
    r = g.standard_normal((30, 20))
    c = 0.6 * r + 0.8 * g.standard_normal((30, 20)) + 3.0
    s = so.scores(c, r)
    rho = np.corrcoef(c.ravel(), r.ravel())[0, 1]
    assert s["zl2"] == pytest.approx(2.0 * (1.0 - rho), rel=1e-12)
    assert 0.0 <= s["sfr"] <= 1.0
    sign = lambda a: 1 if a > 0 else (-1 if a < 0 else 0)
    want = sum(1 for a, b in zip(c.ravel().tolist(), r.ravel().tolist()) if sign(a) != sign(b)) / c.size
    assert s["sfr"] == want
    assert s["l1"] == pytest.approx(sum(abs(a - b) for a, b in zip(c.ravel().tolist(), r.ravel().tolist())) / c.size, rel=1e-13)


def test_token_rel_l2_bruteforce_and_max_reduce():
    g = np.random.default_rng(6)
    r, c = g.standard_normal((2, 5, 8)), g.standard_normal((2, 5, 8))
    want = []
    for b in range(2):
        for t in range(5):
            num = math.sqrt(sum((c[b, t, d] - r[b, t, d]) ** 2 for d in range(8)))
            den = math.sqrt(sum(r[b, t, d] ** 2 for d in range(8)))
            want.append(num / den)
    np.testing.assert_allclose(so.token_rel_l2(c, r), want, rtol=1e-13)
    assert so.scores(c, r, "max_token")["rel_l2"] == pytest.approx(max(want), rel=1e-13)
    glob = math.sqrt(np.sum((c - r) ** 2)) / math.sqrt(np.sum(r ** 2))
    assert so.scores(c, r, "global")["rel_l2"] == pytest.approx(glob, rel=1e-13)


def test_flag_is_strict_and_any_metric():
    assert not so.flag({"rel_l2": 0.02}, {"rel_l2": 0.02})          # Gamma == tau is not flagged
    assert so.flag({"rel_l2": np.nextafter(0.02, 1.0)}, {"rel_l2": 0.02})
    sc = {"rel_l2": 0.0, "l1": 0.0, "zl2": 0.0, "sfr": 0.3}
    assert so.flag(sc, {"rel_l2": 1.0, "sfr": 0.25})                # one metric over is enough
    assert not so.flag(sc, {"rel_l2": 1.0, "l1": 1.0})              # disabled metrics are ignored


def test_one_percent_token_corruption_needs_the_per_token_reduce():
    r = ref_signal(T=400, D=64)
    c, tok = si.attack_tokens(r, 0.01, "scale", seed=2, dtype="f32")
    r32 = r.astype(np.float32)
    assert so.scores(c, r32, "max_token")["rel_l2"] == pytest.approx(0.5, rel=1e-6)
    assert so.scores(c, r32, "global")["rel_l2"] < 0.08             # diluted by ~ sqrt(0.01)
    t = so.token_rel_l2(c, r32)
    assert set(np.nonzero(t > 0.1)[0]) == set(tok)


# ------------------------------------------------------------------ EMA
def test_ema_constant_input_closed_form():
    c = np.random.default_rng(7).standard_normal((4, 6))
    m, beta = np.zeros_like(c), 0.9
    for t in range(1, 25):
        m = so.ema_update(m, [c, c, c], [0, 0, 0], beta)
        np.testing.assert_allclose(m, (1.0 - beta ** t) * c, rtol=1e-12)


def test_ema_mean_is_over_the_clean_set_only():
    g = np.random.default_rng(8)
    xs = [g.standard_normal((3, 5)) for _ in range(4)]
    m0 = g.standard_normal((3, 5))
    got = so.ema_update(m0, xs, [0, 1, 0, 1], 0.8)
    np.testing.assert_allclose(got, 0.8 * m0 + 0.2 * (xs[0] + xs[2]) / 2.0, rtol=1e-14)
    np.testing.assert_array_equal(so.ema_update(m0, xs, [1, 1, 1, 1], 0.8), m0)   # nothing clean: unchanged


def test_momentum_deviation_lemma_bound():
    """Lemma momentum_dev: a fraction gamma of workers perturbing by at most eps moves the EMA
    by at most gamma*eps overall and by (1-beta)*gamma*eps in one step."""
    g = np.random.default_rng(9)
    d, n_bad, eps, beta = 8, 3, 0.7, 0.9
    m_nom = m_obs = np.zeros(50)
    for t in range(40):
        honest = [g.standard_normal(50) for _ in range(d)]
        pert = []
        for r in range(d):
            if r < n_bad:
                delta = g.standard_normal(50)
                delta *= eps / np.linalg.norm(delta)
                pert.append(honest[r] + delta)
            else:
                pert.append(honest[r])
        prev_gap = np.linalg.norm(m_obs - m_nom)
        m_nom_next = so.ema_update(m_nom, honest, [0] * d, beta)
        one_step = so.ema_update(m_nom, pert, [0] * d, beta)
        assert np.linalg.norm(one_step - m_nom_next) <= (1 - beta) * n_bad / d * eps * (1 + 1e-12)
        m_obs = so.ema_update(m_obs, pert, [0] * d, beta)
        m_nom = m_nom_next
        assert np.linalg.norm(m_obs - m_nom) <= n_bad / d * eps * (1 + 1e-12)
    assert np.linalg.norm(m_obs - m_nom) > 0


def test_non_finite_submission_is_flagged_and_constant_signals_have_no_zscore():
    r = ref_signal(T=8, D=8)
    c = r.copy()
    c[2, 3] = np.nan
    assert so.flag(so.scores(c, r), {"rel_l2": 1e9})
    assert so.flag(so.scores(c, r, "global"), {"l1": 1e9})
    ones = -np.ones_like(r) * 0.1                      # the constant attack with a value that does not sum exactly
    assert so.scores(ones, r)["zl2"] == 2.0
    assert so.scores(ones, ones * 3)["zl2"] == 0.0
