"""Host-side analysis and calibration utilities against library routines and closed forms (no GPU)."""
import numpy as np
import pytest
from sklearn.metrics import average_precision_score, precision_recall_curve as sk_pr

import oracle
from paper_2604_16883_amd import analysis, calibrate, synth


def test_average_precision_matches_library():
    rng = np.random.default_rng(0)
    for n, p in ((50, 0.3), (400, 0.6), (1000, 0.05)):
        y = rng.random(n) < p
        s = rng.normal(size=n) + 1.5 * y
        s = np.round(s, 1)                       # many ties
        assert analysis.average_precision(s, y) == pytest.approx(average_precision_score(y, s), abs=1e-12)
        pr, rc, th = analysis.precision_recall_curve(s, y)
        sp, sr, st = sk_pr(y, s)
        # the library lists thresholds ascending and appends the (1, 0) end point
        np.testing.assert_allclose(pr[::-1], sp[:-1][-pr.size:], atol=1e-12)
        np.testing.assert_allclose(rc[::-1], sr[:-1][-rc.size:], atol=1e-12)
    # perfect and useless scores
    y = np.array([1, 1, 0, 0], bool)
    assert analysis.average_precision([4, 3, 2, 1], y) == 1.0
    assert analysis.average_precision([1, 2, 3, 4], y) == pytest.approx((1 / 3 + 2 / 4) / 2)


def test_threshold_sweep_is_strict_and_monotone():
    s = np.array([0.1, 0.5, 0.5, 0.9])
    y = np.array([0, 1, 0, 1], bool)
    sw = analysis.threshold_sweep(s, y, [0.0, 0.5, 0.9])
    assert sw["skip_ratio"].tolist() == [1.0, 0.25, 0.0]      # 0.5 is not > 0.5
    assert sw["precision"].tolist() == [0.5, 1.0, 1.0]
    assert sw["recall"].tolist() == [1.0, 0.5, 0.0]
    taus = np.linspace(-1, 1, 41)
    rng = np.random.default_rng(1)
    sw = analysis.threshold_sweep(rng.uniform(-1, 1, 300), rng.random(300) < 0.5, taus)
    assert np.all(np.diff(sw["skip_ratio"]) <= 0) and np.all(np.diff(sw["recall"]) <= 0)


def test_proxy_reliability_on_synthetic_cache_with_oracle():
    """The planted structure makes the proxy informative: groups whose heads are mostly sink-dominated
    have alpha_0 near 1 and score high.  Uses the oracle for both the scores and alpha_0."""
    scores, a0g = [], []
    for seed in range(6):
        w = synth.WORKLOADS["c1"].scaled(512)
        sb = synth.generate(w, seed=100 + seed)
        r = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True)
        scores.append(r.group_score.ravel())
        a0g.append(analysis.group_alpha0(r.alpha0, w.group_size).ravel())
        st = analysis.skipped_vs_active_alpha0(r.alpha0, r.mask, w.group_size)
        assert st["skipped_mean"] > st["active_mean"]
    scores, a0g = np.concatenate(scores), np.concatenate(a0g)
    labels = analysis.sink_labels(a0g)
    assert 0.2 < labels.mean() < 0.9
    ap = analysis.average_precision(scores, labels)
    assert ap > 0.95 and ap == pytest.approx(average_precision_score(labels, scores), abs=1e-12)


def test_threshold_for_skip_ratio_hits_the_quantised_target():
    rng = np.random.default_rng(2)
    for n in (8, 32, 80, 1000):
        s = rng.uniform(-0.2, 1.0, n)
        for target in (0.0, 0.25, 0.6, 1.0):
            tau = calibrate.threshold_for_skip_ratio(s, target)
            assert calibrate.skip_ratio(s, tau) == pytest.approx(round(target * n) / n, abs=1e-12)
    # ties cannot be split by a strict comparison: the closer side is taken
    s = np.array([0.9, 0.5, 0.5, 0.5, 0.1])
    assert calibrate.skip_ratio(s, calibrate.threshold_for_skip_ratio(s, 0.4)) in (0.2, 0.8)
    # monotone: a larger target never raises the threshold
    s = rng.normal(size=200)
    taus = [calibrate.threshold_for_skip_ratio(s, t) for t in np.linspace(0, 1, 21)]
    assert np.all(np.diff(taus) <= 0)


def test_cubic_fit_recovers_a_cubic_and_degrades_gracefully():
    coef = (0.8, -1.5, 0.7, 0.45)
    L = np.array([8192, 16384, 65536, 131072, 262144, 524288], float)
    t = [calibrate.tau_of(coef, x, 524288.0) for x in L]
    got, ln = calibrate.fit_tau_cubic(L, t)
    assert ln == 524288.0
    np.testing.assert_allclose(got, coef, rtol=1e-8, atol=1e-10)
    got, ln = calibrate.fit_tau_cubic([1000, 3000], [0.5, 0.6], len_norm=4000)      # two points: a line
    assert got[0] == 0 and got[1] == 0
    assert calibrate.tau_of(got, 1000, ln) == pytest.approx(0.5) and calibrate.tau_of(got, 3000, ln) == pytest.approx(0.6)
    got, ln = calibrate.fit_tau_cubic([4096], [0.55])                                  # one point: a constant
    assert got == (0.0, 0.0, 0.0, 0.55)


def test_calibrate_end_to_end_with_oracle_scores():
    by_len = {}
    for L in (256, 512, 1024, 2048):
        s = []
        for seed in range(4):
            sb = synth.generate(synth.WORKLOADS["c1"].scaled(L), seed=500 + seed)
            s.append(oracle.route(sb.q, sb.k, sb.seq_lens).group_score.ravel())
        by_len[L] = np.concatenate(s)
    cal = calibrate.calibrate(by_len, target=0.6)
    assert cal["len_norm"] == 2048
    for L, r in cal["realised_skip_ratio"].items():
        assert abs(r - 0.6) <= 0.05, (L, r)          # four exact points through a cubic: only quantisation is left
    # the fitted rule, fed to the oracle, realises the ratio on the calibration inputs
    sb = synth.generate(synth.WORKLOADS["c1"].scaled(1024), seed=500)
    r = oracle.route(sb.q, sb.k, sb.seq_lens, tau_coef=cal["tau_coef"], len_norm=cal["len_norm"])
    assert r.tau[0] == pytest.approx(cal["per_length_tau"][2], abs=1e-9)


def test_concentration_table_bins_and_ratio():
    a0 = np.array([0.41, 0.39, 0.62, 0.8, 0.83, 0.2, np.nan])
    mx = np.array([0.02, 0.04, 0.031, 0.01, 0.03, 0.5, 0.1])
    mn = np.array([1e-4, 3e-4, 2e-4, 1e-5, 3e-5, 1e-3, 1e-3])
    t = analysis.concentration_table(a0, mx, mn)
    assert [t[k]["heads"] for k in (0.4, 0.6, 0.8)] == [2, 1, 2]
    assert t[0.4]["bos"] == pytest.approx(0.40) and t[0.4]["max"] == pytest.approx(0.03)
    assert t[0.4]["mean"] == pytest.approx(2e-4) and t[0.4]["ratio"] == pytest.approx(0.40 / 0.03)
    assert t[0.6]["ratio"] == pytest.approx(0.62 / 0.031)
    assert t[0.8]["ratio"] == pytest.approx(0.815 / 0.02)
    empty = analysis.concentration_table(a0, mx, mn, regimes=(0.95,), half_width=0.01)
    assert empty[0.95]["heads"] == 0 and np.isnan(empty[0.95]["ratio"])


def test_concentration_table_on_oracle_statistics_orders_the_regimes():
    """Graded pull toward token 0 fills the regimes of Table 1 (Section 3); the ratio of the token-0
    weight to the strongest other weight grows with the regime, the table's qualitative content."""
    import dataclasses
    cols = []
    for i, gain in enumerate((9.0, 12.0, 15.0)):
        w = dataclasses.replace(synth.WORKLOADS["c0"].scaled(600), sink_gain=gain, sink_frac=1.0, planted_per_head=0)
        sb = synth.generate(w, seed=70 + i)
        a0, mx, mean, _ = oracle.concentration(sb.q, sb.k, sb.v, sb.seq_lens)
        np.testing.assert_allclose(a0 + mean * (600 - 1), 1.0, rtol=1e-12)
        cols.append((a0.ravel(), mx.ravel(), mean.ravel()))
    cat = [np.concatenate([c[j] for c in cols]) for j in range(3)]
    t = analysis.concentration_table(*cat, half_width=0.1)
    filled = [k for k in sorted(t) if t[k]["heads"] > 0]
    assert len(filled) >= 2
    ratios = [t[k]["ratio"] for k in filled]
    assert all(a < b for a, b in zip(ratios, ratios[1:]))
