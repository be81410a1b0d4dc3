"""Host-side runtime model of Sec. 3.3 (paper_2310_18813_amd/model_fit.py) against the oracle's plain
definitions, closed forms and brute force.  No GPU."""
import math

import numpy as np
import pytest

from paper_2310_18813_amd import model_fit as mf


@pytest.fixture(scope="module")
def orc():
    from oracle import oracle as om
    return om.Oracle("f64")


def test_root_of_eq11_is_the_argmin_of_eq7(orc):
    """Eq. 11 is dt/ds = 0 for t of Eq. 7: its root must be where a dense scan of Eq. 7, evaluated through the
    oracle's Eq. 1-3 with t_L = alpha s + beta and l = c s^gamma, is smallest."""
    c, gamma = 0.9, 0.548                      # the curve the paper fits in Fig. 2 / Eq. 5
    for alpha_b, beta in [(0.02, 1.0), (0.1, 1.0), (0.5, 1.0), (0.03, 3.3), (2.0, 5.0)]:
        root = mf.s_opt_continuous(alpha_b, beta, c, gamma)
        grid = np.linspace(0.01, 200.0, 200000)
        t = [orc.time_model(128.0, alpha_b * s + beta, 0.0, s, c * s ** gamma) for s in grid[::50]]
        s_scan = grid[::50][int(np.argmin(t))]
        assert abs(root - s_scan) <= 0.03 * max(1.0, s_scan), (alpha_b, beta, root, s_scan)
        # and the library's own Eq. 7 agrees with the oracle's Eq. 1-3
        for s in (0.5, 1.0, 3.0, 8.0):
            assert mf.model_time(s, alpha_b, beta, c, gamma, 128.0) == pytest.approx(
                orc.time_model(128.0, alpha_b * s + beta, 0.0, s, c * s ** gamma), rel=1e-12)


def test_delta_is_the_numerator_of_the_derivative():
    c, gamma, alpha_b, beta = 0.8, 0.6, 0.07, 2.0
    for s in (0.3, 1.0, 2.5, 7.0, 20.0):
        h = 1e-6 * s
        dt = (mf.model_time(s + h, alpha_b, beta, c, gamma) - mf.model_time(s - h, alpha_b, beta, c, gamma)) / (2 * h)
        assert dt * (c * s ** gamma + 1.0) ** 2 == pytest.approx(mf.delta(s, alpha_b, beta, c, gamma), rel=1e-5, abs=1e-9)


def test_s_opt_falls_as_the_slope_grows():
    """The monotonicity argument that closes Sec. 3.3: larger alpha_b (larger batch) -> smaller s_opt."""
    prev = float("inf")
    for alpha_b in (0.005, 0.01, 0.05, 0.1, 0.5, 1.0, 5.0):
        s = mf.s_opt_continuous(alpha_b, 1.0, 0.9, 0.548)
        assert s <= prev + 1e-9
        prev = s
    assert mf.s_opt_continuous(0.0, 1.0, 0.9, 0.548) == 1.0e4   # free proposals: no finite optimum


def test_fits_recover_exact_inputs():
    a, b = mf.fit_line([0, 1, 2, 4, 8], [3.0 + 0.25 * s for s in [0, 1, 2, 4, 8]])
    assert a == pytest.approx(0.25) and b == pytest.approx(3.0)
    ss = list(range(1, 9))
    c, g = mf.fit_power(ss, [0.9 * s ** 0.548 for s in ss])
    assert c == pytest.approx(0.9) and g == pytest.approx(0.548)
    with pytest.raises(ValueError):
        mf.fit_line([1, 1], [2, 3])


def test_expected_length_estimators(orc):
    rng = np.random.default_rng(5)
    l_i = rng.geometric(0.3, size=500) - 1            # accepted-prefix lengths with per-token success 0.7
    for s in (0, 1, 2, 4, 8, 80):
        assert mf.l_from_samples(list(l_i), s) == pytest.approx(orc.l_estimate(l_i, s), rel=1e-12)
    # histogram form: rounds run with 8 proposals, lengths clipped at 8
    hist = [int((np.minimum(l_i, 8) == k).sum()) for k in range(9)]
    for s in (0, 1, 3, 8):
        assert mf.l_from_histogram(hist, s) == pytest.approx(orc.l_estimate(l_i, s), rel=1e-12)
    with pytest.raises(ValueError):
        mf.l_from_histogram(hist, 9)
    # closed form of Eq. 6 under independence: alpha = 0.7, s = 4 -> 1.7731; s = 0 -> 0
    assert mf.l_iid(0.7, 4) == pytest.approx(0.7 + 0.49 + 0.343 + 0.2401)
    assert mf.l_iid(0.7, 0) == 0.0 and mf.l_iid(1.0, 5) == 5.0
    # and the estimator converges to it
    big = rng.geometric(0.3, size=200000) - 1
    assert mf.l_from_samples(list(big), 4) == pytest.approx(mf.l_iid(0.7, 4), rel=1e-2)


def test_grid_argmin_matches_the_oracle_lut(orc):
    """s_opt_grid is the profiling stage's arg-min on Eq. 1-3: same choice as the oracle's LUT builder on the
    per-token latencies the model implies (ties: smaller s)."""
    rng = np.random.default_rng(11)
    for _ in range(20):
        S = 8
        l = [mf.l_iid(float(rng.uniform(0.2, 0.95)), s) for s in range(S + 1)]
        tL = np.cumsum(rng.uniform(0.0, 0.5, size=S + 1)) + 2.0
        tS = float(rng.uniform(0.0, 0.3))
        lat = np.array([[mf.total_time(1.0, tL[s], tS, s, l[s]) for s in range(S + 1)]])
        assert mf.s_opt_grid(list(range(S + 1)), list(tL), tS, l) == int(orc.lut_build(lat, rel_eps=0.0)[0])


def test_explain_puts_model_and_grid_side_by_side():
    l = [mf.l_iid(0.7, s) for s in range(9)]
    Bs = [1, 8, 64]
    s_list = [0, 1, 2, 4, 8]
    grid = [[3.0 + a * s for s in s_list] for a in (0.01, 0.1, 0.8)]
    res = mf.explain(Bs, s_list, grid, [0.1, 0.12, 0.2], l)
    assert 0.0 < res["gamma"] < 1.0
    roots = [r["s_opt_model"] for r in res["rows"]]
    picks = [r["s_opt_grid"] for r in res["rows"]]
    assert roots[0] >= roots[1] >= roots[2] and picks[0] >= picks[1] >= picks[2]
    for r, a in zip(res["rows"], (0.01, 0.1, 0.8)):
        assert r["alpha_b"] == pytest.approx(a) and r["beta"] == pytest.approx(3.0)
