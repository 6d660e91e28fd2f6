"""Pins for the oracle's latency calibration (Sec. 5.2) and the cost curve handed to the controller (Eq. 6).

The static fit is checked against a planted line, numpy's polynomial fit, the zero gradient of the squared residual
and brute-force perturbations; the online update against the closed form of a geometric sequence; the cost curve
against values assembled by hand from the hand-summed configuration of App. E.
"""
import numpy as np
import pytest

from paper_2605_29727_amd import synth


def test_planted_line_is_recovered(oracle):
    pred = np.array([1.0, 3.0, 5.0, 7.0, 9.0])
    obs = 2.5 * pred + 0.75                      # small integers and binary fractions: every sum and mean is exact
    a, b = oracle.calib_fit(pred, obs)
    assert a == 2.5 and b == 0.75
    a, b = oracle.calib_fit(pred[:2], obs[:2])   # two points determine the line
    assert a == 2.5 and b == 0.75
    a, b = oracle.calib_fit(pred, np.full(5, 3.0))
    assert a == 0.0 and b == 3.0


@pytest.mark.parametrize("seed", range(4))
def test_equals_library_fit_and_is_not_transposed(oracle, seed):
    n = 40
    pred = 1e-3 * (1.0 + 10.0 * synth.uniform(seed, "calib_pred", (n,)))
    obs = 1.7 * pred + 4e-4 + 2e-4 * (synth.uniform(seed, "calib_noise", (n,)) - 0.5)
    a, b = oracle.calib_fit(pred, obs)
    pa, pb = np.polyfit(pred, obs, 1)
    assert a == pytest.approx(pa, rel=1e-9) and b == pytest.approx(pb, rel=1e-9)
    ta, _ = oracle.calib_fit(obs, pred)           # regressing the other way is a different line
    assert abs(ta - a) > 0.5
    # zero gradient of the squared residual: orthogonal to the regressor and to the constant
    r = obs - (a * pred + b)
    assert abs(r.sum()) < 1e-12 * np.abs(obs).sum() and abs((r * pred).sum()) < 1e-12 * np.abs(obs * pred).sum()


def test_fit_minimises_rmse_and_beats_the_raw_prediction(oracle):
    """Sec. 5.2: the calibrated curve lowers the RMSE of the bare roofline; here: no other line does better."""
    pred = np.linspace(0.02, 0.06, 25)
    obs = 1.3 * pred + 0.004 + 0.003 * np.sin(np.arange(25.0))      # a curve that no line fits exactly
    a, b = oracle.calib_fit(pred, obs)
    rmse = lambda s, o: float(np.sqrt(np.mean((obs - (s * pred + o)) ** 2)))
    best = rmse(a, b)
    assert best < rmse(1.0, 0.0)
    for da in (-0.05, 0.0, 0.05):
        for db in (-5e-4, 0.0, 5e-4):
            if da or db:
                assert rmse(a + da, b + db) > best


def test_undetermined_fits_are_refused(oracle):
    with pytest.raises(ValueError):
        oracle.calib_fit(np.array([1.0]), np.array([2.0]))
    with pytest.raises(ValueError):
        oracle.calib_fit(np.array([3.0, 3.0, 3.0]), np.array([1.0, 2.0, 3.0]))


def test_ema_closed_form(oracle):
    """A constant ratio r = obs/pred is approached geometrically: c_k = r + (c_0 - r)(1 - alpha)^k."""
    r, c0, alpha = 1.75, 1.0, 0.125
    c = c0
    for k in range(1, 40):
        c = oracle.calib_ema(c, alpha, 3.5, 2.0)
        assert c == pytest.approx(r + (c0 - r) * (1 - alpha) ** k, rel=1e-13)
    assert oracle.calib_ema(0.4, 1.0, 6.0, 4.0) == 1.5         # alpha = 1: the last ratio
    assert oracle.calib_ema(0.4, 0.0, 6.0, 4.0) == 0.4         # alpha = 0: never moves
    assert oracle.calib_ema(1.0, 0.5, 1.0, 4.0) == 0.625       # obs over pred, not pred over obs


def test_cost_curve_by_hand(oracle):
    """The hand-summed configuration of the cost-model pins (one layer, h=2, one 2-wide head, hffn=3, V=5, one byte
    per element, c=2) at s = 2 and 3 new tokens.  FLOPs(s) = s*(8+16+8+24+12+20) for the projections, FFN and LM
    head plus 2 * 4*s*(2+s) for scores and PV = 104 s + 8 s^2: s=2: 240, s=3: 384.  Elements(s) = 54 weights + 8 KV
    read + 4 s KV write + attention activations 4s + 8s + 4s + 2s(2+s) + FFN 16 s + LM head 7 s = 62 + 47 s + 2 s^2:
    s=2: 164, s=3: 221.  With peak 60 FLOP/s and 82 B/s: R(2) = max(4, 2) = 4, R(3) = max(6.4, 221/82) = 6.4."""
    cost = oracle.cost_curve(2, 2, 1, 2, 1, 1, 2, 3, 5, 1, 60.0, 82.0, calib_scale=2.0, calib_offset=0.5, c_ema=1.5,
                             t_other=10.0)
    assert cost[0] == pytest.approx(10.0 + 1.5 * (2.0 * 4.0 + 0.5))          # N = 1 draft node: root + 1 = 2 tokens
    assert cost[1] == pytest.approx(10.0 + 1.5 * (2.0 * 6.4 + 0.5))
    flat = oracle.cost_curve(5, 2, 1, 2, 1, 1, 2, 3, 5, 1, 60.0, 82.0, c_ema=0.0, t_other=3.0)
    assert flat.tolist() == [3.0] * 5


def test_cost_curve_grows_with_the_budget(oracle):
    c = oracle.cost_curve(256, 8192, 32, 4096, 32, 8, 128, 14336, 128256, 2, 2.5e15, 8e12, t_other=1e-4)
    assert np.all(np.diff(c) > 0)
    one = oracle.verify_cost(65, 8192, 32, 4096, 32, 8, 128, 14336, 128256, 2, 2.5e15, 8e12)
    assert c[63] == pytest.approx(1e-4 + one["latency_s"], rel=1e-14)
