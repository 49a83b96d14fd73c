"""Pins for the oracle's alternative signal smoothers (CPU only): sliding window, momentum
and paragraph mean of the paper's Appendix "Signal Smoothing" (N = 10), checked against
library routines (pandas rolling and grouped expanding means), closed forms
(step, constant and linear series) and hand-computed values; then the way accept_exit
drives them (cadence, paragraph ends, freezing, the gate)."""
import numpy as np
import pandas as pd
import pytest

from oracle import specexit_oracle as O

from test_oracle_accept_exit import fresh_state


def cfg(smoother, **kw):
    return O.ExitCfg(smoother=smoother, **kw)


def series_of(smoother, s, **kw):
    c = cfg(smoother, **kw)
    return np.array([O.smooth_series(s[:t + 1], c) for t in range(len(s))])


def noisy(n, seed):
    return np.random.default_rng(seed).random(n)


# ----------------------------------------------------------------------------- sliding window

def test_window_is_the_library_rolling_mean():
    s = noisy(57, 1)
    for N in (1, 2, 10, 16):
        ref = pd.Series(s).rolling(N, min_periods=1).mean().to_numpy()
        np.testing.assert_allclose(series_of(O.SMOOTH_WINDOW, s, window=N), ref, rtol=0, atol=1e-14)


def test_window_step_response_counts_exactly_ten_samples_including_the_latest():
    s = [0.0] * 12 + [1.0] * 12
    x = series_of(O.SMOOTH_WINDOW, s)
    # j + 1 ones are inside the window j rounds after the step: a window of 9 or 11, or one
    # that leaves the latest sample out, gives other fractions
    np.testing.assert_allclose(x[12:22], (np.arange(10) + 1) / 10.0, atol=1e-15)
    assert x[11] == 0.0 and x[22] == 1.0


def test_window_default_is_the_papers_n():
    assert O.ExitCfg().window == 10


def test_window_of_one_is_no_smoothing():
    s = noisy(20, 2)
    np.testing.assert_array_equal(series_of(O.SMOOTH_WINDOW, s, window=1), series_of(O.SMOOTH_NONE, s))


# ----------------------------------------------------------------------------- momentum

def test_momentum_forecasts_a_linear_series_exactly():
    # s_i = a + b i: every difference is b, so the forecast of the next value is s_t + b
    a, b = 0.25, 0.03125
    s = a + b * np.arange(30)
    x = series_of(O.SMOOTH_MOMENTUM, s)
    np.testing.assert_allclose(x[1:], s[1:] + b, atol=1e-14)
    assert x[0] == s[0]                                      # one observation: its own forecast


def test_momentum_is_the_secant_through_the_window_ends():
    # the differences telescope: mean difference = (s_t - s_{t-N+1}) / (N-1)
    s = noisy(64, 3)
    x = series_of(O.SMOOTH_MOMENTUM, s)
    for t in range(len(s)):
        n = min(10, t + 1)
        ref = s[t] if n == 1 else s[t] + (s[t] - s[t - n + 1]) / (n - 1)
        assert abs(x[t] - ref) < 1e-14


def test_momentum_hand_example():
    # N = 3 over (1, 4, 2, 8): last three are 4, 2, 8; differences -2, +6; mean 2; forecast 10
    assert O.smooth_series([1.0, 4.0, 2.0, 8.0], cfg(O.SMOOTH_MOMENTUM, window=3)) == 10.0
    # only two values so far: one difference
    assert O.smooth_series([1.0, 4.0], cfg(O.SMOOTH_MOMENTUM, window=3)) == 7.0
    # values older than the window do not matter
    assert O.smooth_series([99.0, 4.0, 2.0, 8.0], cfg(O.SMOOTH_MOMENTUM, window=3)) == 10.0
    # the oldest value of the window does
    assert O.smooth_series([1.0, 5.0, 2.0, 8.0], cfg(O.SMOOTH_MOMENTUM, window=3)) == 9.5


def test_momentum_ignores_interior_values():
    s = noisy(10, 4)
    s2 = s.copy()
    s2[1:9] = noisy(8, 5)
    c = cfg(O.SMOOTH_MOMENTUM)
    assert abs(O.smooth_series(s, c) - O.smooth_series(s2, c)) < 1e-14


# ----------------------------------------------------------------------------- paragraph mean

def test_paragraph_mean_is_the_library_expanding_mean_per_paragraph():
    s = noisy(40, 6)
    starts = [0, 7, 8, 21, 33]
    par = np.zeros(40, int)
    for p in starts[1:]:
        par[p:] += 1
    ref = pd.Series(s).groupby(par).expanding().mean().to_numpy()
    c = cfg(O.SMOOTH_PARAGRAPH)
    got = []
    for t in range(40):
        start = max(p for p in starts if p <= t)
        got.append(O.smooth_series(s[:t + 1], c, par_start=start))
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-14)


def test_paragraph_mean_hand_example():
    c = cfg(O.SMOOTH_PARAGRAPH)
    assert O.smooth_series([2.0, 4.0, 9.0], c) == 5.0
    assert O.smooth_series([2.0, 4.0, 9.0], c, par_start=1) == 6.5
    assert O.smooth_series([2.0, 4.0, 9.0], c, par_start=2) == 9.0


# ----------------------------------------------------------------------------- shared properties

@pytest.mark.parametrize("smoother", [O.SMOOTH_EWMA, O.SMOOTH_NONE, O.SMOOTH_WINDOW, O.SMOOTH_MOMENTUM, O.SMOOTH_PARAGRAPH])
def test_a_constant_signal_is_a_fixed_point(smoother):
    x = series_of(smoother, [0.625] * 25)
    np.testing.assert_allclose(x, 0.625, atol=1e-15)


@pytest.mark.parametrize("smoother", [O.SMOOTH_WINDOW, O.SMOOTH_PARAGRAPH, O.SMOOTH_EWMA])
def test_averaging_smoothers_stay_inside_the_range_seen(smoother):
    s = noisy(80, 7)
    x = series_of(smoother, s)
    for t in range(len(s)):
        assert s[:t + 1].min() - 1e-15 <= x[t] <= s[:t + 1].max() + 1e-15


def test_ewma_series_form_equals_the_recurrence_used_in_accept_exit():
    s = noisy(30, 8)
    x = series_of(O.SMOOTH_EWMA, s)
    # closed form of the recurrence seeded with the first observation
    a = 0.1
    for t in range(len(s)):
        ref = (1 - a) ** t * s[0] + sum(a * (1 - a) ** (t - i) * s[i] for i in range(1, t + 1))
        assert abs(x[t] - ref) < 1e-14


# ----------------------------------------------------------------------------- inside accept_exit

def drive(smoother, sigs, toks, split, window=10, thr=None):
    """One sequence, chain of one draft token that is always accepted; toks[t] is that token."""
    kw = dict(thr_conf=2.0) if thr is None else thr          # confidence can never pass: no exit
    c = O.ExitCfg(smoother=smoother, window=window, stop_think_token=999, **kw)
    state = fresh_state(1)
    hist = O.new_histories(1)
    xs, flags = [], []
    for s, tk in zip(sigs, toks):
        out = O.accept_exit(c, np.array([[5, tk]], np.int32), None, np.array([[tk, 6]], np.int32),
                            np.array([s], np.float64), np.array([100], np.int32),
                            np.array(sorted(split), np.int32), *state, hist=hist)
        assert out["accept_len"][0] == 1
        xs.append(state[0][0].copy())
        flags.append(int(out["exit_flag"][0]))
    return np.array(xs), flags, state, hist


def test_accept_exit_window_and_momentum_follow_the_series_functions():
    r = np.random.default_rng(9)
    sigs = np.stack([r.random(30), r.random(30), r.random(30) * 400], axis=1)
    for smoother in (O.SMOOTH_WINDOW, O.SMOOTH_MOMENTUM):
        xs, flags, state, _ = drive(smoother, sigs, [7] * 30, split=[3])
        for j in range(3):
            np.testing.assert_allclose(xs[:, j], series_of(smoother, sigs[:, j]), atol=1e-12)
        assert state[1][0] == 30 and not any(flags)


def test_accept_exit_paragraph_mean_restarts_after_a_round_that_accepts_a_split_token():
    sigs = np.array([[0.1, 0, 0], [0.3, 0, 0], [0.5, 0, 0], [0.9, 0, 0], [0.7, 0, 0], [0.2, 0, 0]])
    toks = [7, 7, 3, 7, 3, 7]                               # rounds 2 and 4 accept the split token 3
    xs, flags, _, hist = drive(O.SMOOTH_PARAGRAPH, sigs, toks, split=[3])
    # the closing round still belongs to its paragraph; the next round starts a new one
    np.testing.assert_allclose(xs[:, 0], [0.1, 0.2, 0.3, 0.9, 0.8, 0.2], atol=1e-15)
    assert hist[0].par_start == 5 and not any(flags)


def test_accept_exit_alternative_smoothers_gate_on_the_smoothed_value():
    # window of 4: the mean crosses 0.8 only when the fourth high value arrives
    sigs = [[0.0, 1, 0]] * 4 + [[1.0, 1, 0]] * 4
    thr = dict(thr_conf=0.8, thr_prog=0.3, thr_rem=200.0)
    xs, flags, state, _ = drive(O.SMOOTH_WINDOW, np.array(sigs), [3] * 8, split=[3], window=4, thr=thr)
    assert flags == [0, 0, 0, 0, 0, 0, 0, 1]
    assert state[2][0] == 0
    # momentum over the same series overshoots and fires at the first jump: 1 + (1 - 0) / 3 > 0.8
    xs, flags, state, _ = drive(O.SMOOTH_MOMENTUM, np.array(sigs), [3] * 5, split=[3], window=4, thr=thr)
    assert flags == [0, 0, 0, 0, 1]
    np.testing.assert_allclose(xs[4, 0], 1.0 + 1.0 / 3.0, atol=1e-15)


def test_accept_exit_history_is_frozen_after_the_exit():
    thr = dict(thr_conf=0.8, thr_prog=0.3, thr_rem=200.0)
    sigs = np.array([[0.9, 0.9, 10.0]] * 4)
    xs, flags, state, hist = drive(O.SMOOTH_WINDOW, sigs, [3] * 4, split=[3], thr=thr)
    assert flags == [1, 0, 0, 0]
    assert len(hist[0].values) == 1 and state[1][0] == 1
