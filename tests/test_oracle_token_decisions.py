"""Pins of the oracle's token-level decisions on a logits row (CPU only): the top-1 softmax probability that the
draft stop rule compares with its threshold, and the top-1 / top-2 gap the parity tests use to recognise a near-tie.
Each is checked against a library routine it must reduce to, closed forms, and planted rows; the same pins must
fail on copies of the two functions with one plausible slip planted in their source."""
import inspect

import numpy as np
import pytest
import torch

from oracle import knnssd_oracle as O


def _pin_top1_prob(f):
    rng = np.random.default_rng(11)
    # (i) the library's softmax at temperature 1, probability of the arg-max token, on rows whose arg-max sits at the
    # front, in the middle and at the end, with large offsets (the subtraction of the maximum must not change it)
    for v, where, shift in ((50, 0, 0.0), (1000, 437, 80.0), (32000, 31999, -300.0)):
        row = rng.standard_normal(v).astype(np.float32) * 3.0
        row[where] = row.max() + 1.5
        row = (row + np.float32(shift)).astype(np.float32)
        want = torch.softmax(torch.from_numpy(row).double(), -1)
        assert int(want.argmax()) == where
        assert abs(f(row) - float(want[where])) <= 1e-12 * float(want[where]) + 1e-15
        assert abs(f(row) - float(want.max())) <= 1e-12
    # (ii) closed forms: V equal logits -> 1/V; one logit a above V-1 equal ones -> 1 / (1 + (V-1) e^-a)
    assert abs(f(np.full(64, 3.25, np.float32)) - 1.0 / 64) <= 1e-15
    for a in (0.5, 2.0, 7.0):
        row = np.zeros(1000, np.float32)
        row[123] = a
        assert abs(f(row) - 1.0 / (1.0 + 999.0 * np.exp(-np.float64(np.float32(a))))) <= 1e-13
    # (iii) temperature is 1: doubling the logits must give the closed form for 2a, not the one for a
    row = np.zeros(10, np.float32)
    row[4] = 1.0
    assert abs(f(2.0 * row) - 1.0 / (1.0 + 9.0 * np.exp(-2.0))) <= 1e-13
    # (iv) two-token row: the logistic function of the gap
    assert abs(f(np.array([0.3, 1.7], np.float32)) - 1.0 / (1.0 + np.exp(-(np.float64(np.float32(1.7)) - np.float64(np.float32(0.3)))))) <= 1e-13
    # (v) a probability: in (0, 1], 1 for a single token, and no overflow on huge logits
    assert f(np.array([5.0], np.float32)) == 1.0
    assert 0.0 < f(np.array([3e4, -3e4, 0.0], np.float32)) <= 1.0


def _pin_top2_margin(f):
    rng = np.random.default_rng(12)
    for v in (2, 7, 1000):
        row = rng.standard_normal(v).astype(np.float32)
        s = np.sort(row.astype(np.float64))            # the definition written out: full sort, last two
        assert f(row) == s[-1] - s[-2]
        assert f(row + np.float32(100.0)) == np.sort((row + np.float32(100.0)).astype(np.float64))[-1] - \
            np.sort((row + np.float32(100.0)).astype(np.float64))[-2]
    # a tie for the maximum is a margin of zero; planted gap at arbitrary places
    assert f(np.array([1.0, 4.0, 4.0, -2.0], np.float32)) == 0.0
    row = np.full(500, -1.0, np.float32)
    row[17] = 2.0
    row[400] = 1.25
    assert f(row) == 0.75
    assert f(row[::-1].copy()) == 0.75
    # never negative, and it is the gap to the runner-up, not to the minimum or the mean
    assert f(np.array([-5.0, 3.0, 2.5, -100.0], np.float32)) == 0.5


def test_top1_prob_pins():
    _pin_top1_prob(O.top1_prob)


def test_top2_margin_pins():
    _pin_top2_margin(O.top2_margin)


def _mutant(func, old, new):
    src = inspect.getsource(func)
    assert src.count(old) == 1, "mutation anchor not found exactly once"
    ns = dict(vars(O))
    exec(src.replace(old, new), ns)
    return ns[func.__name__]


TOP1_MUTATIONS = {
    "temperature_two": ("np.exp(l - l.max())", "np.exp((l - l.max()) / 2.0)"),
    "first_token_instead_of_argmax": ("float(1.0 / np.exp(l - l.max()).sum())", "float(np.exp(l[0] - l.max()) / np.exp(l - l.max()).sum())"),
    "no_max_subtraction_in_fp32": ("l = logits_row.astype(np.float64)", "l = logits_row.astype(np.float32)"),
    "sum_without_the_top_token": ("np.exp(l - l.max()).sum()", "(np.exp(l - l.max()).sum() - 1.0 + 1e-300)"),
}
TOP2_MUTATIONS = {
    "gap_to_third": ("part[-1] - part[-2]", "part[-1] - part[-3 if len(part) > 2 else -2]"),
    "row_not_ordered": ("np.partition(logits_row.astype(np.float64), -2)", "logits_row.astype(np.float64)"),
    "sign": ("float(part[-1] - part[-2])", "float(part[-2] - part[-1])"),
}


@pytest.mark.parametrize("name", sorted(TOP1_MUTATIONS))
def test_top1_prob_pins_catch_planted_mistake(name):
    bad = _mutant(O.top1_prob, *TOP1_MUTATIONS[name])
    with pytest.raises((AssertionError, FloatingPointError, ZeroDivisionError)):
        with np.errstate(over="raise", invalid="raise", divide="raise"):
            _pin_top1_prob(bad)


@pytest.mark.parametrize("name", sorted(TOP2_MUTATIONS))
def test_top2_margin_pins_catch_planted_mistake(name):
    bad = _mutant(O.top2_margin, *TOP2_MUTATIONS[name])
    with pytest.raises(AssertionError):
        _pin_top2_margin(bad)
