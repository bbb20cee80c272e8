"""Pins for the penalty and utility functions (Sec. 3.1 eq. (2), Sec. 6.1)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import sneakpeek_oracle as orc

KINDS = [orc.PEN_STEP, orc.PEN_LINEAR, orc.PEN_SIGMOID]


@pytest.mark.parametrize("kind", KINDS)
def test_no_penalty_when_on_time_including_equality(kind):
    d = np.array([10.0, 10.0, 10.0, 250.0])
    e = np.array([0.0, 9.999, 10.0, 250.0])
    assert np.all(orc.penalty(kind, d, e) == 0.0)
    # eq. (2): all deadlines met -> utility is the accuracy itself
    assert np.all(orc.utility(0.83, kind, d, e) == 0.83)


def test_step_penalty_is_an_indicator_and_late_utility_is_zero():
    d = np.array([10.0, 10.0])
    e = np.array([10.0000001, 1e6])
    assert np.all(orc.penalty(orc.PEN_STEP, d, e) == 1.0)
    assert np.all(orc.utility(0.9, orc.PEN_STEP, d, e) == 0.0)


def test_linear_penalty_closed_form():
    d = 40.0
    assert orc.penalty(orc.PEN_LINEAR, d, 50.0) == pytest.approx(0.25, rel=1e-15)
    assert orc.penalty(orc.PEN_LINEAR, d, 60.0) == pytest.approx(0.5, rel=1e-15)
    assert orc.penalty(orc.PEN_LINEAR, d, 80.0) == 1.0
    assert orc.penalty(orc.PEN_LINEAR, d, 500.0) == 1.0


def test_sigmoid_penalty_closed_form_points():
    d = 40.0
    assert orc.penalty(orc.PEN_SIGMOID, d, 60.0) == pytest.approx(0.5, rel=1e-15)      # x = 1/2
    assert orc.penalty(orc.PEN_SIGMOID, d, 80.0) == 1.0                                 # x = 1
    assert orc.penalty(orc.PEN_SIGMOID, d, 123.0) == 1.0                                # x > 1
    assert orc.penalty(orc.PEN_SIGMOID, d, 40.0 + 1e-9) < 1e-30                         # x -> 0+
    # x = 1/4: x^3 / (x^3 + (1-x)^3) = 1 / 28
    assert orc.penalty(orc.PEN_SIGMOID, d, 50.0) == pytest.approx(1.0 / 28.0, rel=1e-14)


def test_sigmoid_equals_rational_form_and_is_symmetric():
    d = Fraction(64)
    for num in range(1, 64):
        x = Fraction(num, 64)
        e = d + x * d
        want = x ** 3 / (x ** 3 + (1 - x) ** 3)
        got = float(orc.penalty(orc.PEN_SIGMOID, float(d), float(e)))
        assert got == pytest.approx(float(want), rel=1e-13)
        mirror = float(orc.penalty(orc.PEN_SIGMOID, float(d), float(d + (1 - x) * d)))
        assert got + mirror == pytest.approx(1.0, rel=1e-13)


@pytest.mark.parametrize("kind", KINDS)
def test_penalty_is_monotone_and_bounded(kind):
    d = 25.0
    e = np.linspace(0.0, 80.0, 4001)
    g = orc.penalty(kind, d, e)
    assert np.all(np.diff(g) >= 0)
    assert g.min() == 0.0 and g.max() == 1.0
    u = orc.utility(0.7, kind, d, e)
    assert np.all(u >= 0) and np.all(u <= 0.7)


@pytest.mark.parametrize("kind", KINDS)
def test_dead_exactly_when_penalty_is_one_away_from_rounding(kind):
    d = np.array([10.0, 10.0, 10.0, 10.0, 10.0])
    e = np.array([5.0, 10.0, 15.0, 20.0, 30.0])
    dead = orc.is_dead(kind, d, e)
    assert np.array_equal(dead, orc.penalty(kind, d, e) >= 1.0)
    want = [False, False, True, True, True] if kind == orc.PEN_STEP else [False, False, False, True, True]
    assert dead.tolist() == want


def test_broadcasting_deadline_rows_against_completion_columns():
    d = np.array([10.0, 20.0, 40.0])[None, :]
    e = np.array([15.0, 30.0])[:, None]
    g = orc.penalty(orc.PEN_LINEAR, d, e)
    assert g.shape == (2, 3)
    assert g.tolist() == [[0.5, 0.0, 0.0], [1.0, 0.5, 0.0]]
