"""Pins for the closed forms of Eq. (3)-(8)."""
import math
import os
import random

import pytest

from oracle import speedup_model as M

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_eq7_reproduces_the_printed_worked_example():
    for N, E, a, printed, measured in _rows("eq7_worked_example.txt"):
        rho = M.ppsd_gain(float(a), int(E), int(N))
        # the paper prints two decimals (1.31); the exact value is 1.3189...
        assert abs(rho - float(printed)) < 0.01
        assert abs(rho - 32 / (0.3226 * 8 + 0.6774 * 32)) < 1e-12


def test_eq7_limits():
    for N, E, a, gain in _rows("eq7_limits.txt"):
        assert M.ppsd_gain(float(a), int(E), int(N)) == pytest.approx(float(gain), abs=1e-12)
    # E not dividing N: ceil(N/E) stages, alpha = 0 falls slightly below 1
    assert M.ppsd_gain(0.0, 12, 32) == pytest.approx(32 / 36)


def test_eq4_closed_form_equals_its_sum():
    for a in (0.0, 0.1, 0.5, 0.8, 0.99):
        for g in (1, 2, 5, 10, 40):
            assert M.expected_accept_len(a, g) == pytest.approx(M.expected_accept_len_sum(a, g), abs=1e-12)
    assert M.expected_accept_len(1.0, 7) == 7 == pytest.approx(M.expected_accept_len_sum(1.0, 7))
    assert M.expected_accept_len(0.5, 1) == 0.5            # gamma = 1: accepted length = alpha


def test_eq4_is_the_mean_of_the_accept_process():
    rng = random.Random(1)
    a, g, n = 0.7, 5, 200000
    tot = 0
    for _ in range(n):
        k = 0
        while k < g and rng.random() < a:
            k += 1
        tot += k
    assert tot / n == pytest.approx(M.expected_accept_len(a, g), abs=0.02)


def test_eq5_follows_from_eq3_under_the_papers_assumptions():
    # T_T(gamma) = T_T(1) = N layer-times, T_D(1) = E layer-times (Sec. 3.1)
    for a in (0.3, 0.8):
        for g in (1, 5, 10):
            for E, N in ((8, 32), (10, 40)):
                assert M.sd_gain(N, E, N, a, g) == pytest.approx(M.eesd_gain(a, g, E, N), rel=1e-12)
    assert M.eesd_gain(1.0, 5, 8, 32) == pytest.approx(M.eesd_gain(1 - 1e-9, 5, 8, 32), rel=1e-6)


def test_eq6_and_eq8():
    assert M.overall_acceptance(0.8, 1) == pytest.approx(0.8)
    assert M.overall_acceptance(0.8, 10) < M.overall_acceptance(0.8, 5) < 0.8
    for a in (0.2, 0.6, 0.9):
        lam = M.ppsd_over_eesd(a, 5, 8, 32)
        assert lam > 1.0
        want = (1 - a) * (5 * 8 + 32) / ((a * 8 + (1 - a) * 4 * 8) * (1 - a ** 6))
        assert lam == pytest.approx(want, rel=1e-12)
    # alpha -> 1 limit of Eq. (8) is (gamma + N/E) / (gamma + 1)
    assert M.ppsd_over_eesd(1.0, 5, 8, 32) == pytest.approx((5 + 4) / 6)


def test_tick_model_has_eq7_as_its_expectation():
    rng = random.Random(2)
    for a, E, N in ((0.3226, 8, 32), (0.8, 8, 32), (0.7, 10, 40)):
        acc = [rng.random() < a for _ in range(200000)]
        gain = len(acc) * (N / E) / M.pipeline_ticks(acc, E, N)
        assert gain == pytest.approx(M.ppsd_gain(a, E, N), rel=0.01)
    assert M.pipeline_ticks([True] * 10, 8, 32) == 10
    assert M.pipeline_ticks([False] * 10, 8, 32) == 40
