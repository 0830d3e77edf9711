"""Pins for the timing-model oracle (no GPU): the closed form of Sec. 4.2 against an event-by-event
schedule under Eq. limitation, the fit against the textbook normal equations, Theorem 4 (convexity
in 1/r_2) as a property, and hand-worked values."""
import numpy as np
import pytest

from oracle.pipeline_model import (LinearModel, best_r, best_r_overlap, fit_linear, makespan, makespan_overlap,
                                   simulate, simulate_overlap)


def _rand_models(rng):
    return tuple(LinearModel(float(rng.uniform(0.0, 0.5)), float(rng.uniform(1e-5, 1e-3)))
                 for _ in range(3))


def test_hand_worked_makespan():
    """T = 1200 tokens, t_in = 0.1 + 1e-3 m, t_e = 0.2 + 2e-3 m, t_out = 0.1 + 1e-3 m:
    r = 1: 1.3 + 2.6 + 1.3 = 5.2;  r = 3 (m = 400): 0.5 + 1.0 + 0.5 + 2 * 1.0 = 4.0."""
    mi, me, mo = LinearModel(0.1, 1e-3), LinearModel(0.2, 2e-3), LinearModel(0.1, 1e-3)
    assert makespan(1, 1200, mi, me, mo) == pytest.approx(5.2, abs=1e-12)
    assert makespan(3, 1200, mi, me, mo) == pytest.approx(4.0, abs=1e-12)
    # symmetric links: the paper's 2 t_a2e + t_e + (r_2 - 1) max(t_e, t_a2e)
    m = 1200 / 4
    ta2e, te = 0.1 + 1e-3 * m, 0.2 + 2e-3 * m
    assert makespan(4, 1200, mi, me, mo) == pytest.approx(2 * ta2e + te + 3 * max(te, ta2e), abs=1e-12)


def test_closed_form_equals_event_schedule():
    rng = np.random.default_rng(0)
    for _ in range(300):
        mi, me, mo = _rand_models(rng)
        T = float(rng.integers(1, 20000))
        for r in (1, 2, 3, 5, 8, 17, 64):
            assert makespan(r, T, mi, me, mo) == pytest.approx(simulate(r, T, mi, me, mo), rel=1e-12)


def test_convex_in_inverse_r():
    """Theorem 4: the objective is convex in u = 1/r_2 (checked by midpoint convexity on a grid)."""
    rng = np.random.default_rng(1)
    for _ in range(100):
        mi, me, mo = _rand_models(rng)
        T = float(rng.integers(64, 20000))
        f = lambda u: makespan(1.0 / u, T, mi, me, mo)   # real-valued r = 1/u
        us = np.linspace(1.0 / 64, 1.0, 200)
        for a, b in zip(us[:-2], us[2:]):
            assert f(0.5 * (a + b)) <= 0.5 * (f(a) + f(b)) + 1e-9


def test_best_r_special_cases():
    zero = LinearModel(0.0, 0.0)
    # no start-up cost anywhere: more chunks always help -> r_max
    assert best_r(4096, LinearModel(0, 1e-3), LinearModel(0, 1e-3), LinearModel(0, 1e-3), 16) == 16
    # start-up cost only (nothing scales with tokens): chunking can only add -> 1
    assert best_r(4096, LinearModel(0.1, 0), LinearModel(0.2, 0), LinearModel(0.1, 0), 16) == 1
    # transfers free: a single stage, r - 1 extra start-ups -> 1
    assert best_r(4096, zero, LinearModel(0.2, 1e-3), zero, 16) == 1


def test_fit_linear_against_normal_equations():
    rng = np.random.default_rng(2)
    x = rng.uniform(1, 100, 40)
    t = 0.17 + 8.59e-3 * x + rng.normal(0, 0.01, 40)
    a, b, r2 = fit_linear(x, t)
    n, sx, sy, sxx, sxy = len(x), x.sum(), t.sum(), (x * x).sum(), (x * t).sum()
    b_ref = (n * sxy - sx * sy) / (n * sxx - sx * sx)
    a_ref = (sy - b_ref * sx) / n
    assert a == pytest.approx(a_ref, rel=1e-9) and b == pytest.approx(b_ref, rel=1e-9)
    assert 0.99 < r2 <= 1.0
    a, b, r2 = fit_linear([1, 2, 3, 4], [3, 5, 7, 9])      # exact line t = 1 + 2x
    assert (a, b, r2) == (pytest.approx(1.0), pytest.approx(2.0), pytest.approx(1.0))


def test_overlap_models_hand_worked_and_limits():
    """Two sets of task models (alone / beside other tasks).  T = 1200: alone t_in = t_out = 0.1 + 1e-3 m,
    t_e = 0.2 + 2e-3 m -> r = 1: 5.2.  Beside: every task 50 % slower -> r = 3 (m = 400):
    0.75 + 1.5 + 0.75 + 2 * 1.5 = 6.0 > 5.2, so one chunk wins although the paper's model (4.0 at r = 3)
    would cut."""
    alone = (LinearModel(0.1, 1e-3), LinearModel(0.2, 2e-3), LinearModel(0.1, 1e-3))
    beside = tuple(LinearModel(1.5 * m.alpha, 1.5 * m.beta) for m in alone)
    assert makespan_overlap(1, 1200, alone, beside) == pytest.approx(5.2, abs=1e-12)
    assert makespan_overlap(3, 1200, alone, beside) == pytest.approx(6.0, abs=1e-12)
    assert best_r(1200, *alone, 8) > 1 and best_r_overlap(1200, alone, beside, 8) == 1
    # equal sets: the paper's model
    for r in (1, 2, 5):
        assert makespan_overlap(r, 1200, alone, alone) == makespan(r, 1200, *alone)
    assert best_r_overlap(1200, alone, alone, 8) == best_r(1200, *alone, 8)
    # a mild slowdown still leaves chunking ahead
    mild = tuple(LinearModel(1.05 * m.alpha, 1.05 * m.beta) for m in alone)
    assert best_r_overlap(1200, alone, mild, 8) > 1


def test_overlap_closed_form_equals_event_schedule_and_bounds():
    rng = np.random.default_rng(5)
    for _ in range(200):
        alone = _rand_models(rng)
        beside = tuple(LinearModel(m.alpha * float(rng.uniform(1.0, 2.0)), m.beta * float(rng.uniform(1.0, 2.0)))
                       for m in alone)
        T = float(rng.integers(1, 20000))
        for r in (1, 2, 3, 8, 33):
            assert makespan_overlap(r, T, alone, beside) == pytest.approx(simulate_overlap(r, T, alone, beside), rel=1e-12)
            # tasks that are never faster beside others than alone: never better than the paper's model
            assert makespan_overlap(r, T, alone, beside) >= makespan(r, T, *alone) - 1e-12
        rb = best_r_overlap(T, alone, beside, 16)
        assert makespan_overlap(rb, T, alone, beside) == min(makespan_overlap(r, T, alone, beside) for r in range(1, 17))
