"""Pins of the oracle's SLO-aware partition adjuster (paper, "Dynamic Adjusting Method": Eq. 1-4,
Algorithm 1) against what the paper and the mathematics fix: the queueing derivation, closed forms,
a library least-squares routine, textbook percentile examples, a hand-worked trace, invariants."""
import math
import os
import random

import numpy as np
import pytest

from oracle import controller as OC

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "controller_trace.txt")


def test_eq1_latency_is_inversely_proportional_to_the_share():
    # Eq. 1: l_x = 100 / x * l_100; with b = 0 and lambda = 0 Eq. 4 is Eq. 1
    l100 = 7.5
    for x in (10, 25, 50, 100):
        assert OC.estimate_tpot(x, 100 * l100, 0.0) == pytest.approx(100.0 / x * l100, rel=1e-15)
        assert OC.estimate_ttft(x, 100 * l100, 0.0, 0.0) == pytest.approx(100.0 / x * l100, rel=1e-15)
    assert OC.estimate_tpot(50, 750, 0) == pytest.approx(2 * OC.estimate_tpot(100, 750, 0))


def test_eq2_eq3_mm1_waiting_time_has_the_shape_of_eq4():
    # Eq. 2: w = 1 / (mu_x - r), mu_x = 1 / l_x, l_x from Eq. 1.  Eq. 3: w = 100 l_100 / (x - lambda),
    # lambda = 100 r l_100.  The two must agree wherever the queue is stable.
    l100, r = 0.02, 12.0                     # 20 ms prefill at the full GPU, 12 requests / s
    lam = 100 * r * l100                     # 24 percent
    for x in (25, 30, 50, 80, 100):
        mu = x / (100.0 * l100)
        assert OC.estimate_ttft(x, 100 * l100, lam, 0.0) == pytest.approx(1.0 / (mu - r), rel=1e-12)
    assert OC.estimate_ttft(24, 100 * l100, lam, 0.0) == math.inf      # saturated: the queue grows without bound
    assert OC.estimate_ttft(10, 100 * l100, lam, 0.0) == math.inf


def test_fit_recovers_exact_parameters():
    a1, lam, b1 = 300.0, 12.0, 5.0
    pts = [(x, a1 / (x - lam) + b1) for x in (30, 40, 60, 80, 50)]
    fa, fl, fb = OC.fit_ttft(pts)
    assert fl == lam and fa == pytest.approx(a1, rel=1e-9) and fb == pytest.approx(b1, rel=1e-8)
    a2, b2 = 400.0, 3.0
    pts = [(y, a2 / y + b2) for y in (20, 50, 70, 50)]
    fa, fb = OC.fit_tpot(pts)
    assert fa == pytest.approx(a2, rel=1e-10) and fb == pytest.approx(b2, rel=1e-9)


def test_fit_is_ordinary_least_squares_library_cross_check():
    rng = np.random.default_rng(3)
    ys = rng.integers(10, 101, size=12)
    ts = 500.0 / ys + 4.0 + rng.normal(0, 0.3, size=12)
    a, b = OC.fit_tpot(list(zip(ys.tolist(), ts.tolist())))
    pa, pb = np.polyfit(1.0 / ys, ts, 1)
    assert a == pytest.approx(pa, rel=1e-9) and b == pytest.approx(pb, rel=1e-8)
    # TTFT: lambda is the grid point whose straight-line fit (library routine) leaves the least error
    xs = rng.integers(30, 101, size=14)
    tt = 900.0 / (xs - 17.0) + 20.0 + rng.normal(0, 0.05, size=14)
    a1, lam, b1 = OC.fit_ttft(list(zip(xs.tolist(), tt.tolist())))
    sse = []
    for cand in range(0, int(xs.min())):
        coef = np.polyfit(1.0 / (xs - cand), tt, 1)
        sse.append(float(((np.polyval(coef, 1.0 / (xs - cand)) - tt) ** 2).sum()))
    assert lam == float(np.argmin(sse)) == 17.0
    pa, pb = np.polyfit(1.0 / (xs - lam), tt, 1)
    assert a1 == pytest.approx(pa, rel=1e-8) and b1 == pytest.approx(pb, rel=1e-7)


def test_single_share_history_falls_back_to_eq1():
    a1, lam, b1 = OC.fit_ttft([(40, 90.0), (40, 120.0)])
    assert (a1, lam, b1) == (120.0 * 40, 0.0, 0.0)
    assert OC.estimate_ttft(80, a1, lam, b1) == pytest.approx(60.0)          # twice the share, half the latency
    a2, b2 = OC.fit_tpot([(25, 8.0)])
    assert (a2, b2) == (200.0, 0.0)


def test_nearest_rank_percentile_textbook_cases():
    five = [15, 20, 35, 40, 50]
    assert [OC.nearest_rank_percentile(five, p) for p in (5, 30, 40, 50, 100)] == [15, 20, 20, 35, 50]
    ten = [3, 6, 7, 8, 8, 10, 13, 15, 16, 20]
    assert [OC.nearest_rank_percentile(ten, p) for p in (25, 50, 75, 90, 100)] == [7, 8, 15, 16, 20]
    assert OC.nearest_rank_percentile(list(range(1, 101)), 90) == 90
    with pytest.raises(ValueError):
        OC.nearest_rank_percentile([], 90)


def _samples_with_p90(v):
    """ten samples whose 9th smallest is v"""
    return [v * 0.5] * 8 + [v, v * 3.0]


def test_hand_worked_trace():
    runs = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if not line:
            continue
        run, it, x0, y0, ttft, tpot, x, y = line[0], *[float(v) for v in line[1:]]
        adj = runs.setdefault(run, OC.Adjuster(slo_ttft=100.0, slo_tpot=20.0, p_slo=90.0, window_size=1, max_step=4, step_size=10))
        for v in _samples_with_p90(ttft):
            adj.observe_ttft(v)
        for v in _samples_with_p90(tpot):
            adj.observe_tpot(v)
        assert adj.step(int(it), int(x0), int(y0)) == (int(x), int(y)), f"run {run} window {int(it)}"
    assert set(runs) == {"A", "B", "C", "D"}


def test_invariants_under_random_observations():
    rnd = random.Random(11)
    for trial in range(200):
        step_size = rnd.choice((5, 10, 20))
        adj = OC.Adjuster(slo_ttft=rnd.uniform(50, 400), slo_tpot=rnd.uniform(5, 60), p_slo=rnd.choice((50.0, 90.0, 99.0)),
                          window_size=rnd.choice((1, 3, 8)), max_step=rnd.choice((1, 2, 4)), step_size=step_size)
        x, y = rnd.choice(range(step_size, 101, step_size)), rnd.choice(range(step_size, 101, step_size))
        for it in range(40):
            for _ in range(rnd.randint(0, 6)):
                adj.observe_ttft(rnd.uniform(10, 600))
                adj.observe_tpot(rnd.uniform(1, 90))
            had = bool(adj.ttft_window) and bool(adj.tpot_window)
            nx, ny = adj.step(it, x, y)
            assert step_size <= nx <= 100 and step_size <= ny <= 100
            if it % adj.window_size > 0 or not had:
                assert (nx, ny) == (x, y)
            # one phase is favoured per window, by at most max_step steps
            assert not (nx > x and ny > y)
            assert abs(nx - x) + abs(ny - y) <= adj.max_step * step_size
            assert (nx - x) % step_size == 0 and (ny - y) % step_size == 0
            x, y = nx, ny


def test_share_moves_towards_the_failing_phase_only():
    adj = OC.Adjuster(slo_ttft=100.0, slo_tpot=20.0, window_size=1)
    for v in _samples_with_p90(400.0):
        adj.observe_ttft(v)
    for v in _samples_with_p90(5.0):
        adj.observe_tpot(v)
    x, y = adj.step(0, 30, 70)
    assert x > 30 and y == 70
    adj = OC.Adjuster(slo_ttft=100.0, slo_tpot=20.0, window_size=1)
    for v in _samples_with_p90(40.0):
        adj.observe_ttft(v)
    for v in _samples_with_p90(50.0):
        adj.observe_tpot(v)
    x, y = adj.step(0, 70, 30)
    assert x == 70 and y > 30
