"""TEST INFRASTRUCTURE ONLY: plain fp64 reference of the paper's SLO-aware partition adjuster.

Nothing in the product path imports this module; only tests, the smoke check and the CPU baseline
of the bench may.  It shares no code with the C++ controller.

Paper, "Dynamic Adjusting Method":
  * Latency modelling (Eq. 1-4): processing latency is inversely proportional to the share,
    l_x = 100 / x * l_100 (Eq. 1); prefill waiting + processing follows an M/M/1 queue,
    w = 1 / (mu_x - r) (Eq. 2), which with mu_x = 1 / l_x gives w ~ 1 / (x - lambda),
    lambda = 100 r l_100 (Eq. 3); hence
        TTFT_x = a1 / (x - lambda) + b1,      TPOT_y = a2 / y + b2          (Eq. 4)
    with a1, lambda, b1, a2, b2 learned from observed latencies.
  * Algorithm 1: every `window_size` iterations take the observed TTFT / TPOT at the SLO's
    percentile, update the two models, and raise the share of the phase whose SLO fails, one
    `step_size` at a time and at most `max_step` times, until the model predicts the SLO is met;
    the prediction uses the share normalised by x + y.

Readings where the paper is silent or the printed algorithm is broken (each is mirrored by the
C++ side and listed in the design notes):
  R1  the loop counter is incremented once per pass (the listing never increments it);
  R2  x' and y' start as the normalised current shares (the listing reads x' before assigning it);
  R3  "both SLOs fail -> keep the partition" is tested first (the prose says so; the listing's
      if / else-if would take the TTFT branch);
  R4  raising a share past 100 lowers the other share by the same step instead; no share goes below
      one step;
  R5  the normalised share is a percentage, 100 x / (x + y), the unit of x in Eq. 4;
  R6  the observed latency "at p_SLO" is the nearest-rank percentile of the window's samples;
      an empty window keeps the partition;
  R7  model fitting is ordinary least squares over the history of (share, observed latency) points,
      one point per window: TPOT on the regressor 1 / y; TTFT on 1 / (x - lambda) with lambda taken
      from the integer grid 0 .. min(x) - 1 that minimises the squared error (a larger lambda wins
      only if it lowers the error by more than 1e-12 (1 + error): ties go to the smallest lambda).  While the history has fewer than two distinct shares the slope cannot be fitted
      and Eq. 1 is used alone: b = 0, lambda = 0, a = latency * share of the latest point;
  R8  the history keeps the latest `history` points (default 64).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field


def estimate_ttft(x: float, a1: float, lam: float, b1: float) -> float:
    """Eq. 4, left.  Shares at or below lambda are saturated queues: infinite waiting time."""
    if x <= lam:
        return math.inf
    return a1 / (x - lam) + b1


def estimate_tpot(y: float, a2: float, b2: float) -> float:
    """Eq. 4, right."""
    return a2 / y + b2


def nearest_rank_percentile(samples, p: float) -> float:
    """Smallest sample such that at least p percent of the samples are <= it (R6)."""
    if not samples:
        raise ValueError("empty window")
    s = sorted(float(v) for v in samples)
    k = max(1, math.ceil(p / 100.0 * len(s)))
    return s[k - 1]


def _ols(us, vs):
    """least squares v = a u + b; returns (a, b, sse)"""
    n = len(us)
    mu, mv = sum(us) / n, sum(vs) / n
    suu = sum((u - mu) ** 2 for u in us)
    suv = sum((u - mu) * (v - mv) for u, v in zip(us, vs))
    a = suv / suu
    b = mv - a * mu
    sse = sum((a * u + b - v) ** 2 for u, v in zip(us, vs))
    return a, b, sse


def fit_tpot(points):
    """points: [(y, tpot)], latest last.  Returns (a2, b2) (R7)."""
    ys = [float(p[0]) for p in points]
    if len(set(ys)) < 2:
        y, t = points[-1]
        return float(t) * float(y), 0.0
    a, b, _ = _ols([1.0 / y for y in ys], [float(p[1]) for p in points])
    return a, b


def fit_ttft(points):
    """points: [(x, ttft)], latest last.  Returns (a1, lambda, b1) (R7)."""
    xs = [float(p[0]) for p in points]
    if len(set(xs)) < 2:
        x, t = points[-1]
        return float(t) * float(x), 0.0, 0.0
    ts = [float(p[1]) for p in points]
    best = None
    for lam in range(0, int(math.ceil(min(xs)))):
        if lam >= min(xs):
            break
        a, b, sse = _ols([1.0 / (x - lam) for x in xs], ts)
        if best is None or sse < best[3] - 1e-12 * (1.0 + best[3]):
            best = (a, float(lam), b, sse)
    return best[0], best[1], best[2]


def increase_share(up: int, other: int, step_size: int):
    """One step for the phase that needs more (R4)."""
    if up + step_size <= 100:
        return up + step_size, other
    return up, max(step_size, other - step_size)


@dataclass
class Adjuster:
    slo_ttft: float
    slo_tpot: float
    p_slo: float = 90.0
    window_size: int = 100
    max_step: int = 4
    step_size: int = 10
    history: int = 64
    ttft_window: list = field(default_factory=list)
    tpot_window: list = field(default_factory=list)
    ttft_points: list = field(default_factory=list)    # (x, observed TTFT), one per window
    tpot_points: list = field(default_factory=list)
    model_ttft: tuple = (0.0, 0.0, 0.0)                 # a1, lambda, b1
    model_tpot: tuple = (0.0, 0.0)                      # a2, b2

    def observe_ttft(self, v: float):
        self.ttft_window.append(float(v))

    def observe_tpot(self, v: float):
        self.tpot_window.append(float(v))

    def step(self, it: int, x0: int, y0: int):
        """Algorithm 1 with the repairs R1-R6.  Returns the partition to use from now on."""
        if it % self.window_size > 0:
            return x0, y0
        if not self.ttft_window or not self.tpot_window:
            self.ttft_window.clear()
            self.tpot_window.clear()
            return x0, y0
        ttft = nearest_rank_percentile(self.ttft_window, self.p_slo)
        tpot = nearest_rank_percentile(self.tpot_window, self.p_slo)
        self.ttft_window.clear()
        self.tpot_window.clear()
        self.ttft_points = (self.ttft_points + [(x0, ttft)])[-self.history:]
        self.tpot_points = (self.tpot_points + [(y0, tpot)])[-self.history:]
        self.model_ttft = fit_ttft(self.ttft_points)
        self.model_tpot = fit_tpot(self.tpot_points)
        ttft_fails, tpot_fails = ttft > self.slo_ttft, tpot > self.slo_tpot
        if ttft_fails and tpot_fails:
            return x0, y0
        x, y = x0, y0
        step = 0
        if ttft_fails:
            xn = 100.0 * x / (x + y)
            while step < self.max_step and estimate_ttft(xn, *self.model_ttft) > self.slo_ttft:
                x, y = increase_share(x, y, self.step_size)
                xn = 100.0 * x / (x + y)
                step += 1
        elif tpot_fails:
            yn = 100.0 * y / (x + y)
            while step < self.max_step and estimate_tpot(yn, *self.model_tpot) > self.slo_tpot:
                y, x = increase_share(y, x, self.step_size)
                yn = 100.0 * y / (x + y)
                step += 1
        return x, y
