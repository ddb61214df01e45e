"""CPU oracle for TIDE's refresh-interval analysis.  TEST INFRASTRUCTURE ONLY.

Plain fp64 statements of the quantities the paper reasons with when it picks the
refresh interval (Sec. 3.2 routing stability; Sec. 3.3 "Interval-based Expert
Refresh", Eq. 4-7), evaluated on per-step expert activation counts
counts[t][e] = number of tokens of step t that selected expert e.

Nothing here is shared with, imported by, or derived from the HIP path.  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import it.

Readings (listed in the design document):
  A1  the "current optimal placement" of step t is the top-B set of that step's own
      counts under (hits descending, lower expert id first); Delta K_t counts the
      experts of step t's set that were not in step t-1's (as many leave as enter).
  A2  a step whose count vector is all zero has similarity 0 with every step,
      itself included.
  A3  Eq. 7 is read as the sum of Eq. 5 and Eq. 6 with the I/O constant kept:
      min over tau in 1..T-1 of  C_io * (B*T/tau) * (1-(1-d)^tau) + C_cpu * T * B * f(tau);
      equal totals are resolved to the smaller tau.  "Greedy search" is read as the
      exhaustive scan of the T-1 candidates (T is a few tens).

Parity pins (tests/test_analysis_pins.py): hand-worked values, scipy's cosine
distance, set arithmetic on a full sort, the closed forms the paper states for the
migration model, and limiting cases of the optimisation whose answer is known.
No function is "parity unpinned" except where noted in the design document for
absolute values that need the paper's data.
"""
from __future__ import annotations

import math
from typing import Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------
# routing stability (Sec. 3.2; Fig. 1a, Fig. 2)
# --------------------------------------------------------------------------
def cosine_similarity_matrix(counts: np.ndarray) -> np.ndarray:
    """sim[i][j] = <c_i, c_j> / (|c_i| |c_j|) over the steps' activation vectors (A2 for zero vectors)."""
    c = np.asarray(counts, dtype=np.float64)
    n_steps = c.shape[0]
    sim = np.zeros((n_steps, n_steps), dtype=np.float64)
    norm = [math.sqrt(float(np.dot(c[i], c[i]))) for i in range(n_steps)]
    for i in range(n_steps):
        for j in range(n_steps):
            if norm[i] > 0.0 and norm[j] > 0.0:
                sim[i, j] = float(np.dot(c[i], c[j])) / (norm[i] * norm[j])
    return sim


def unique_experts(counts: np.ndarray) -> np.ndarray:
    """Number of distinct experts activated at each step (Fig. 2a)."""
    c = np.asarray(counts)
    return np.array([int(sum(1 for v in row if v > 0)) for row in c], dtype=np.int64)


# --------------------------------------------------------------------------
# drift (Eq. 4) and the migration model (Eq. 5)
# --------------------------------------------------------------------------
def top_b_set(hist: np.ndarray, budget: int) -> set:
    ranked = sorted(range(len(hist)), key=lambda e: (-int(hist[e]), e))
    return set(ranked[:budget])


def drift_rates(counts: np.ndarray, budget: int) -> np.ndarray:
    """d_t = |Delta K_t| / B for t = 1..S-1 (Eq. 4, reading A1); d_0 = 0 by convention."""
    c = np.asarray(counts)
    d = np.zeros(c.shape[0], dtype=np.float64)
    prev = top_b_set(c[0], budget)
    for t in range(1, c.shape[0]):
        cur = top_b_set(c[t], budget)
        d[t] = len(cur - prev) / float(budget)
        prev = cur
    return d


def expected_migrations(budget: int, n_steps: int, tau: int, d: float) -> float:
    """Experts moved over n_steps steps when refreshing every tau steps: (B T / tau)(1 - (1-d)^tau)  (Eq. 5 without C_io)."""
    return budget * n_steps / float(tau) * (1.0 - (1.0 - d) ** tau)


def fit_drift(migrations: float, budget: int, n_steps: int, tau: int) -> float:
    """The constant d for which Eq. 5 reproduces a measured migration count."""
    frac = migrations * tau / float(budget * n_steps)
    frac = min(max(frac, 0.0), 1.0)
    return 1.0 - (1.0 - frac) ** (1.0 / tau)


# --------------------------------------------------------------------------
# cost model and the optimal interval (Eq. 5-7)
# --------------------------------------------------------------------------
def lat_io(c_io: float, budget: int, n_steps: int, tau: int, d: float) -> float:
    return c_io * expected_migrations(budget, n_steps, tau, d)


def lat_cpu(c_cpu: float, budget: int, n_steps: int, f_tau: float) -> float:
    """Eq. 6: C_cpu * T * B * f(tau)."""
    return c_cpu * n_steps * budget * f_tau


def interval_costs(budget: int, n_steps: int, d: float, c_io: float, c_cpu: float, f: Sequence[float]) -> np.ndarray:
    """total[tau-1] = Lat_io(tau) + Lat_cpu(tau) for tau = 1..T-1; f[tau-1] = f(tau)."""
    return np.array([lat_io(c_io, budget, n_steps, tau, d) + lat_cpu(c_cpu, budget, n_steps, float(f[tau - 1]))
                     for tau in range(1, n_steps)], dtype=np.float64)


def optimal_interval(budget: int, n_steps: int, d: float, c_io: float, c_cpu: float, f: Sequence[float]) -> Tuple[int, float]:
    """argmin over tau in 1..T-1 of the total cost (Eq. 7, reading A3); returns (tau, cost)."""
    costs = interval_costs(budget, n_steps, d, c_io, c_cpu, f)
    best = 0
    for i in range(1, len(costs)):
        if costs[i] < costs[best]:
            best = i
    return best + 1, float(costs[best])
