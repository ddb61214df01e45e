"""Pins of the interval-analysis oracle (oracle/tide_analysis.py) to things other than itself:
hand-worked fixtures, scikit-learn's cosine similarity, scipy's cosine distance, exact rational
arithmetic, the closed forms the paper states for its migration model, and limiting cases."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import tide_analysis as ana

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "analysis_handworked.json")))


def test_handworked_stability():
    g = GOLD["stability"]
    counts = np.array(g["counts"])
    assert np.allclose(ana.cosine_similarity_matrix(counts), np.array(g["cosine"]), atol=1e-12)
    assert ana.unique_experts(counts).tolist() == g["unique"]
    for t, want in enumerate(g["top_sets"]):
        assert ana.top_b_set(counts[t], g["budget"]) == set(want)
    assert ana.drift_rates(counts, g["budget"]).tolist() == g["drift"]


def test_cosine_against_libraries():
    from scipy.spatial.distance import cosine as cosine_distance
    from sklearn.metrics.pairwise import cosine_similarity
    rng = np.random.default_rng(5)
    counts = rng.poisson(1.0, size=(12, 64))
    counts[7] = 0                                    # a step without any activation
    sim = ana.cosine_similarity_matrix(counts)
    lib = cosine_similarity(counts.astype(np.float64))
    lib[7, :] = 0.0                                   # the library leaves 0/0 at 0 as well; be explicit
    lib[:, 7] = 0.0
    assert np.allclose(sim, lib, atol=1e-12)
    assert abs(sim[2, 5] - (1.0 - cosine_distance(counts[2], counts[5]))) < 1e-12
    assert np.allclose(sim, sim.T) and np.all(sim <= 1 + 1e-12) and np.all(sim >= 0)
    assert np.allclose(np.diag(sim)[[i for i in range(12) if i != 7]], 1.0)
    # scale invariance: a step with twice the tokens and the same mix is identical
    assert abs(ana.cosine_similarity_matrix(np.array([counts[1], 2 * counts[1]]))[0, 1] - 1.0) < 1e-12


def test_unique_and_drift_properties():
    rng = np.random.default_rng(6)
    counts = rng.poisson(0.7, size=(20, 48))
    assert ana.unique_experts(counts).tolist() == np.count_nonzero(counts, axis=1).tolist()
    budget = 8
    d = ana.drift_rates(counts, budget)
    assert d[0] == 0.0
    # an independent statement: full lexicographic sort (numpy), then set difference
    prev = None
    for t in range(counts.shape[0]):
        order = np.lexsort((np.arange(48), -counts[t]))      # last key is primary: hits descending, then id
        cur = set(order[:budget].tolist())
        if prev is not None:
            assert d[t] == len(cur - prev) / budget == len(prev - cur) / budget
        prev = cur
    assert set(np.round(d * budget).astype(int)) <= set(range(budget + 1))
    same = np.tile(counts[3], (4, 1))
    assert ana.drift_rates(same, budget).tolist() == [0.0] * 4
    a = np.zeros((2, 32), dtype=int)
    a[0, :8] = 5
    a[1, 8:16] = 5
    assert ana.drift_rates(a, 8).tolist() == [0.0, 1.0]      # disjoint hot sets: everything moves


def test_migration_model_closed_forms():
    g = GOLD["migrations"]
    assert abs(ana.expected_migrations(g["budget"], g["n_steps"], g["tau"], g["d"]) - g["expected"]) < 1e-9
    # the paper: at tau = 1 the model is the full-refresh baseline B*T*d
    assert abs(ana.expected_migrations(g["budget"], g["n_steps"], 1, g["d"]) - g["at_tau_1"]) < 1e-9
    for B, T, d in ((64, 32, 0.05), (32, 64, 0.3), (128, 16, 0.9)):
        assert abs(ana.expected_migrations(B, T, 1, d) - B * T * d) < 1e-9
        # as tau grows the model tends to B*T/tau
        assert abs(ana.expected_migrations(B, T, 400, d) * 400 / (B * T) - 1.0) < 1e-6
        m = [ana.expected_migrations(B, T, tau, d) for tau in range(1, T)]
        assert all(x > y for x, y in zip(m, m[1:]))          # fewer migrations with a longer interval
        # constant d in the product form of the survival probability
        for tau in (1, 3, 7):
            surv = 1.0
            for _ in range(tau):
                surv *= (1.0 - d)
            assert abs(ana.expected_migrations(B, T, tau, d) - B * T / tau * (1.0 - surv)) < 1e-9
            assert abs(ana.fit_drift(ana.expected_migrations(B, T, tau, d), B, T, tau) - d) < 1e-9    # the inverse is ill-conditioned near d = 1
    assert ana.expected_migrations(64, 32, 4, 0.0) == 0.0
    assert abs(ana.expected_migrations(64, 32, 4, 1.0) - 64 * 32 / 4) < 1e-12


def test_handworked_optimum_and_limits():
    g = GOLD["optimum"]
    B, T, d, cio, ccpu, f = g["budget"], g["n_steps"], g["d"], g["c_io"], g["c_cpu"], g["f"]
    for tau in range(1, T):
        assert abs(ana.lat_io(cio, B, T, tau, d) - g["lat_io"][tau - 1]) < 1e-12
        assert abs(ana.lat_cpu(ccpu, B, T, f[tau - 1]) - g["lat_cpu"][tau - 1]) < 1e-12
    assert ana.optimal_interval(B, T, d, cio, ccpu, f) == (g["tau"], pytest.approx(g["cost"], abs=1e-12))
    # no CPU cost: the longest interval wins; no I/O cost and a strictly increasing miss curve: refresh every step
    f_inc = [0.01 * tau * tau for tau in range(1, 32)]
    assert ana.optimal_interval(64, 32, 0.1, 1.0, 0.0, f_inc)[0] == 31
    assert ana.optimal_interval(64, 32, 0.1, 0.0, 1.0, f_inc)[0] == 1
    # equal totals: the smaller interval
    assert ana.optimal_interval(4, 6, 0.0, 1.0, 1.0, [0.5] * 5)[0] == 1


def test_optimum_against_exact_rational_arithmetic():
    rng = np.random.default_rng(8)
    for _ in range(20):
        B, T = int(rng.integers(1, 100)), int(rng.integers(3, 40))
        d = Fraction(int(rng.integers(0, 50)), 64)
        cio, ccpu = Fraction(int(rng.integers(1, 64)), 8), Fraction(int(rng.integers(0, 64)), 16)
        f = np.cumsum(rng.integers(0, 5, size=T - 1)).tolist()
        exact = [cio * Fraction(B * T, tau) * (1 - (1 - d) ** tau) + ccpu * T * B * Fraction(f[tau - 1], 64) for tau in range(1, T)]
        want = min(range(len(exact)), key=lambda i: (exact[i], i)) + 1
        tau, cost = ana.optimal_interval(B, T, float(d), float(cio), float(ccpu), [v / 64 for v in f])
        # floating point may break an exact tie differently only if two exact totals are equal
        if exact.count(min(exact)) == 1:
            assert tau == want
        assert abs(cost - float(min(exact))) <= 1e-9 * max(1.0, float(min(exact)))
