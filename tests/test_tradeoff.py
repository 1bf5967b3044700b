"""The closed forms of Sec. 4 against the values the paper prints."""
import os

import numpy as np
import pytest

from paper_2307_05908_amd import tradeoff as T

GOLD = os.path.join(os.path.dirname(__file__), "golden", "tradeoff_paper_values.txt")


def _rows():
    for line in open(GOLD):
        line = line.strip()
        if line and not line.startswith("#"):
            q, k, p, v, tol = line.split()
            yield q, int(k), float(p), float(v), float(tol)


@pytest.mark.parametrize("q,k,p,v,tol", list(_rows()))
def test_printed_values(q, k, p, v, tol):
    got = T.normalized_latency_mid(p) if q == "norm_latency" else T.avg_compute_units_mid(k, p)
    assert abs(got - v) <= tol


def test_eq6_is_eq3_times_eq5():
    for k in (1, 3, 5):
        for p in np.linspace(0, 1, 11):
            assert abs(T.compute_per_token_mid(k, p) - T.normalized_latency_mid(p) * T.avg_compute_units_mid(k, p)) < 1e-12


def test_theorem_is_expectation_of_identities():
    """E[N] = l - (l-1)p with N - 1 ~ Bin(l-1, 1-p) (proof of Theorem 4.1): enumerate the binomial."""
    from math import comb
    d, dbar, ell, k, p = 40, 24, 9, 3, 0.37
    eN = sum(comb(ell - 1, j) * (1 - p) ** j * p ** (ell - 1 - j) * (1 + j) for j in range(ell))
    assert abs(eN - (ell - (ell - 1) * p)) < 1e-12
    lat = sum(comb(ell - 1, j) * (1 - p) ** j * p ** (ell - 1 - j) * T.latency_of_runs(d, dbar, ell, 1 + j) for j in range(ell))
    com = sum(comb(ell - 1, j) * (1 - p) ** j * p ** (ell - 1 - j) * T.compute_of_runs(d, dbar, ell, k, 1 + j) for j in range(ell))
    assert abs(lat - T.expected_latency(d, dbar, ell, p)) < 1e-9
    assert abs(com - T.expected_compute(d, dbar, ell, k, p)) < 1e-9
    # runs of lengths X_i summing to l take sum(d + (X_i - 1) dbar) time units
    X = [3, 1, 4, 1]
    assert sum(T.run_time(d, dbar, x) for x in X) == T.latency_of_runs(d, dbar, sum(X), len(X))
    # for large l and dbar = d/2 the theorem tends to Eq. 3
    assert abs(T.expected_latency(40, 20, 10**6, 0.5) / 10**6 - T.per_token_latency_mid(40, 0.5)) < 1e-4
