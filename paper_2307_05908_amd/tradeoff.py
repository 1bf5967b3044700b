"""Closed forms of the paper's latency / compute analysis (Sec. 4).

Unit: one transformer layer on one token = one time unit on one compute unit.
d = layers, dbar = exit layer, k = early candidates, ell = tokens, p = match
rate p_correct.  Pure host arithmetic, used by the benchmark report to put
the measured layer-row counts next to what the analysis predicts.
"""
from __future__ import annotations


def per_token_latency_mid(d: float, p: float) -> float:
    """Approximate per-token latency for dbar = d/2, ell >> 1 (Eq. 3): d(1 - p/2)."""
    return d * (1.0 - p / 2.0)


def normalized_latency_mid(p: float) -> float:
    """Eq. 3 divided by plain decoding's d time units per token."""
    return 1.0 - p / 2.0


def avg_compute_units_mid(k: int, p: float) -> float:
    """Average busy compute units per time unit for dbar = d/2 (Eq. 5)."""
    return (k + 2.0 - p) / (2.0 - p)


def compute_per_token_mid(k: int, p: float) -> float:
    """Average compute per token in units of d for dbar = d/2 (Eq. 6) = Eq. 3 x Eq. 5 / d."""
    return (2.0 + k - p) / 2.0


def expected_latency(d: int, dbar: int, ell: int, p: float) -> float:
    """Theorem 4.1: expected time units to generate ell tokens."""
    return d * ell - (d - dbar) * (ell - 1) * p


def expected_compute(d: int, dbar: int, ell: int, k: int, p: float) -> float:
    """Theorem 4.1: expected total compute units."""
    return expected_latency(d, dbar, ell, p) + k * (d - dbar) * ell


def latency_of_runs(d: int, dbar: int, ell: int, n_runs: int) -> int:
    """Per-sequence identity in the proof of Theorem 4.1: dbar*ell + (d-dbar)*N."""
    return dbar * ell + (d - dbar) * n_runs


def compute_of_runs(d: int, dbar: int, ell: int, k: int, n_runs: int) -> int:
    """Per-sequence identity in the proof of Theorem 4.1: (dbar + k(d-dbar))*ell + (d-dbar)*N."""
    return (dbar + k * (d - dbar)) * ell + (d - dbar) * n_runs


def run_time(d: int, dbar: int, x: int) -> int:
    """Time units of one run of length x (proof of Theorem 4.1): d + (x-1)*dbar."""
    return d + (x - 1) * dbar
