"""Oracle for the granularity-control formulas (Section 6.1, Eq. 4 and Eq. 5;
Section 6.2, the multiplexing penalty; Section 7, Eq. 11 and the SLO constraint).

TEST INFRASTRUCTURE ONLY: plain float64 numpy statements of the paper's scalar
formulas in the paper's notation, used by the tests to check the library's
host-side controller.  Nothing in the product imports this module.

Readings where the paper leaves a choice (also listed in the design document):
  * the coefficient of variation uses the population standard deviation of the
    arrival intervals (nu_t = sigma_t / mu_t);
  * the normalisation constants of Eq. 4 are taken over the candidate set:
    T_max = max_k T_k, L_min = min_k L_k;
  * ties of the arg max go to the lowest index k.
"""
from __future__ import annotations

import math
from typing import Sequence

import numpy as np


def coefficient_of_variation(intervals: Sequence[float]) -> float:
    """nu_t = sigma_t / mu_t of the request arrival intervals (Section 6)."""
    x = np.asarray(intervals, dtype=np.float64)
    return float(np.std(x) / np.mean(x))


def granularity_scores(T: Sequence[float], L: Sequence[float], nu_k: Sequence[float], nu_t: float,
                       alpha: float, sigma: float) -> np.ndarray:
    """Eq. 4, the bracket times the matching term, for every candidate k."""
    T = np.asarray(T, dtype=np.float64)
    L = np.asarray(L, dtype=np.float64)
    nu_k = np.asarray(nu_k, dtype=np.float64)
    T_max, L_min = T.max(), L.min()
    return (alpha * T / T_max + (1.0 - alpha) * L_min / L) * np.exp(-np.abs(nu_t - nu_k) / sigma)


def select_granularity(T, L, nu_k, nu_t: float, alpha: float, sigma: float) -> int:
    """g* = arg max_k of Eq. 4."""
    return int(np.argmax(granularity_scores(T, L, nu_k, nu_t, alpha, sigma)))


def parallel_instances(mu_total: float, T_k: float, beta1: float, beta2: float, eta_k: int) -> int:
    """Eq. 5: M(g_k) = floor(mu_total / mu_k), mu_k = T_k / (beta1 + beta2 * eta_k)."""
    mu_k = T_k / (beta1 + beta2 * eta_k)
    return int(math.floor(mu_total / mu_k))


def multiplexing_penalty(gamma0: float, alpha: float, cv: float) -> float:
    """gamma(CV) = gamma0 * (1 + alpha * CV^2) (Section 6.2)."""
    return gamma0 * (1.0 + alpha * cv * cv)


def scaling_granularity(G_max: int, beta: float, gamma: float, cv: float, q: float, Q_max: float) -> int:
    """Eq. 11: m = floor(G_max / (1 + beta * exp(-gamma * cv * q_hat))), q_hat = min(q / Q_max, 1)."""
    q_hat = min(q / Q_max, 1.0)
    return int(math.floor(G_max / (1.0 + beta * math.exp(-gamma * cv * q_hat))))


def slo_satisfied(T_j: float, S_j: float, mu_jk: Sequence[float], Q_j: float, r_j: float) -> bool:
    """Section 7's constraint: (T_j - S_j) * sum_k mu_jk / Q_j >= r_j."""
    return bool((T_j - S_j) * float(np.sum(np.asarray(mu_jk, dtype=np.float64))) / Q_j >= r_j)
