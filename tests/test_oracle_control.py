"""Pins for the oracle's granularity-control formulas (Section 6.1 Eq. 4-5, Section 6.2,
Section 7 Eq. 11 and the SLO constraint): hand-worked values, limits and monotonicity
that the formulas fix, so that a dropped term, a swapped ratio or a wrong sign fails."""
import math

import numpy as np
import pytest

from oracle import control


def test_cv_of_known_samples():
    assert control.coefficient_of_variation([2.0, 2.0, 2.0]) == 0.0                 # steady arrivals
    assert control.coefficient_of_variation([1.0, 3.0]) == pytest.approx(0.5)        # mean 2, deviation 1
    assert control.coefficient_of_variation([0.0, 0.0, 0.0, 4.0]) == pytest.approx(math.sqrt(3.0))   # mean 1, variance 3
    x = np.random.default_rng(0).exponential(2.5, size=200000)                       # Poisson arrivals: CV -> 1
    assert control.coefficient_of_variation(x) == pytest.approx(1.0, abs=0.01)
    assert control.coefficient_of_variation(10 * x) == pytest.approx(control.coefficient_of_variation(x))   # scale-free


def test_scores_hand_worked_two_candidates():
    # g1: T=100, L=10, nu=0.5 ; g2: T=50, L=5, nu=2 ; alpha=0.5, sigma=1  =>  T_max=100, L_min=5
    # bracket(g1) = 0.5*1 + 0.5*(5/10) = 0.75 ; bracket(g2) = 0.5*0.5 + 0.5*1 = 0.75
    s = control.granularity_scores([100, 50], [10, 5], [0.5, 2.0], nu_t=0.5, alpha=0.5, sigma=1.0)
    assert s[0] == pytest.approx(0.75)
    assert s[1] == pytest.approx(0.75 * 0.22313016014842982)      # exp(-1.5)
    assert control.select_granularity([100, 50], [10, 5], [0.5, 2.0], 0.5, 0.5, 1.0) == 0
    assert control.select_granularity([100, 50], [10, 5], [0.5, 2.0], 2.0, 0.5, 1.0) == 1     # bursty traffic: the fine one


def test_scores_limits():
    T, L, nu = [80.0, 100.0, 60.0], [4.0, 8.0, 2.0], [1.0, 1.0, 1.0]
    assert control.select_granularity(T, L, nu, 1.0, alpha=1.0, sigma=1.0) == 1      # throughput only: largest T
    assert control.select_granularity(T, L, nu, 1.0, alpha=0.0, sigma=1.0) == 2      # latency only: smallest L
    s = control.granularity_scores(T, L, nu, 1.0, 1.0, 1.0)
    assert s[1] == pytest.approx(1.0) and s[0] == pytest.approx(0.8)                 # T/T_max with a matching term of 1
    s = control.granularity_scores(T, L, nu, 1.0, 0.0, 1.0)
    assert s[2] == pytest.approx(1.0) and s[1] == pytest.approx(0.25)                # L_min/L
    # sharper sigma makes the match decide; the matching term is symmetric in nu_t - nu_k
    a = control.granularity_scores([1, 1], [1, 1], [1.0, 3.0], 2.0, 0.5, 0.7)
    assert a[0] == pytest.approx(a[1])
    wide = control.granularity_scores([1, 1], [1, 1], [1.0, 3.0], 1.0, 0.5, 100.0)
    assert wide[1] / wide[0] == pytest.approx(math.exp(-0.02))
    assert control.select_granularity([5, 5], [1, 1], [1.0, 1.0], 1.0, 0.5, 1.0) == 0  # tie: lowest index


def test_parallel_instances_hand_worked():
    # mu_k = 100 / (1 + 0.25*4) = 50 ; floor(1000 / 50) = 20
    assert control.parallel_instances(1000.0, 100.0, 1.0, 0.25, 4) == 20
    # more stages, more coordination overhead, lower per-instance capacity => more instances needed
    assert control.parallel_instances(1000.0, 100.0, 1.0, 0.25, 12) == 40
    assert control.parallel_instances(1049.0, 100.0, 1.0, 0.25, 4) == 20             # floor
    assert control.parallel_instances(10.0, 100.0, 1.0, 0.0, 4) == 0


def test_multiplexing_penalty():
    assert control.multiplexing_penalty(0.2, 0.5, 0.0) == pytest.approx(0.2)          # stable workload: the base penalty
    assert control.multiplexing_penalty(0.2, 0.5, 2.0) == pytest.approx(0.6)          # 0.2 * (1 + 0.5*4)
    assert control.multiplexing_penalty(0.2, 0.5, -2.0) == pytest.approx(0.6)         # quadratic in CV


def test_scaling_granularity_sigmoid():
    # empty queue: floor(8 / (1 + 3)) = 2, whatever the CV
    assert control.scaling_granularity(8, 3.0, 2.0, cv=5.0, q=0.0, Q_max=100.0) == 2
    # cv=2, full queue: 8 / (1 + 3*exp(-4)) = 8 / 1.054947 = 7.58 -> 7
    assert control.scaling_granularity(8, 3.0, 2.0, cv=2.0, q=100.0, Q_max=100.0) == 7
    assert control.scaling_granularity(8, 3.0, 2.0, cv=2.0, q=1e9, Q_max=100.0) == 7  # queue length saturates at the capacity
    # cv * q_hat = ln(3)/2 makes the denominator exactly 2
    assert control.scaling_granularity(8, 3.0, 2.0, cv=math.log(3.0) / 2 + 1e-12, q=100.0, Q_max=100.0) == 4
    prev = 0
    for q in range(0, 101, 5):                                                         # finer with load, never coarser
        m = control.scaling_granularity(16, 4.0, 3.0, 1.5, float(q), 100.0)
        assert m >= prev
        prev = m
    assert control.scaling_granularity(16, 4.0, 3.0, 1.5, 100.0, 100.0) < 16 + 1


def test_slo_constraint():
    # (10 - 2) * (3 + 5) / 16 = 4 requests within the deadline
    assert control.slo_satisfied(10.0, 2.0, [3.0, 5.0], 16.0, 4.0)
    assert not control.slo_satisfied(10.0, 2.0, [3.0, 5.0], 16.0, 4.01)
    assert not control.slo_satisfied(10.0, 9.5, [3.0, 5.0], 16.0, 1.0)                 # initialisation eats the deadline
