"""The library's host-side granularity controller (Section 6.1 Eq. 4-5, Section 6.2, Section 7
Eq. 11 and the SLO constraint) against the oracle's formulas on seeded random inputs, plus the
error paths.  Host arithmetic only: runs without a GPU."""
import numpy as np
import pytest

from oracle import control
from paper_2510_11938_amd import binding


def test_cv_matches_oracle():
    rng = np.random.default_rng(5)
    for n in (1, 2, 17, 4096):
        x = rng.gamma(0.7, 3.0, size=n) + 1e-3
        assert binding.ctl_cv(x) == pytest.approx(control.coefficient_of_variation(x), rel=1e-12, abs=1e-15)
    with pytest.raises(binding.FxpError):
        binding.ctl_cv([])
    with pytest.raises(binding.FxpError):
        binding.ctl_cv([0.0, 0.0])


def test_granularity_selection_matches_oracle():
    rng = np.random.default_rng(6)
    for trial in range(200):
        K = int(rng.integers(1, 9))
        T, L, nu = rng.uniform(1, 500, K), rng.uniform(0.5, 80, K), rng.uniform(0, 4, K)
        nu_t, alpha, sigma = float(rng.uniform(0, 5)), float(rng.uniform(0, 1)), float(rng.uniform(0.05, 3))
        cands = [binding.Granularity(2 ** (k % 6), 8, float(T[k]), float(L[k]), float(nu[k])) for k in range(K)]
        best, scores = binding.ctl_select_granularity(cands, nu_t, alpha, sigma)
        want = control.granularity_scores(T, L, nu, nu_t, alpha, sigma)
        np.testing.assert_allclose(scores, want, rtol=1e-13)
        assert best == control.select_granularity(T, L, nu, nu_t, alpha, sigma)
    tie = [binding.Granularity(1, 1, 5.0, 1.0, 1.0), binding.Granularity(2, 1, 5.0, 1.0, 1.0)]
    assert binding.ctl_select_granularity(tie, 1.0, 0.5, 1.0)[0] == 0
    with pytest.raises(binding.FxpError):
        binding.ctl_select_granularity(tie, 1.0, 1.5, 1.0)            # alpha outside [0,1]
    with pytest.raises(binding.FxpError):
        binding.ctl_select_granularity(tie, 1.0, 0.5, 0.0)            # sigma must be positive
    with pytest.raises(binding.FxpError):
        binding.ctl_select_granularity([binding.Granularity(1, 1, 0.0, 1.0, 1.0)], 1.0, 0.5, 1.0)


def test_instances_penalty_scaling_and_slo_match_oracle():
    rng = np.random.default_rng(7)
    for trial in range(300):
        cap, T = float(rng.uniform(0, 1e4)), float(rng.uniform(1, 500))
        b1, b2, eta = float(rng.uniform(0.1, 2)), float(rng.uniform(0, 1)), int(rng.integers(1, 65))
        assert binding.ctl_parallel_instances(cap, T, b1, b2, eta) == control.parallel_instances(cap, T, b1, b2, eta)
        g0, al, cv = float(rng.uniform(0, 1)), float(rng.uniform(0, 2)), float(rng.uniform(0, 6))
        assert binding.ctl_multiplexing_penalty(g0, al, cv) == pytest.approx(control.multiplexing_penalty(g0, al, cv), rel=1e-14)
        G, be, ga = int(rng.integers(1, 65)), float(rng.uniform(0, 10)), float(rng.uniform(0, 5))
        q, Q = float(rng.uniform(0, 300)), float(rng.uniform(1, 200))
        assert binding.ctl_scaling_granularity(G, be, ga, cv, q, Q) == control.scaling_granularity(G, be, ga, cv, q, Q)
        mu = rng.uniform(0.1, 50, int(rng.integers(1, 9)))
        dl, init, ql, req = float(rng.uniform(1, 30)), float(rng.uniform(0, 5)), float(rng.uniform(1, 100)), float(rng.uniform(0, 40))
        assert binding.ctl_slo_satisfied(dl, init, mu, ql, req) == control.slo_satisfied(dl, init, mu, ql, req)
    with pytest.raises(binding.FxpError):
        binding.ctl_parallel_instances(10.0, 0.0, 1.0, 1.0, 4)
    with pytest.raises(binding.FxpError):
        binding.ctl_scaling_granularity(0, 1.0, 1.0, 1.0, 1.0, 1.0)
    with pytest.raises(binding.FxpError):
        binding.ctl_slo_satisfied(1.0, 0.0, [1.0], 0.0, 1.0)
