"""Closed-form rate model (paper Sec. 3.3, Eq. 1-6) against Monte Carlo and algebra."""
import numpy as np
import pytest
from oracle import ratecheck as rc

CASES = [(0.7, 4), (0.5, 8), (0.8, 8), (0.7, 8), (0.6, 8), (0.7, 1), (0.7, 16)]


@pytest.mark.parametrize("alpha,gamma", CASES)
def test_eq1_eq3_match_monte_carlo(alpha, gamma):
    mean, frac_v, se = rc.monte_carlo(alpha, gamma, 300_000, seed=int(alpha * 100) * 97 + gamma)
    assert abs(mean - rc.expected_tokens(alpha, gamma)) < 4 * se + 1e-3
    rho = rc.rho_steady(alpha, gamma)
    assert abs(frac_v - rho) < 4 * np.sqrt(rho * (1 - rho) / 300_000) * 3 + 1e-3


@pytest.mark.parametrize("alpha,gamma", CASES)
def test_eq3_is_fixed_point_and_cesaro_limit_of_eq2(alpha, gamma):
    rho = rc.rho_steady(alpha, gamma)
    assert abs(rho * alpha ** (gamma + 1) + (1 - rho) * alpha - rho) < 1e-14
    it = rc.rho_iterates(alpha, gamma, 4000)
    assert abs(it.mean() - rho) < 1e-3
    # iterates follow rho* + (alpha - rho*) (alpha^(gamma+1) - alpha)^j
    j = np.arange(20)
    assert np.allclose(it[:20], rho + (alpha - rho) * (alpha ** (gamma + 1) - alpha) ** j, atol=1e-14)


def test_geometric_sum_is_sum_of_powers():
    for alpha, gamma in CASES:
        assert abs(rc.geometric_tokens(alpha, gamma) - sum(alpha ** k for k in range(gamma + 1))) < 1e-12


def test_theorem1_more_than_one_token_per_step():
    for alpha in np.linspace(0.01, 0.99, 50):
        for gamma in range(1, 33):
            assert rc.expected_tokens(alpha, gamma) > 1.0


def test_eq6_is_upper_envelope_and_eq5_below_it():
    for alpha, gamma in CASES:
        assert rc.expected_tokens(alpha, gamma) < rc.pipespec_high_alpha(alpha, gamma)
        assert abs(rc.expected_tokens(alpha, gamma, rho=1.0) - rc.pipespec_high_alpha(alpha, gamma)) < 1e-12
        for c in (2.0, 4.0, 10.0):
            assert rc.sd_speedup(alpha, gamma, c) < rc.pipespec_high_alpha(alpha, gamma)
    # as the drafter becomes free (c -> inf) synchronous SD reaches the same envelope
    assert abs(rc.sd_speedup(0.7, 8, 1e12) - rc.pipespec_high_alpha(0.7, 8)) < 1e-9
    # low acceptance: synchronous SD loses to autoregressive decoding, PipeSpec does not
    assert rc.sd_speedup(0.1, 8, 4.0) < 1.0 < rc.expected_tokens(0.1, 8)


def test_accepted_length_pmf_sums_to_one_and_mean():
    for alpha, gamma in CASES:
        p = rc.accepted_length_pmf(alpha, gamma)
        assert abs(p.sum() - 1) < 1e-12
        assert abs((p * np.arange(gamma + 1)).sum() - alpha * (1 - alpha ** gamma) / (1 - alpha)) < 1e-12
