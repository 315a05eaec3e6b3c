"""Closed-form token-rate model of the paper (Sec. 3.3, Eq. 1-6) and a Monte Carlo of the
acceptance chain it describes.  Test infrastructure only; host-side, no GPU.

Notation follows the paper: alpha = per-token acceptance probability between two
consecutive stages, gamma = window size, rho = probability that a step of M_i is a
verification step, c = draft/target speed ratio.
"""
import numpy as np


def geometric_tokens(alpha, gamma):
    """Expected tokens of a verification step: (1 - alpha^(gamma+1)) / (1 - alpha)  (Eq. 1, second term)."""
    return (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha)


def rho_iterates(alpha, gamma, n):
    """rho(t_0..t_n) from the recursion of Eq. 2, rho(t_0) = alpha, applied for every j >= 1."""
    out = np.empty(n + 1)
    out[0] = alpha
    for j in range(1, n + 1):
        out[j] = out[j - 1] * alpha ** (gamma + 1) + (1.0 - out[j - 1]) * alpha
    return out


def rho_steady(alpha, gamma):
    """Steady-state verification probability, Eq. 3."""
    return alpha / (1.0 - alpha ** (gamma + 1) + alpha)


def expected_tokens(alpha, gamma, rho=None):
    """E[N(M_i)] per decoding step, Eq. 1 (= PipeSpec(P) of Eq. 4 with the steady-state rho)."""
    if rho is None:
        rho = rho_steady(alpha, gamma)
    return (1.0 - rho) * 1.0 + rho * geometric_tokens(alpha, gamma)


def sd_speedup(alpha, gamma, c):
    """Synchronous speculative decoding, Eq. 5."""
    return (1.0 - alpha ** (gamma + 1)) / ((1.0 - alpha) * (gamma / c + 1.0))


def pipespec_high_alpha(alpha, gamma):
    """High-acceptance approximation, Eq. 6."""
    return geometric_tokens(alpha, gamma)


def monte_carlo(alpha, gamma, steps, seed):
    """Simulate the two-state chain behind Eq. 1-3 with Bernoulli(alpha) acceptances.

    State V (verification step): draw gamma acceptances; the step yields 1 + (number of
    leading successes) tokens; the next step is again V iff all gamma succeeded and one
    further Bernoulli(alpha) (the first token of the next window matching the verifier's
    new token) succeeds.  State N (no verification): 1 token; next step is V w.p. alpha.
    The first step is V w.p. alpha.  Returns (mean tokens/step, fraction of V steps,
    standard error of the mean tokens/step).
    """
    rng = np.random.default_rng(seed)
    in_v = rng.random() < alpha
    tokens = np.empty(steps)
    n_v = 0
    for t in range(steps):
        if in_v:
            n_v += 1
            acc = rng.random(gamma) < alpha
            lead = gamma if acc.all() else int(np.argmin(acc))
            tokens[t] = 1 + lead
            in_v = (lead == gamma) and (rng.random() < alpha)
        else:
            tokens[t] = 1
            in_v = rng.random() < alpha
    return tokens.mean(), n_v / steps, tokens.std(ddof=1) / np.sqrt(steps)


def accepted_length_pmf(alpha, gamma):
    """P(n = k), k = 0..gamma, when each of gamma compared positions matches independently w.p. alpha."""
    p = np.array([alpha ** k * (1.0 - alpha) for k in range(gamma)] + [alpha ** gamma])
    return p
