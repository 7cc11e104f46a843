"""Oracle: the closed forms of section 3 and appendix A.5 (float64).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.
"""
from __future__ import annotations

import numpy as np


def expected_tokens(alpha: float, gamma: int) -> float:
    """Equation 1: mean number of tokens one run of Algorithm 1 produces,
    a geometric variable with success probability 1-alpha capped at gamma+1."""
    if alpha == 1.0:
        return float(gamma + 1)
    return (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha)


def capped_geometric_pmf(alpha: float, gamma: int) -> np.ndarray:
    """P(n = k), k = 0..gamma, for i.i.d. acceptance probability alpha
    (section 3.1): k acceptances then a rejection, or all gamma accepted."""
    pmf = np.array([alpha ** k * (1.0 - alpha) for k in range(gamma)] + [alpha ** gamma])
    return pmf


def walltime_improvement(alpha: float, gamma: int, c: float) -> float:
    """Theorem 3.8: expected walltime improvement factor."""
    return expected_tokens(alpha, gamma) / (gamma * c + 1.0)


def ops_increase(alpha: float, gamma: int, c_hat: float) -> float:
    """Theorem 3.11: expected factor of increase in total arithmetic operations."""
    return (gamma * c_hat + gamma + 1.0) / expected_tokens(alpha, gamma)


def min_improvement(alpha: float, c: float) -> float:
    """Corollary 3.9: the gamma = 1 improvement factor (1+alpha)/(1+c)."""
    return (1.0 + alpha) / (1.0 + c)


def optimal_gamma(alpha: float, c: float, gamma_max: int = 64) -> int:
    """Section 3.5: the integer gamma maximising Theorem 3.8 (numeric search)."""
    best, best_g = -np.inf, 1
    for g in range(1, gamma_max + 1):
        v = walltime_improvement(alpha, g, c)
        if v > best:
            best, best_g = v, g
    return best_g


def lenient_alpha(p, q, lenience: float) -> float:
    """Appendix A.5: acceptance rate with lenience l, sum_x min(p(x)/l, q(x))."""
    p = np.asarray(p, np.float64)
    q = np.asarray(q, np.float64)
    return float(np.sum(np.minimum(p / lenience, q)))
