"""Metric definitions of the paper, written out (test infrastructure).

Equation 1 (Section 1): speedup = (1 - alpha^(gamma+1)) / ((1 - alpha)(gamma*c + 1)).
Equation 2 (Section 3.1): acceptance rate = accepted draft tokens / drafted tokens.
Average acceptance length tau (Section 3.1): tokens obtained per target forward
pass; Table 1 satisfies tau = gamma*rate + 1, i.e. tau counts the corrected /
bonus token of each step.
"""
from __future__ import annotations

from typing import Sequence


def acceptance_rate(n_acc: Sequence[int], gamma: int) -> float:
    """Equation 2."""
    return sum(n_acc) / (len(n_acc) * gamma)


def mean_tau(n_acc: Sequence[int]) -> float:
    """Average acceptance length: accepted drafts plus the one token the target adds."""
    return sum(a + 1 for a in n_acc) / len(n_acc)


def alpha_hat(n_acc: Sequence[int], gamma: int) -> float:
    """Per-token acceptance probability (the alpha of Equation 1): accepted over
    examined candidates, where a step that rejects at position k examined k+1."""
    examined = sum(a + 1 if a < gamma else gamma for a in n_acc)
    return sum(n_acc) / examined


def expected_tau(alpha: float, gamma: int) -> float:
    """Numerator of Equation 1: expected tokens per step when each candidate is
    accepted independently with probability alpha."""
    if alpha == 1.0:
        return gamma + 1.0
    return (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha)


def eq1_speedup(alpha: float, gamma: int, c: float) -> float:
    """Equation 1."""
    return expected_tau(alpha, gamma) / (gamma * c + 1.0)


def best_gamma(alpha: float, c: float, gamma_max: int) -> int:
    """The candidate count in [0, gamma_max] with the largest Equation 1 value (the smallest
    such count on ties), by trying every one."""
    values = [eq1_speedup(alpha, g, c) for g in range(gamma_max + 1)]
    return values.index(max(values))
