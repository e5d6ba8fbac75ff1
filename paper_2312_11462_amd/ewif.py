"""Expected walltime improvement factors of Section 4, for choosing the K matrix of a cascade.

Host-side arithmetic on scalars (no device work, nothing from the verify path): acceptance rates and cost
coefficients in, expected tokens per target run and walltime factors out, under Section 4's assumption that
token acceptances are independent with a fixed rate.
  phi(alpha, k, x)            Theorem 4.1 (Eq. 1): generating function of the tokens one speculative step yields
  expected_tokens(alpha, k)   phi'(1) = (1 - alpha^(k+1)) / (1 - alpha)
  ewif_sd(alpha, k, c)        corollary of Theorem 4.1: plain speculative decoding
  ewif_vertical(...)          Theorem 4.2: a draft model that is itself drafted for n steps by a smaller one
  ewif_horizontal(...)        Theorem 4.3: a different draft model (rate, cost) per drafted position
  d_ewif_horizontal(...)      its corollary: derivative with respect to one position's acceptance rate
  best_k_sd / best_split_horizontal   small exhaustive searches over the step limits
"""
from __future__ import annotations

from typing import Sequence


def phi(alpha: float, k: int, x: float) -> float:
    """Probability generating function of the number of tokens (1 .. k+1) a speculative step emits,
    1 + (x - 1) (1 - (alpha x)^(k+1)) / (1 - alpha x)  (Theorem 4.1)."""
    ax = alpha * x
    geom = float(k + 1) if abs(1.0 - ax) < 1e-15 else (1.0 - ax ** (k + 1)) / (1.0 - ax)
    return 1.0 + (x - 1.0) * geom


def phi_coefficients(alpha: float, k: int):
    """P(i tokens) for i = 0 .. k+1 (the proof of Theorem 4.1): alpha^(i-1) - alpha^i for 1 <= i <= k, alpha^k for k+1."""
    return [0.0] + [alpha ** (i - 1) - alpha ** i for i in range(1, k + 1)] + [alpha ** k]


def expected_tokens(alpha: float, k: int) -> float:
    return float(k + 1) if abs(1.0 - alpha) < 1e-15 else (1.0 - alpha ** (k + 1)) / (1.0 - alpha)


def ewif_sd(alpha: float, k: int, c: float) -> float:
    """Corollary of Theorem 4.1: tokens per target run over the cost c k + 1 of a step."""
    return expected_tokens(alpha, k) / (c * k + 1.0)


def ewif_vertical(alpha: float, alpha_below: float, k: int, n: int, c_d1: float, c_d2: float) -> float:
    """Theorem 4.2.  alpha: target vs the upper draft model; alpha_below, k: the speculative step between the two
    draft models; n: steps of the upper draft model per target review; c_d1, c_d2: cost coefficients."""
    p = phi(alpha_below, k, alpha) ** n
    tokens = (1.0 - alpha * p) / (1.0 - alpha)
    return tokens / (1.0 + n * c_d1 + n * k * c_d2)


def ewif_horizontal(alphas: Sequence[float], costs: Sequence[float]) -> float:
    """Theorem 4.3: position i is drafted by a model with acceptance rate alphas[i-1] and cost costs[i-1]."""
    if len(alphas) != len(costs):
        raise ValueError("one cost per drafted position")
    num, prod = 1.0, 1.0
    for a in alphas:
        prod *= a
        num += prod
    return num / (1.0 + sum(costs))


def d_ewif_horizontal(alphas: Sequence[float], costs: Sequence[float], l: int) -> float:
    """Corollary of Theorem 4.3: dT / d alpha_l (l counted from 1)."""
    k = len(alphas)
    if not 1 <= l <= k:
        raise ValueError("l out of range")
    s = 0.0
    for i in range(l, k + 1):
        prod = 1.0
        for j in range(1, i + 1):
            if j != l:
                prod *= alphas[j - 1]
        s += prod
    return s / (1.0 + sum(costs))


def best_k_sd(alpha: float, c: float, k_max: int = 64):
    """(k, EWIF) of the best step limit for plain speculative decoding."""
    best = max(range(0, k_max + 1), key=lambda k: ewif_sd(alpha, k, c))
    return best, ewif_sd(alpha, best, c)


def best_split_horizontal(models: Sequence[tuple], k_max: int = 32):
    """models: (alpha, cost) per draft model, in the order of the horizontal cascade (larger model first).
    Returns (counts per model, EWIF) maximising Theorem 4.3 over all splits with at most k_max positions."""
    best_counts, best_val = tuple(0 for _ in models), 1.0

    def rec(i, counts, left):
        nonlocal best_counts, best_val
        if i == len(models):
            al, cs = [], []
            for (a, c), n in zip(models, counts):
                al += [a] * n
                cs += [c] * n
            v = ewif_horizontal(al, cs)
            if v > best_val + 1e-15:
                best_counts, best_val = tuple(counts), v
            return
        for n in range(0, left + 1):
            rec(i + 1, counts + [n], left - n)

    rec(0, [], k_max)
    return best_counts, best_val
