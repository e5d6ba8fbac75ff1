"""Pins of the Section 4 calculators (CPU only): the generating function against the distribution the proof
of Theorem 4.1 writes out, against brute-force enumeration and against the oracle's own accept routine run
on i.i.d. acceptances; Theorem 4.2 against a direct simulation of the two-level process; Theorem 4.3 against
enumeration; the corollaries by finite differences and inequalities."""
import itertools

import numpy as np
import pytest

from oracle import csd_oracle as O
from paper_2312_11462_amd import ewif as E


@pytest.mark.parametrize("alpha,k", [(0.3, 1), (0.62, 4), (0.8, 9), (0.95, 3)])
def test_phi_is_the_generating_function_of_the_written_distribution(alpha, k):
    p = E.phi_coefficients(alpha, k)
    assert abs(sum(p) - 1.0) < 1e-12
    for x in (0.0, 0.37, 1.0, 1.3):
        assert abs(E.phi(alpha, k, x) - sum(pi * x ** i for i, pi in enumerate(p))) < 1e-12
    mean = sum(i * pi for i, pi in enumerate(p))
    assert abs(E.expected_tokens(alpha, k) - mean) < 1e-12
    h = 1e-6
    assert abs((E.phi(alpha, k, 1 + h) - E.phi(alpha, k, 1 - h)) / (2 * h) - mean) < 1e-6


def test_length_law_against_the_accept_routine_with_iid_acceptances():
    """One-hot drafts accepted with probability p(x) = alpha at every position: the accepted-length law of the
    oracle's accept routine is the one Theorem 4.1's proof writes out."""
    alpha, k, V, n = 0.6, 4, 4, 60000
    p = np.zeros((n, k + 1, V), np.float32)
    p[:, :, 0] = alpha
    p[:, :, 1] = 1.0 - alpha
    rng = np.random.default_rng(11)
    u = (rng.integers(0, 1 << 24, size=(n, k)).astype(np.float32) / np.float32(1 << 24))
    us = (rng.integers(0, 1 << 24, size=n).astype(np.float32) / np.float32(1 << 24))
    n_acc, _ = O.accept(p, None, np.zeros((n, k), np.int32), u, us)
    hist = np.bincount(n_acc + 1, minlength=k + 2) / n
    want = np.array(E.phi_coefficients(alpha, k))
    assert np.abs(hist - want).max() < 4 * np.sqrt(0.25 / n) + 1e-3
    assert abs((n_acc + 1).mean() - E.expected_tokens(alpha, k)) < 0.02


def test_sd_corollary_and_best_k():
    assert abs(E.ewif_sd(0.8, 5, 0.1) - (1 - 0.8 ** 6) / (0.2 * 1.5)) < 1e-12
    k, v = E.best_k_sd(0.8, 0.05, 40)
    assert all(E.ewif_sd(0.8, kk, 0.05) <= v + 1e-12 for kk in range(41))
    assert E.best_k_sd(0.5, 1.0, 10)[0] == 0            # a draft as costly as the target never pays


def _simulate_vertical(alpha, alpha_below, k, n, rng, trials):
    tot = 0
    for _ in range(trials):
        drafted = 0
        for _ in range(n):                               # n steps of the upper draft model, each keeps 1 .. k+1 tokens
            a = 0
            while a < k and rng.random() < alpha_below:
                a += 1
            drafted += a + 1
        kept = 0
        while kept < drafted and rng.random() < alpha:   # the target keeps a prefix and adds one token
            kept += 1
        tot += kept + 1
    return tot / trials


def test_vertical_cascade_theorem_against_simulation():
    rng = np.random.default_rng(5)
    alpha, ab, k, n = 0.7, 0.5, 3, 2
    sim = _simulate_vertical(alpha, ab, k, n, rng, 200000)
    tokens = E.ewif_vertical(alpha, ab, k, n, 0.0, 0.0)           # zero costs: the numerator alone
    assert abs(sim - tokens) < 0.02
    assert abs(E.ewif_vertical(alpha, ab, k, n, 0.1, 0.01) - tokens / (1 + n * 0.1 + n * k * 0.01)) < 1e-12
    # corollary: phi_(alpha', k)(alpha) < alpha, so a free lower model always helps
    for a, a2, kk in itertools.product((0.2, 0.6, 0.9), (0.1, 0.5, 0.95), (1, 4, 12)):
        assert E.phi(a2, kk, a) < a
        assert E.ewif_vertical(a, a2, kk, 3, 0.1, 0.0) > E.ewif_sd(a, 3, 0.1)


def test_horizontal_cascade_theorem_by_enumeration_and_its_derivative():
    alphas, costs = [0.9, 0.8, 0.5, 0.4], [0.1, 0.1, 0.01, 0.01]
    exp = 0.0
    for outcome in itertools.product((0, 1), repeat=4):
        pr, kept = 1.0, 0
        for a, o in zip(alphas, outcome):
            pr *= a if o else 1 - a
        for o in outcome:
            if not o:
                break
            kept += 1
        exp += pr * (kept + 1)
    assert abs(E.ewif_horizontal(alphas, costs) - exp / (1 + sum(costs))) < 1e-12
    assert abs(E.ewif_horizontal([0.7] * 5, [0.03] * 5) - E.ewif_sd(0.7, 5, 0.03)) < 1e-12   # one model: Theorem 4.1
    for l in range(1, 5):
        h = 1e-6
        up = list(alphas); up[l - 1] += h
        dn = list(alphas); dn[l - 1] -= h
        fd = (E.ewif_horizontal(up, costs) - E.ewif_horizontal(dn, costs)) / (2 * h)
        assert abs(E.d_ewif_horizontal(alphas, costs, l) - fd) < 1e-6
    # earlier positions matter more when rates are equal (the paper's reading of the corollary)
    eq = [0.7] * 4
    d = [E.d_ewif_horizontal(eq, costs, l) for l in range(1, 5)]
    assert d[0] > d[1] > d[2] > d[3]


def test_best_split_prefers_the_better_model_first_and_the_cheap_one_last():
    counts, val = E.best_split_horizontal([(0.8, 0.1), (0.5, 0.005)], k_max=12)
    assert sum(counts) <= 12 and counts[0] >= 1 and counts[1] >= 1
    assert val >= E.best_k_sd(0.8, 0.1, 12)[1] - 1e-12 and val >= E.best_k_sd(0.5, 0.005, 12)[1] - 1e-12
