"""Pins for the oracle's temperature / nucleus sampler (Sec. V-A "Models": Step-Audio-2 decodes with
temperature 0.7 and top_p 0.9): a hand-worked distribution, limits that reduce to the arg-max,
exact interval counts against the softmax, and an independent numpy formulation."""
import numpy as np
import pytest

from oracle import binding as ob

TWO64 = 1 << 64


def omega(u: float) -> int:
    return min(TWO64 - 1, int(u * TWO64))


def test_hand_worked_distribution():
    # weights 1, 1/2, 1/4, 1/8, 1/8 (total 2): cumulative shares 0.5, 0.75, 0.875, 0.9375, 1
    logits = np.log(np.array([1.0, 0.5, 0.25, 0.125, 0.125])) + 3.0
    # top_p 0.8 -> nucleus {0, 1, 2} with mass 1.75: token 0 below 1/1.75, 1 below 1.5/1.75, else 2
    for u, want in [(0.0, 0), (0.5, 0), (0.571, 0), (0.572, 1), (0.857, 1), (0.858, 2), (0.999999, 2)]:
        tok, n, gap = ob.sample(logits, 1.0, 0.8, omega(u))
        assert (tok, n) == (want, 3), (u, tok, n)
    # equal weights: the lower index enters the nucleus first
    assert ob.sample(logits, 1.0, 0.9, omega(0.99))[:2] == (3, 4)      # {0,1,2,3}, last one drawn
    assert ob.sample(logits, 1.0, 0.95, omega(0.9999))[:2] == (4, 5)   # all five
    # permuting the entries permutes the answer
    perm = np.array([4, 2, 0, 3, 1])
    for u in (0.1, 0.6, 0.9):
        tok, _, _ = ob.sample(logits, 1.0, 0.8, omega(u))
        tok_p, _, _ = ob.sample(logits[perm], 1.0, 0.8, omega(u))
        assert perm[tok_p] == tok


def test_limits_reduce_to_argmax():
    rng = np.random.default_rng(0)
    for _ in range(20):
        logits = rng.normal(0, 3, size=500)
        best = int(np.argmax(logits))
        for u in (0.0, 0.3, 0.999):
            assert ob.sample(logits, 0.01, 0.9, omega(u))[0] == best      # temperature -> 0
            assert ob.sample(logits, 1.0, 1e-9, omega(u))[:2] == (best, 1)  # top_p -> 0: one element


def test_interval_counts_match_the_softmax():
    """top_p = 1: the draw is the inverse CDF of softmax(l / T) in the sampler's order, so a regular
    grid of N random words must hit token i round(p_i N) times, give or take one grid point"""
    rng = np.random.default_rng(1)
    logits = rng.normal(0, 2, size=40)
    for T in (1.0, 0.7):
        p = np.exp((logits - logits.max()) / T)
        p /= p.sum()
        N = 20000
        counts = np.zeros(40, dtype=int)
        for k in range(N):
            counts[ob.sample(logits, T, 1.0, omega((k + 0.5) / N))[0]] += 1
        assert np.all(np.abs(counts - p * N) <= 1.0 + 1e-6 * N)


def numpy_nucleus(logits, T, top_p, u):
    """the textbook formulation in float64: sort by probability, cut the cumulative sum at top_p,
    renormalise, invert the CDF"""
    p = np.exp((logits - logits.max()) / T)
    order = np.lexsort((np.arange(len(p)), -p))     # larger p first, lower index first
    cum = np.cumsum(p[order])
    cut = int(np.searchsorted(cum, top_p * cum[-1], side="left"))
    x = u * cum[cut]
    return int(order[int(np.searchsorted(cum[:cut + 1], x, side="right"))]), cut + 1


@pytest.mark.parametrize("T,top_p", [(0.7, 0.9), (1.0, 0.5), (1.3, 0.99), (0.7, 1.0)])
def test_against_numpy_formulation(T, top_p):
    rng = np.random.default_rng(2)
    agree = 0
    for trial in range(200):
        logits = rng.normal(0, 2.5, size=3000).astype(np.float32).astype(np.float64)
        u = float(rng.random())
        tok, n, gap = ob.sample(logits, T, top_p, omega(u))
        want_tok, want_n = numpy_nucleus(logits, T, top_p, u)
        if gap < 1e-7:        # a draw on an edge: the two roundings may part
            continue
        assert tok == want_tok, (trial, tok, want_tok, gap)
        # (entries whose weight is below 2^-33 of the largest carry no integer mass: with
        # top_p = 1 the oracle's nucleus ends where the mass is complete, numpy's at the last entry)
        assert n == want_n or (top_p == 1.0 and n <= want_n), (trial, n, want_n)
        agree += 1
    assert agree > 190


def test_monotone_in_the_random_word():
    rng = np.random.default_rng(3)
    logits = rng.normal(0, 2, size=200)
    p = np.exp(logits - logits.max())
    rank = np.empty(200, dtype=int)
    rank[np.lexsort((np.arange(200), -p))] = np.arange(200)
    last = -1
    for k in range(400):
        tok = ob.sample(logits, 0.7, 0.9, omega(k / 400))[0]
        assert rank[tok] >= last
        last = rank[tok]


def test_refusals():
    logits = np.zeros(8)
    assert ob.sample(logits, 0.0, 0.9, 1)[0] == -1
    assert ob.sample(logits, 1.0, 0.0, 1)[0] == -1
    assert ob.sample(logits, 1.0, 1.5, 1)[0] == -1
    bad = logits.copy(); bad[3] = np.nan
    assert ob.sample(bad, 1.0, 0.9, 1)[0] == -1
