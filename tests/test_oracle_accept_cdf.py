"""Brute force over every value the uniform r can take (all 2^24 of them) for the two
decisions of the oracle's sample path: the accept test and the inverse-CDF draw."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle as O

N = 1 << 24


@pytest.fixture(scope="module")
def all_r():
    return np.arange(N, dtype=np.float64) / N


@pytest.mark.parametrize("p,q", [(0.3, 0.7), (0.7, 0.3), (0.25, 0.25), (1e-9, 0.5), (0.5, 1e-9),
                                 (0.123456789, 0.987654321), (0.0, 0.4), (0.4, 0.0), (0.0, 0.0),
                                 (1.0, 1.0), (3.0e-5, 3.1e-5)])
def test_accept_count_is_min_1_p_over_q(all_r, p, q):
    got = O.accept_count(all_r, p, q)
    # exact count of k in [0, 2^24) with (k / 2^24) * q < p
    fp, fq = Fraction(p), Fraction(q)
    if fq == 0:
        want = N if fp > 0 else 0
    else:
        bound = fp * N / fq                      # k < bound
        want = min(N, int(bound) + (0 if bound == int(bound) else 1)) if bound > 0 else 0
    assert abs(got - want) <= 1
    assert abs(got / N - O.accept_prob(p, q)) <= 2.0 / N
    if p >= q and p > 0:
        assert got == N                           # r < 1 always: p >= q never rejects


def test_accept_single_decisions():
    assert O.accept(0.0, 1e-300, 1.0) == 1
    assert O.accept(0.0, 0.0, 1.0) == 0           # p = 0 is never accepted
    assert O.accept(0.5, 0.1, 0.0) == 1           # q = 0, p > 0
    assert O.accept(0.5, 0.0, 0.0) == 0
    assert O.accept(0.49, 0.5, 1.0) == 1 and O.accept(0.5, 0.5, 1.0) == 0   # strict


def test_accept_margin_hand_values():
    """Distance of r from the accept boundary p/q, in units of r; values worked out by hand."""
    inf = float("inf")
    assert O.accept_margin(0.5, 0.3, 0.5) == pytest.approx(0.1, abs=1e-15)      # |0.5 - 0.6|
    assert O.accept_margin(0.25, 0.5, 1.0) == 0.25                               # |0.25 - 0.5|
    assert O.accept_margin(0.75, 0.25, 0.5) == 0.25                              # |0.75 - 0.5|
    assert O.accept_margin(0.5, 0.25, 0.5) == 0.0                                # on the boundary
    assert O.accept_margin(0.125, 0.75, 0.25) == 2.875                           # p/q = 3: far above any r
    assert O.accept_margin(0.9, 0.2, 0.0) == inf                                 # q = 0: r plays no part
    assert O.accept_margin(0.9, 0.0, 0.0) == 0.0 and O.accept_margin(0.1, 1e-31, 0.0) == 0.0
    # the sign of the gap must not matter, and the unit is r (division by q, not p)
    assert O.accept_margin(0.7, 0.3, 0.5) == pytest.approx(O.accept_margin(0.5, 0.3, 0.5), abs=1e-15)


def test_session_accept_margin_is_the_minimum_over_the_positions_examined():
    """A session's accept_margin covers positions 0..n (the tests Algorithm 2's loop really
    makes) and nothing after the first rejection; recomputed here as |r - p/q| from the random
    words and the per-position scalars."""
    rng = np.random.default_rng(5)
    V, gamma = 50, 6
    seen_reject_before_end = False
    for trial in range(40):
        logits = rng.normal(0, 2, (gamma + 1, V)).astype(np.float32)
        Q = rng.dirichlet(np.ones(V), gamma).astype(np.float32)
        tokens = rng.integers(0, V, gamma).astype(np.int32)
        o = O.verify_batch(logits, O.F32, Q, tokens, V, gamma=gamma, seed=77, step=trial, session_base=3)
        res = o["res"][0]
        n = int(res["n"])
        last = min(n, gamma - 1)
        per_pos = []
        for i in range(last + 1):
            r = O.u01(O.random_block(77, trial, 3, i)[0])
            assert r == o["r_acc"][i]
            per_pos.append(abs(r - o["p_tok"][i] / o["q_tok"][i]))
        assert res["accept_margin"] == pytest.approx(min(per_pos), rel=1e-12, abs=1e-15)
        if n < gamma - 1:
            seen_reject_before_end = True
    assert seen_reject_before_end


WEIGHTS = [
    [0.1, 0.2, 0.3, 0.4],
    [0.0, 0.5, 0.0, 0.25, 0.25, 0.0],
    [0.0, 0.0, 1.0],
    [3.0, 1.0, 0.0, 4.0, 1.0, 5.0, 9.0, 2.0],      # unnormalised
    [1e-12, 1.0, 1e-12],
    [0.7],
]


@pytest.mark.parametrize("w", WEIGHTS)
def test_inverse_cdf_counts_match_weights(all_r, w):
    w = np.array(w, dtype=np.float64)
    tok = O.inverse_cdf_many(w, all_r)
    assert (np.diff(tok) >= 0).all()               # monotone in r
    counts = np.bincount(tok, minlength=w.size)
    assert counts.sum() == N and tok.min() >= 0
    cdf = [Fraction(0)]
    for x in w:
        cdf.append(cdf[-1] + Fraction(float(x)))
    total = cdf[-1]
    for y in range(w.size):
        # k with cdf[y] <= (k/N) * total < cdf[y+1]
        lo = cdf[y] * N / total
        hi = cdf[y + 1] * N / total
        ceil = lambda f: int(f) + (0 if f == int(f) else 1)
        want = ceil(hi) - ceil(lo)
        assert abs(int(counts[y]) - want) <= 1, (y, counts[y], want)
        if w[y] == 0.0:
            assert counts[y] == 0                  # zero-mass tokens are never drawn


def test_inverse_cdf_margin_and_degenerate_input():
    w = np.array([0.25, 0.0, 0.5, 0.25])
    k, margin = O.inverse_cdf(w, 0.5)              # t = 0.5: inside token 2, 0.25 from each end
    assert k == 2 and margin == 0.25
    k, margin = O.inverse_cdf(w, 0.25)             # t on the boundary 0.25: strict > moves on
    assert k == 2 and margin == 0.0
    k, margin = O.inverse_cdf(w, 0.2499)
    assert k == 0 and abs(margin - 0.0001) < 1e-12
    assert O.inverse_cdf(np.zeros(5), 0.3)[0] == -1
    assert O.inverse_cdf(w, 1.0 - 2.0 ** -24)[0] == 3
    assert O.inverse_cdf(w, 0.0)[0] == 0
    assert O.inverse_cdf(np.array([0.0, 0.0, 2.0, 0.0]), 0.0)[0] == 2
