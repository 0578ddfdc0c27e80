"""Pins for the oracle's per-node selection (the paper's Weighted Reservoir Sampling listing, its
second algorithm) and its sampling law."""
import heapq
import itertools
import random
from decimal import Decimal, getcontext

import numpy as np
import pytest
from scipy import stats

import oracle

getcontext().prec = 60
Q = 65536


def _one_pass_reservoir(stream, m):
    """What a reservoir computes, by a library routine: heapq.nsmallest reads the stream once and
    keeps at most m items in a heap, evicting its worst when a better one arrives.  Items are
    (K, x, slot); 'better' is the oracle's total order (K ascending, x descending, slot ascending)."""
    kept = heapq.nsmallest(m, iter(stream), key=lambda item: (item[0], -item[1], item[2]))
    return sorted(s for _, _, s in kept)


def test_top_m_equals_a_one_pass_reservoir_in_any_arrival_order():
    """The oracle sorts all keys and keeps m; the method is a reservoir that sees each neighbour
    once (Weighted Reservoir Sampling listing, Sec. III-A: O(|N(v)|) time, O(m) space).  Both must
    choose the same slots, and a reservoir's choice must not depend on the order of arrival."""
    rnd = random.Random(10)
    for trial in range(400):
        deg = rnd.randrange(2, 200)
        m = rnd.randrange(1, deg)
        seed, node, hop = rnd.getrandbits(64), rnd.getrandbits(33), rnd.randrange(4)
        w = [rnd.choice([Q, 3 * Q]) for _ in range(deg)]
        items = []
        for s in range(deg):
            x = oracle.draw(seed, hop, node, s)
            items.append((oracle.key(x, w[s]), x, s))
        want = oracle.select(seed, hop, node, deg, m, w)
        assert want == _one_pass_reservoir(items, m)
        shuffled = items[:]
        rnd.shuffle(shuffled)
        assert want == _one_pass_reservoir(shuffled, m)


def test_selection_equals_top_m_of_real_keys():
    """The m largest k = u^(1/w) in exact (60-digit) arithmetic are the slots the oracle takes."""
    rnd = random.Random(11)
    for trial in range(150):
        deg = rnd.randrange(5, 80)
        m = rnd.randrange(1, min(deg, 12))
        seed, node, hop = rnd.getrandbits(64), rnd.getrandbits(20), rnd.randrange(3)
        gamma = rnd.choice([1, 2, 4, 8, 1.5])
        w = [int(gamma * Q) if rnd.random() < 0.4 else Q for _ in range(deg)]
        real = []
        for s in range(deg):
            u = Decimal(oracle.draw(seed, hop, node, s) + 1) / Decimal(1 << 32)
            k = (u.ln() * Decimal(Q) / Decimal(w[s])).exp()     # u^(1/w)
            real.append((k, s))
        real.sort(reverse=True)
        # require a visible gap between the m-th and (m+1)-th real key, so fixed-point
        # rounding (2^-29 in log2) cannot decide the case
        if (real[m - 1][0] - real[m][0]) < Decimal(10) ** -7:
            continue
        assert oracle.select(seed, hop, node, deg, m, w) == sorted(s for _, s in real[:m])


def test_degree_at_most_fanout_takes_all_and_zero_degree():
    assert oracle.select(1, 0, 7, 0, 5) == []
    assert oracle.select(1, 0, 7, 3, 5) == [0, 1, 2]
    assert oracle.select(1, 0, 7, 5, 5) == [0, 1, 2, 3, 4]
    got = oracle.select(1, 0, 7, 6, 5)
    assert len(got) == 5 and got == sorted(set(got)) and all(0 <= s < 6 for s in got)


def test_equal_weights_reduce_to_largest_draws():
    """gamma = 1, everything cached or nothing cached: uniform sampling (Sec. III-A), and the
    chosen slots are those with the largest draws x, ties to the smaller slot."""
    rnd = random.Random(12)
    for _ in range(200):
        deg = rnd.randrange(2, 300)
        m = rnd.randrange(1, deg)
        seed, node, hop = rnd.getrandbits(64), rnd.getrandbits(30), rnd.randrange(3)
        xs = [(-oracle.draw(seed, hop, node, s), s) for s in range(deg)]
        expect = sorted(s for _, s in sorted(xs)[:m])
        assert oracle.select(seed, hop, node, deg, m, None) == expect
        assert oracle.select(seed, hop, node, deg, m, [5 * Q] * deg) == expect


def test_uniform_inclusion_chi_square():
    """Equal weights: every slot is included with probability m/d.  With without-replacement
    covariance, X2 = (d-1)/(d T p (1-p)) * sum (O_j - T p)^2 is chi-square with d-1 dof."""
    for d, m, T in [(7, 3, 6000), (40, 10, 6000), (100, 25, 3000)]:
        counts = np.zeros(d)
        for t in range(T):
            for s in oracle.select(99, 1, 1000 + t, d, m):
                counts[s] += 1
        p = m / d
        X2 = (d - 1) / (d * T * p * (1 - p)) * np.sum((counts - T * p) ** 2)
        assert stats.chi2.sf(X2, d - 1) > 1e-4, (d, m, X2)


def test_weighted_single_draw_law():
    """m = 1: P(slot j) = w_j / sum w (the A-Res property behind Alg. 2)."""
    w = np.array([1, 4, 1, 1, 4, 2.5, 1, 1], dtype=float)
    wq = [int(v * Q) for v in w]
    T = 20000
    counts = np.zeros(len(w))
    for t in range(T):
        (s,) = oracle.select(5, 0, t, len(w), 1, wq)
        counts[s] += 1
    chi = stats.chisquare(counts, T * w / w.sum())
    assert chi.pvalue > 1e-4, (counts, chi)


def test_weighted_subsets_match_successive_draws_brute_force():
    """m > 1: the subset law equals m successive weighted draws without replacement."""
    w = [1.0, 4.0, 1.0, 4.0, 1.0, 2.0]
    d, m = len(w), 3
    prob = {}
    for perm in itertools.permutations(range(d), m):
        p, rest = 1.0, sum(w)
        for j in perm:
            p *= w[j] / rest
            rest -= w[j]
        key = tuple(sorted(perm))
        prob[key] = prob.get(key, 0.0) + p
    assert abs(sum(prob.values()) - 1) < 1e-12
    wq = [int(v * Q) for v in w]
    T = 30000
    obs = {k: 0 for k in prob}
    for t in range(T):
        obs[tuple(oracle.select(17, 2, 10 ** 6 + t, d, m, wq))] += 1
    keys = sorted(prob)
    chi = stats.chisquare([obs[k] for k in keys], [T * prob[k] for k in keys])
    assert chi.pvalue > 1e-4, chi


def test_draws_depend_on_every_key_component():
    base = oracle.select(1, 0, 50, 64, 8)
    assert base == oracle.select(1, 0, 50, 64, 8)
    assert base != oracle.select(2, 0, 50, 64, 8)
    assert base != oracle.select(1, 1, 50, 64, 8)
    assert base != oracle.select(1, 0, 51, 64, 8)
    assert base != oracle.select(1 << 32 | 1, 0, 50, 64, 8)      # high half of the seed
    assert base != oracle.select(1, 0, 50 | (1 << 32), 64, 8)    # high half of the node id
