"""Pins for the sampling oracle (oracle/sampling.py): exact hand arithmetic, reductions to
argmax, invariances, a brute-force twin built on a full sort, and the measure of each token's
u-interval against the softmax probabilities.  None re-uses the oracle's own code."""
import math
import os

import numpy as np
import pytest

from oracle import sampling as S

GOLD = os.path.join(os.path.dirname(__file__), "golden", "sampling_worked_example.txt")


def test_worked_example_with_exact_probabilities():
    T = 0.8
    logits = np.array([T * math.log(w) for w in (1.0, 4.0, 0.5, 2.0, 1.0)])
    assert S.top_k_candidates(logits, 3) == [1, 3, 0]          # equal logits: lower index first
    w, total = S.candidate_probabilities(logits, [1, 3, 0], T)
    assert np.allclose(w / total, [4 / 7, 2 / 7, 1 / 7], rtol=0, atol=1e-15)
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 8
    for u, tok in rows:
        for dt in (np.float64, np.float32):
            assert S.sample_top_k(logits, float(u), T, 3, dt) == int(tok), (u, dt)


def test_k_one_and_cold_temperature_reduce_to_argmax():
    rng = np.random.default_rng(5)
    for _ in range(20):
        logits = rng.normal(size=97) * 3
        u = float(rng.random())
        assert S.sample_top_k(logits, u, 0.8, 1) == int(np.argmax(logits))
        assert S.sample_top_k(logits, min(u, 0.999), 1e-4, 10) == int(np.argmax(logits))


def test_shift_invariance_and_k_larger_than_vocabulary():
    rng = np.random.default_rng(6)
    logits = rng.normal(size=40)
    for u in (0.01, 0.33, 0.77, 0.98):
        a = S.sample_top_k(logits, u, 0.8, 10)
        assert S.sample_top_k(logits + 123.0, u, 0.8, 10) == a
    small = np.array([0.3, -1.0, 2.0])
    assert S.top_k_candidates(small, 10) == [2, 0, 1]
    assert S.sample_top_k(small, 0.9999, 0.8, 10) in (0, 1, 2)


def test_ties_are_ordered_by_index_also_at_the_cut():
    logits = np.array([1.0, 5.0, 5.0, 1.0, 1.0, 0.0])
    assert S.top_k_candidates(logits, 2) == [1, 2]
    assert S.top_k_candidates(logits, 4) == [1, 2, 0, 3]       # the cut falls inside a group of equals: lowest indices stay


def _brute_force(logits, u, T, k):
    """Independent twin: stable full sort, library softmax, searchsorted on the cumulative sum."""
    order = np.argsort(-logits, kind="stable")[:k]
    z = logits[order] / T
    p = np.exp(z - z.max())
    p /= p.sum()
    j = int(np.searchsorted(np.cumsum(p), u, side="right"))
    return int(order[min(j, len(order) - 1)])


def test_agrees_with_brute_force_twin():
    rng = np.random.default_rng(7)
    checked = 0
    for trial in range(300):
        n = int(rng.integers(3, 400))
        logits = rng.normal(size=n) * float(rng.uniform(0.2, 6.0))
        u, T, k = float(rng.random()), float(rng.uniform(0.2, 2.0)), int(rng.integers(1, 25))
        if S.decision_margin(logits, u, T, k) < 1e-9:
            continue                                           # u on a boundary: either neighbour is right
        assert S.sample_top_k(logits, u, T, k) == _brute_force(logits, u, T, k)
        checked += 1
    assert checked > 290


def test_u_intervals_have_the_softmax_measure():
    """Sweeping u over a fine grid, the share of draws that return a token equals its probability
    under softmax(logits / T) restricted to the top k (a dropped temperature, a softmax over the
    whole vocabulary or an ascending walk would all fail here)."""
    rng = np.random.default_rng(8)
    logits = rng.normal(size=60) * 2.0
    T, k, n = 0.8, 10, 20000
    counts = {}
    for i in range(n):
        t = S.sample_top_k(logits, (i + 0.5) / n, T, k)
        counts[t] = counts.get(t, 0) + 1
    top = np.argsort(-logits, kind="stable")[:k]
    p = np.exp(logits[top] / T)
    p /= p.sum()
    assert set(counts) <= set(int(t) for t in top)
    for t, pt in zip(top, p):
        assert abs(counts.get(int(t), 0) / n - pt) <= 1.5 / n + 1e-12
    # descending walk: the first interval belongs to the most likely token
    assert S.sample_top_k(logits, 0.0, T, k) == int(top[0])


def test_fp32_decisions_equal_fp64_away_from_boundaries():
    rng = np.random.default_rng(9)
    same = 0
    for _ in range(200):
        logits = (rng.normal(size=500) * 3).astype(np.float32)
        u = float(np.float32(rng.random()))
        if S.decision_margin(logits, u, 0.8, 10) > 1e-5:
            assert S.sample_top_k(logits, u, 0.8, 10, np.float32) == S.sample_top_k(logits, u, 0.8, 10, np.float64)
            same += 1
    assert same > 180


def test_decision_margin_against_a_brute_force_twin_and_by_hand():
    """decision_margin decides which draws the GPU test holds to an exact token.  Twin: sort the softmax
    probabilities of the k largest logits (library sort and softmax), accumulate, and take the distance from u to
    the nearest inner edge.  By hand: probabilities 4/7, 2/7, 1/7 have inner edges 4/7 and 6/7."""
    logits = np.log(np.array([1.0, 4.0, 2.0], dtype=np.float64))            # candidates in order: 1, 2, 0
    for u, want in ((0.5, 4 / 7 - 0.5), (0.6, 0.6 - 4 / 7), (0.8, 6 / 7 - 0.8), (0.0, 4 / 7), (0.99, 0.99 - 6 / 7)):
        assert abs(S.decision_margin(logits, u, 1.0, 3) - want) <= 1e-12
    assert S.decision_margin(logits, 0.3, 1.0, 1) == 1.0                     # one candidate: no edge to cross
    rng = np.random.default_rng(31)
    for _ in range(100):
        V, k, T = int(rng.integers(2, 300)), int(rng.integers(1, 20)), float(rng.uniform(0.2, 2.0))
        lg = (rng.normal(size=V) * 3).astype(np.float64)
        u = float(rng.random())
        order = np.argsort(-lg, kind="stable")[:min(k, V)]
        z = lg[order] / T
        p = np.exp(z - z.max()); p /= p.sum()
        edges = np.cumsum(p)[:-1]
        want = float(np.min(np.abs(edges - u))) if len(edges) else 1.0
        assert abs(S.decision_margin(lg, u, T, k) - want) <= 1e-12
        # what the margin promises: moving u by less than the margin does not change the sampled token
        m = S.decision_margin(lg, u, T, k)
        if m < 1.0 and m > 1e-9:
            for du in (-0.9 * m, 0.9 * m):
                if 0.0 <= u + du < 1.0:
                    assert S.sample_top_k(lg, u + du, T, k) == S.sample_top_k(lg, u, T, k)
