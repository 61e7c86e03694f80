"""Pins for the span-posterior / MBR-decoding oracle."""
import itertools
import math

import numpy as np
import pytest

from oracle import decode_oracle as D
from test_oracle_pins import bracketings, random_grammar


def spans_of(tree, i0=0):
    """(width >= 2 spans, end) of a nested-tuple bracketing whose first leaf is i0."""
    if isinstance(tree, int):
        return [], tree + 1
    ls, mid = spans_of(tree[0], i0)
    rs, end = spans_of(tree[1], mid)
    return [(i0, end)] + ls + rs, end


def posterior_by_enumeration(log_root, L, R, e):
    """Span posteriors from the definition: total weight of the labelled trees that contain the span, over Z."""
    n, P = e.shape
    N = L.shape[0]
    root, emit = np.exp(log_root), np.exp(e)
    mu = np.zeros((n + 1, n + 1))
    Z = 0.0
    for tree in bracketings(0, n):
        nodes = []

        def walk(t):
            if isinstance(t, int):
                return ("l", t)
            me = len(nodes)
            nodes.append(None)
            nodes[me] = (walk(t[0]), walk(t[1]))
            return ("n", me)

        walk(tree)
        wsum = 0.0
        for nt in itertools.product(range(N), repeat=len(nodes)):
            for pt in itertools.product(range(P), repeat=n):
                w = root[nt[0]]
                for idx, (lc, rc) in enumerate(nodes):
                    ls = nt[lc[1]] if lc[0] == "n" else N + pt[lc[1]]
                    rs = nt[rc[1]] if rc[0] == "n" else N + pt[rc[1]]
                    w *= L[nt[idx], ls] * R[nt[idx], rs]
                for i in range(n):
                    w *= emit[i, pt[i]]
                wsum += w
        Z += wsum
        for (i, j) in spans_of(tree)[0]:
            mu[i, j] += wsum
    return mu / Z


@pytest.mark.parametrize("N,P,n", [(2, 2, 4), (2, 3, 5), (3, 2, 4)])
def test_span_posteriors_match_enumeration(N, P, n):
    rng = np.random.default_rng(7 * N + P + n)
    lr, L, R, e = random_grammar(rng, N, P, n, scale=2.0)
    mu, lab = D.span_posteriors(lr, L, R, e)
    ref = posterior_by_enumeration(lr, L, R, e)
    for i in range(n):
        for j in range(i + 2, n + 1):
            assert mu[i, j] == pytest.approx(ref[i, j], rel=1e-10, abs=1e-14)
    assert mu[0, n] == pytest.approx(1.0, rel=1e-12)
    assert sum(mu[i, j] for i in range(n) for j in range(i + 2, n + 1)) == pytest.approx(n - 1, rel=1e-12)


@pytest.mark.parametrize("n,seed", [(2, 0), (3, 1), (5, 2), (7, 3), (8, 4)])
def test_mbr_tree_is_the_best_bracketing(n, seed):
    rng = np.random.default_rng(seed)
    mu = np.triu(rng.random((n + 1, n + 1)), 2)
    score, spans = D.mbr_decode(mu, n)
    assert D.is_binary_tree(spans, n)
    assert score == pytest.approx(D.tree_score(mu, spans), rel=1e-12)
    best = max(D.tree_score(mu, spans_of(t)[0]) for t in bracketings(0, n))
    assert score == pytest.approx(best, rel=1e-12)
    n_trees = sum(1 for _ in bracketings(0, n))
    assert n_trees == math.comb(2 * (n - 1), n - 1) // n


def test_decode_recovers_a_planted_tree_and_breaks_ties_to_the_left():
    n = 6
    planted = [(0, 6), (0, 2), (2, 6), (3, 6), (3, 5)]
    mu = np.zeros((n + 1, n + 1))
    for (i, j) in planted:
        mu[i, j] = 1.0
    score, spans = D.mbr_decode(mu, n)
    assert sorted(spans) == sorted(planted) and score == 5.0
    # all-equal posteriors: every tree ties, the smallest split point wins everywhere -> right-branching tree
    score, spans = D.mbr_decode(np.triu(np.ones((n + 1, n + 1)), 2), n)
    assert spans == [(0, 6), (1, 6), (2, 6), (3, 6), (4, 6)]
    assert not D.is_binary_tree([(0, 6), (0, 3), (2, 6), (0, 2), (3, 6)], n)  # crossing spans
