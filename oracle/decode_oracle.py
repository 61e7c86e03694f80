"""CPU oracle for span posteriors and minimum-Bayes-risk tree decoding.  TEST INFRASTRUCTURE ONLY.

The paper evaluates its grammars as unsupervised parsers (sentence-level F1, Sec. 4 "Evaluation"), which needs
a tree per sentence.  The tree used here is the one that maximises the expected number of correct spans under
the posterior: with mu(i,j) = sum_A P(A spans (i,j) | sentence) (the span marginals that the reverse pass of the
inside algorithm yields, Sec. 3.2 "Recomputation" / inside-outside by back-propagation),

    best(i, i+1) = 0,     best(i, j) = mu(i, j) + max_{i<k<j} ( best(i, k) + best(k, j) ),

and the tree is read off the arg-max split points (smallest k on ties).  Width-1 spans are in every tree and
are left out of the score.  Plain Python / numpy, double precision; shares no code with the HIP path.
Pinned in tests/test_decode_oracle.py (enumeration of all bracketings; span posteriors by enumeration of all
labelled trees).
"""
from __future__ import annotations

import numpy as np

from . import spcfg_oracle as O


def span_posteriors(log_root, L, R, e):
    """mu[i, j] for 0 <= i < j <= n (width >= 2 from the reverse pass; width 1 is 1), and the arg-max label."""
    n = e.shape[0]
    out = O.inside_backward_sentence(log_root, L, R, e, 1.0, return_marginals=True)
    obar = out[-1]
    mu = np.zeros((n + 1, n + 1))
    lab = np.full((n + 1, n + 1), -1, dtype=np.int64)
    for i in range(n):
        mu[i, i + 1] = 1.0
    for (i, j), v in obar.items():
        mu[i, j] = v.sum()
        lab[i, j] = int(np.argmax(v))
    return mu, lab


def mbr_decode(mu, n):
    """Returns (score, spans): the width >= 2 spans of the best tree in pre-order, and sum of their mu."""
    best = np.zeros((n + 1, n + 1))
    split = np.zeros((n + 1, n + 1), dtype=np.int64)
    for w in range(2, n + 1):
        for i in range(n - w + 1):
            j = i + w
            cand = [best[i, k] + best[k, j] for k in range(i + 1, j)]
            kk = int(np.argmax(cand))  # first maximum = smallest k
            best[i, j] = mu[i, j] + cand[kk]
            split[i, j] = i + 1 + kk
    spans = []

    def walk(i, j):
        if j - i < 2:
            return
        spans.append((i, j))
        walk(i, split[i, j])
        walk(split[i, j], j)

    walk(0, n)
    return float(best[0, n]), spans


def tree_score(mu, spans):
    return float(sum(mu[i, j] for (i, j) in spans))


def is_binary_tree(spans, n):
    """True iff `spans` are exactly the n-1 internal nodes of one binary bracketing of (0, n)."""
    s = set(spans)
    if len(s) != n - 1 or len(spans) != n - 1 or (n >= 2 and (0, n) not in s):
        return False

    def ok(i, j):
        if j - i == 1:
            return True
        if (i, j) not in s:
            return False
        ks = [k for k in range(i + 1, j) if (k - i == 1 or (i, k) in s) and (j - k == 1 or (k, j) in s)]
        return any(ok(i, k) and ok(k, j) for k in ks)

    return ok(0, n)
