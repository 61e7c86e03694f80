"""CPU oracle for the simple-PCFG inside pass and its gradients.  TEST INFRASTRUCTURE ONLY.

A plain, slow, double-precision log-space CKY written from the paper's definitions.  It shares no
code with the HIP path and nothing in the product path may import it; only the tests, the smoke
check and the benchmark's cpu_baseline leg call it.

What it computes (paper Sec. 2 and Sec. 3.1, fencepost spans 0 <= i < j <= n):

  width 1:        a_{i,i+1}[A] = log sum_T L[A, N+T] * exp(e_i[T]),   b_{i,i+1}[A] likewise with R
  width w >= 2:   o_ij[A] = log sum_{i<k<j} exp(a_ik[A] + b_kj[A])          (Eq. 1, the eta/zeta recursion)
  non-root span:  a_ij = x + log(L_N exp(o_ij - x)),  b_ij likewise with R_N,  x = max_A o_ij[A]
                                                                 (the log-einsum-exp identity, Sec. 3.2)
  log Z = log sum_A exp(log_root[A] + o_0n[A])                   (rule S -> A)

e_i[T] = log pi(T -> w_i) is given per token.  L, R are [N, N+P] in probability space, nonterminal
children in columns [0, N), preterminal children in columns [N, N+P).  Parents are nonterminals only, so
spans of width 1 carry preterminal vectors and wider spans nonterminal vectors.

The gradients are the exact partial derivatives of sum_b g_b * log Z_b (Sec. 3.2 "Recomputation" gives
d o_ij / d a_ik = exp(a_ik + b_kj - o_ij); the rest is the chain rule through the projection identity).
With g = 1:  grad_log_root[A] is the posterior of A at the root, grad_log_emit[b, i, T] the posterior of
preterminal T over token i, and L * grad_L, R * grad_R are expected rule counts.

Pinned (tests/test_oracle_pins.py) by brute-force enumeration of all labelled binary trees, by a dense
inside pass over the materialised rule tensor T[A,B,C] = L[A,B] R[A,C], by closed forms, by symmetries,
by enumeration-based expected counts, by central finite differences and by gradient invariants.
The paper prints no worked numerical example, so nothing here is pinned to a printed value.
"""
from __future__ import annotations

import numpy as np

_NEG_INF = -np.inf


def _log_project(W, o):
    """x + log(W @ exp(o - x)) for every row of o;  W: [N, K], o: [S, K]  ->  [S, N].   (log-einsum-exp)"""
    x = o.max(axis=1, keepdims=True)
    x = np.where(np.isfinite(x), x, 0.0)  # an all -inf vector projects to -inf
    with np.errstate(divide="ignore"):
        return x + np.log(np.exp(o - x) @ W.T)


def _logsumexp0(t):
    """log sum_k exp(t[k]) along axis 0 with the per-element maximum x* of Eq. 1 as the shift."""
    xs = t.max(axis=0)
    xs_safe = np.where(np.isfinite(xs), xs, 0.0)
    with np.errstate(divide="ignore"):
        return xs_safe + np.log(np.exp(t - xs_safe).sum(axis=0))


def inside_sentence(log_root, L, R, e):
    """Inside pass for one sentence.  e: [n, P] log emissions.  Returns (logZ, a, b, o).

    a, b, o are dicts keyed by the span (i, j); a/b exist for every non-root span, o for width >= 2.
    """
    log_root = np.asarray(log_root, dtype=np.float64)
    L = np.asarray(L, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    e = np.asarray(e, dtype=np.float64)
    n, P = e.shape
    N = L.shape[0]
    assert L.shape == (N, N + P) and R.shape == (N, N + P) and log_root.shape == (N,)
    if n < 2:
        raise ValueError("the root rule S -> A needs a nonterminal over the sentence: n >= 2")
    L_N, L_P, R_N, R_P = L[:, :N], L[:, N:], R[:, :N], R[:, N:]
    a, b, o = {}, {}, {}
    # base case: the children of a width-1 span are preterminals
    a1 = _log_project(L_P, e)
    b1 = _log_project(R_P, e)
    for i in range(n):
        a[(i, i + 1)] = a1[i]
        b[(i, i + 1)] = b1[i]
    for w in range(2, n + 1):
        spans = [(i, i + w) for i in range(n - w + 1)]
        for (i, j) in spans:
            terms = np.stack([a[(i, k)] + b[(k, j)] for k in range(i + 1, j)])
            o[(i, j)] = _logsumexp0(terms)
        if w < n:  # the root span is never a child, so it is not projected
            ow = np.stack([o[s] for s in spans])
            aw = _log_project(L_N, ow)
            bw = _log_project(R_N, ow)
            for r, s in enumerate(spans):
                a[s] = aw[r]
                b[s] = bw[r]
    logZ = _logsumexp0((log_root + o[(0, n)])[:, None])[0]
    return float(logZ), a, b, o


def inside(log_root, L, R, log_emit, lengths):
    """log Z per sentence (float64 [B]).  log_emit: [B, n_max, P]; positions >= lengths[b] are ignored."""
    lengths = np.asarray(lengths)
    out = np.empty(len(lengths), dtype=np.float64)
    for bi, n in enumerate(lengths):
        out[bi] = inside_sentence(log_root, L, R, np.asarray(log_emit)[bi, : int(n)])[0]
    return out


def _safe_exp_diff(x, y):
    """exp(x - y) with the convention exp(-inf - (-inf)) = 0 (a zero-probability item carries no mass)."""
    with np.errstate(invalid="ignore"):
        d = x - y
    return np.exp(np.where(np.isnan(d), _NEG_INF, d))


def _ratio(adj, x, logv):
    """adj * exp(x - logv), i.e. adj / (W p) since logv = x + log(W p); 0 where the adjoint is 0."""
    with np.errstate(over="ignore", invalid="ignore"):
        r = adj * _safe_exp_diff(x, logv)
    return np.where(adj == 0.0, 0.0, r)


def inside_backward_sentence(log_root, L, R, e, g=1.0, return_marginals=False):
    """Forward + reverse pass for one sentence.

    Returns (logZ, grad_L, grad_R, grad_log_root, grad_log_emit) for g * log Z, all float64; with
    return_marginals also the dict of span posteriors obar[(i, j)] (width >= 2).  A sentence with Z = 0
    contributes zero gradients.
    """
    log_root = np.asarray(log_root, dtype=np.float64)
    L = np.asarray(L, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    e = np.asarray(e, dtype=np.float64)
    n, P = e.shape
    N = L.shape[0]
    logZ, a, b, o = inside_sentence(log_root, L, R, e)
    gL = np.zeros_like(L)
    gR = np.zeros_like(R)
    g_root = np.zeros(N)
    g_emit = np.zeros((n, P))
    obar = {}
    if not np.isfinite(logZ):
        return (logZ, gL, gR, g_root, g_emit) + ((obar,) if return_marginals else ())
    L_N, L_P, R_N, R_P = L[:, :N], L[:, N:], R[:, :N], R[:, N:]
    abar = {s: np.zeros(N) for s in a}
    bbar = {s: np.zeros(N) for s in b}

    # root rule: d logZ / d o_0n[A] = exp(log_root[A] + o_0n[A] - logZ)
    obar[(0, n)] = g * _safe_exp_diff(log_root + o[(0, n)], logZ)
    g_root += obar[(0, n)]

    for w in range(n, 1, -1):  # every parent of a span is wider, so its adjoint is final here
        spans = [(i, i + w) for i in range(n - w + 1)]
        if w < n:
            # all spans of this width at once (rows = spans):
            # a = x + log(L_N p), p = exp(o - x):  d a[A] / d L[A,B] = p[B] / (L_N p)[A],
            #                                    d a[A] / d o[B]   = L[A,B] p[B] / (L_N p)[A]
            ow = np.stack([o[s] for s in spans])
            x = ow.max(axis=1, keepdims=True)
            x = np.where(np.isfinite(x), x, 0.0)
            p = np.exp(ow - x)
            ab = np.stack([abar[s] for s in spans])
            bb = np.stack([bbar[s] for s in spans])
            u = _ratio(ab, x, np.stack([a[s] for s in spans]))  # abar / (L_N p)
            v = _ratio(bb, x, np.stack([b[s] for s in spans]))
            gL[:, :N] += u.T @ p
            gR[:, :N] += v.T @ p
            ob = p * (u @ L_N + v @ R_N)
            for r, s in enumerate(spans):
                obar[s] = ob[r]
        # Eq. 1 backward: d o_ij / d a_ik = d o_ij / d b_kj = exp(a_ik + b_kj - o_ij)
        for (i, j) in spans:
            for k in range(i + 1, j):
                gamma = obar[(i, j)] * _safe_exp_diff(a[(i, k)] + b[(k, j)], o[(i, j)])
                abar[(i, k)] += gamma
                bbar[(k, j)] += gamma
    # width 1: same projection backward with the preterminal blocks; eps = exp(e - x)
    leaves = [(i, i + 1) for i in range(n)]
    x = e.max(axis=1, keepdims=True)
    eps = np.exp(e - x)
    ab = np.stack([abar[s] for s in leaves])
    bb = np.stack([bbar[s] for s in leaves])
    u = _ratio(ab, x, np.stack([a[s] for s in leaves]))
    v = _ratio(bb, x, np.stack([b[s] for s in leaves]))
    gL[:, N:] += u.T @ eps
    gR[:, N:] += v.T @ eps
    g_emit[:] = eps * (u @ L_P + v @ R_P)
    out = (logZ, gL, gR, g_root, g_emit)
    return out + ((obar,) if return_marginals else ())


def inside_backward(log_root, L, R, log_emit, lengths, grad_logZ=None):
    """Batched forward + backward.

    Returns dict(logZ [B], grad_L [N,M], grad_R [N,M], grad_log_root [N], grad_log_emit [B,n_max,P]) in
    float64.  Parameter gradients are summed over the batch (weights grad_logZ, default all ones);
    grad_log_emit is per sentence and zero on padding.
    """
    log_emit = np.asarray(log_emit)
    lengths = np.asarray(lengths)
    B, n_max, P = log_emit.shape
    N = np.asarray(L).shape[0]
    out = dict(logZ=np.empty(B), grad_L=np.zeros((N, N + P)), grad_R=np.zeros((N, N + P)),
               grad_log_root=np.zeros(N), grad_log_emit=np.zeros((B, n_max, P)))
    for bi in range(B):
        n = int(lengths[bi])
        g = 1.0 if grad_logZ is None else float(grad_logZ[bi])
        lz, gL, gR, gr, ge = inside_backward_sentence(log_root, L, R, log_emit[bi, :n], g)
        out["logZ"][bi] = lz
        out["grad_L"] += gL
        out["grad_R"] += gR
        out["grad_log_root"] += gr
        out["grad_log_emit"][bi, :n] = ge
    return out
