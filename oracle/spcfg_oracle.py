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
d o_ij / d a_ik = exp(a_ik + b_kj - o_ij); the rest is the chain rule through the projection identity),
taken with respect to the probability-space entries of L and R, also where an entry is zero.
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


def _log_adjoint_project(W, la):
    """log(exp(la) @ W) for every row of la with the row maximum as the shift;  W: [N, K], la: [S, N]  ->  [S, K]."""
    x = la.max(axis=1, keepdims=True)
    x = np.where(np.isfinite(x), x, 0.0)
    with np.errstate(divide="ignore"):
        return x + np.log(np.exp(la - x) @ W)


def _outer_sum(la, lo):
    """sum_s exp(la[s, A] + lo[s, B])  ->  [N, K], each row pair shifted by its own maxima."""
    x = la.max(axis=1, keepdims=True)
    y = lo.max(axis=1, keepdims=True)
    x = np.where(np.isfinite(x), x, 0.0)
    y = np.where(np.isfinite(y), y, 0.0)
    return (np.exp(la - x) * np.exp(x + y)).T @ np.exp(lo - y)


def inside_backward_sentence(log_root, L, R, e, g=1.0, return_marginals=False):
    """Forward + reverse pass for one sentence.

    Returns (logZ, grad_L, grad_R, grad_log_root, grad_log_emit) for g * log Z, all float64; with
    return_marginals also the dict of span posteriors obar[(i, j)] (width >= 2).  A sentence with Z = 0
    contributes zero gradients.

    grad_L, grad_R are derivatives with respect to the entries of L and R themselves (probability space),
    also at entries that are zero.  The reverse pass therefore carries the adjoints of the probability-space
    quantities beta = exp(o), eta = exp(a), zeta = exp(b), each kept as its logarithm (every adjoint of log Z
    is a sum of products of non-negative weights, so the logarithm exists or is -inf):
        lo_ij[A] = log d logZ / d beta_ij[A],   la_ik[A] = log d logZ / d eta_ik[A],   lb_kj likewise.
    The paper's identity d o_ij / d a_ik = exp(a_ik + b_kj - o_ij) (Sec. 3.2 "Recomputation") is the same
    statement multiplied through by eta_ik / beta_ij; written for eta, zeta, beta themselves it stays
    meaningful where a parent's whole block of L or R is zero (eta = 0, a = -inf) and the log-space adjoint
    d logZ / d a = eta * d logZ / d eta would vanish identically although d logZ / d eta does not.
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
    la = {s: np.full(N, _NEG_INF) for s in a}
    lb = {s: np.full(N, _NEG_INF) for s in b}
    lo = {}

    # root rule: Z = sum_A root[A] beta_0n[A]  =>  d logZ / d beta_0n[A] = root[A] / Z
    lo[(0, n)] = log_root - logZ
    obar[(0, n)] = np.exp(lo[(0, n)] + o[(0, n)])
    g_root += obar[(0, n)]

    for w in range(n, 1, -1):  # every parent of a span is wider, so its adjoints are final here
        spans = [(i, i + w) for i in range(n - w + 1)]
        if w < n:
            # eta = L_N beta, zeta = R_N beta (all spans of this width at once, rows = spans):
            #   d logZ / d beta[B] = sum_A adj_eta[A] L[A,B] + adj_zeta[A] R[A,B]
            #   d logZ / d L[A,B] += adj_eta[A] beta[B],   d logZ / d R[A,B] += adj_zeta[A] beta[B]
            ow = np.stack([o[s] for s in spans])
            las = np.stack([la[s] for s in spans])
            lbs = np.stack([lb[s] for s in spans])
            gL[:, :N] += _outer_sum(las, ow)
            gR[:, :N] += _outer_sum(lbs, ow)
            low = np.logaddexp(_log_adjoint_project(L_N, las), _log_adjoint_project(R_N, lbs))
            for r, s in enumerate(spans):
                lo[s] = low[r]
                obar[s] = np.exp(low[r] + ow[r])  # beta * d logZ / d beta: the span posterior
        # beta_ij = sum_k eta_ik * zeta_kj (Eq. 1 in probability space):
        #   adj_eta_ik += adj_beta_ij * zeta_kj,   adj_zeta_kj += adj_beta_ij * eta_ik
        for (i, j) in spans:
            for k in range(i + 1, j):
                la[(i, k)] = np.logaddexp(la[(i, k)], lo[(i, j)] + b[(k, j)])
                lb[(k, j)] = np.logaddexp(lb[(k, j)], lo[(i, j)] + a[(i, k)])
    # width 1: the same projection backward with the preterminal blocks; beta_i = exp(e_i)
    leaves = [(i, i + 1) for i in range(n)]
    las = np.stack([la[s] for s in leaves])
    lbs = np.stack([lb[s] for s in leaves])
    gL[:, N:] += _outer_sum(las, e)
    gR[:, N:] += _outer_sum(lbs, e)
    g_emit[:] = np.exp(np.logaddexp(_log_adjoint_project(L_P, las), _log_adjoint_project(R_P, lbs)) + e)
    out = (logZ, g * gL, g * gR, g * g_root, g * g_emit)
    if return_marginals:
        out += ({s: g * v for s, v in obar.items()},)
    return out


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
