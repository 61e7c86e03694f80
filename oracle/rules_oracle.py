"""CPU oracle for the rule-probability front-end and its backward.  TEST INFRASTRUCTURE ONLY.

The paper's neural parameterisation (App. A) ends in four softmaxes: over the nonterminals for the root rule,
over N u P children for the left and for the right production of every parent, and over the vocabulary for
every preterminal.  This oracle takes the scores (logits) those softmaxes are applied to and produces what the
inside pass consumes:

    log_root = log_softmax(root_logits)                         pi(S -> A)
    L = softmax(L_logits, axis=1),  R = softmax(R_logits, axis=1)   pi(B <- A), pi(A -> C)   (probability space)
    log_emit[b, i, T] = log_softmax(emis_logits[T, :])[tok[b, i]]   pi(T -> w_{b,i}), 0 on padding

and, for upstream gradients w.r.t. those outputs, the gradients w.r.t. the logits (plain chain rule through
softmax / log-softmax / gather).  Double precision, numpy; shares no code with the HIP path.
Pinned in tests/test_rules_oracle.py (normalisation, finite differences, zero-sum rows, composition with
the inside oracle).
"""
from __future__ import annotations

import numpy as np


def _log_softmax(z, axis):
    z = z - z.max(axis=axis, keepdims=True)
    return z - np.log(np.exp(z).sum(axis=axis, keepdims=True))


def forward(root_logits, L_logits, R_logits, emis_logits, tokens, lengths):
    root_logits, L_logits, R_logits, emis_logits = (np.asarray(x, dtype=np.float64) for x in
                                                    (root_logits, L_logits, R_logits, emis_logits))
    tokens = np.asarray(tokens)
    B, n_max = tokens.shape
    P = emis_logits.shape[0]
    log_root = _log_softmax(root_logits[None, :], 1)[0]
    L = np.exp(_log_softmax(L_logits, 1))
    R = np.exp(_log_softmax(R_logits, 1))
    log_emis = _log_softmax(emis_logits, 1)  # [P, V]
    log_emit = np.zeros((B, n_max, P))
    for b in range(B):
        n = int(lengths[b])
        log_emit[b, :n] = log_emis[:, tokens[b, :n]].T
    return dict(log_root=log_root, L=L, R=R, log_emit=log_emit)


def backward(root_logits, L_logits, R_logits, emis_logits, tokens, lengths, grad_log_root, grad_L, grad_R,
             grad_log_emit):
    """Gradients w.r.t. the four logit arrays given gradients w.r.t. forward()'s outputs."""
    fw = forward(root_logits, L_logits, R_logits, emis_logits, tokens, lengths)
    grad_log_root, grad_L, grad_R, grad_log_emit = (np.asarray(x, dtype=np.float64) for x in
                                                    (grad_log_root, grad_L, grad_R, grad_log_emit))
    emis_logits = np.asarray(emis_logits, dtype=np.float64)
    tokens = np.asarray(tokens)
    # log-softmax: d/dz_j sum_i g_i (z_i - lse) = g_j - softmax_j * sum_i g_i
    g_root = grad_log_root - np.exp(fw["log_root"]) * grad_log_root.sum()
    # softmax: d/dz_j sum_i g_i p_i = p_j (g_j - sum_i g_i p_i)
    g_Ll = fw["L"] * (grad_L - (grad_L * fw["L"]).sum(axis=1, keepdims=True))
    g_Rl = fw["R"] * (grad_R - (grad_R * fw["R"]).sum(axis=1, keepdims=True))
    P, V = emis_logits.shape
    soft = np.exp(_log_softmax(emis_logits, 1))
    g_emis = np.zeros((P, V))
    tot = np.zeros(P)
    for b in range(tokens.shape[0]):
        for i in range(int(lengths[b])):
            g_emis[:, tokens[b, i]] += grad_log_emit[b, i]
            tot += grad_log_emit[b, i]
    g_emis -= soft * tot[:, None]
    return dict(grad_root_logits=g_root, grad_L_logits=g_Ll, grad_R_logits=g_Rl, grad_emis_logits=g_emis)
