"""Seeded synthetic inputs for the simple-PCFG inside pass.

This module only draws random grammars and sentences; it holds none of the
inside algorithm's arithmetic, so both the HIP path and the CPU oracle can be
fed from it without sharing any of the method's code.

The grammar follows the paper's rule set (Sec. 2): a root distribution over the
N nonterminals, left/right production matrices L, R of shape [N, N+P] whose rows
are distributions over the children (nonterminals first, then preterminals), and
an emission table [P, V].  The library takes the emissions already gathered per
token, log_emit[b, i, :] = log pi(T -> w_{b,i}).

Sentence lengths and token frequencies imitate the Penn-Treebank-like workloads
the paper trains on (Sec. 4): no treebank text is used, only a length law and a
bounded Zipf law over token ids.
"""
from __future__ import annotations

import numpy as np

# name -> (B, length law, N, P, V, logit scale of L/R, precision)
CONFIGS = {
    "tiny": dict(B=4, lengths=("const", 10), N=30, P=60, V=200, lr_scale=1.0, precision="fp32"),
    "small": dict(B=32, lengths=("uniform", 10, 30), N=512, P=512, V=10000, lr_scale=1.0, precision="fp32"),
    "ptb": dict(B=64, lengths=("normal", 22.0, 10.0, 2, 40), N=2048, P=2048, V=10000, lr_scale=2.0,
                precision="fp32"),
    "scaled": dict(B=32, lengths=("const", 40), N=4096, P=4096, V=10000, lr_scale=1.0, precision="bf16"),
    "long": dict(B=4, lengths=("uniform", 100, 200), N=1024, P=1024, V=10000, lr_scale=1.0, precision="fp32"),
    # correctness-only: peaked rows and structural zeros, to exercise underflow and zero-probability guards
    "adversarial": dict(B=8, lengths=("uniform", 4, 24), N=96, P=80, V=500, lr_scale=8.0, precision="fp32",
                        zero_frac=0.3),
}
_ORDER = ["tiny", "small", "ptb", "scaled", "long", "adversarial"]
BASE_SEED = 20231014


def _softmax_rows(z):
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def _log_softmax_rows(z):
    z = z - z.max(axis=-1, keepdims=True)
    return z - np.log(np.exp(z).sum(axis=-1, keepdims=True))


def draw_lengths(rng, law, B):
    kind = law[0]
    if kind == "const":
        return np.full(B, law[1], dtype=np.int32)
    if kind == "uniform":  # inclusive bounds
        return rng.integers(law[1], law[2] + 1, size=B).astype(np.int32)
    if kind == "normal":  # round, then clamp (no resampling)
        _, mean, sd, lo, hi = law
        return np.clip(np.rint(rng.normal(mean, sd, size=B)), lo, hi).astype(np.int32)
    raise ValueError(kind)


def zipf_tokens(rng, V, size, s=1.1):
    """Bounded Zipf: p(r) ~ r^-s for ranks r = 1..V, token id = r - 1 (inverse CDF on the normalised table)."""
    p = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(p / p.sum())
    u = rng.random(size)
    return np.minimum(np.searchsorted(cdf, u, side="right"), V - 1).astype(np.int64)


def make_inputs(name="tiny", seed=None, pad_value=0.0, **overrides):
    """Return a dict of numpy arrays for one named workload.

    Keys: log_root [N] f32, L, R [N, N+P] f32 (probabilities), log_emit [B, n_max, P] f32,
    lengths [B] i32, tokens [B, n_max] i64 (-1 on padding), plus the scalars N, P, V, B, n_max.
    `overrides` may replace B, N, P, V, lengths (a law tuple or an explicit list), lr_scale, zero_frac.
    Padded token positions of log_emit hold `pad_value` (tests use NaN to catch reads of padding).
    """
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    if seed is None:
        seed = BASE_SEED + _ORDER.index(name)
    rng = np.random.default_rng(seed)
    B, N, P, V = int(cfg["B"]), int(cfg["N"]), int(cfg["P"]), int(cfg["V"])
    M = N + P
    law = cfg["lengths"]
    if isinstance(law, tuple):
        lengths = draw_lengths(rng, law, B)
    else:
        lengths = np.asarray(law, dtype=np.int32)
        assert lengths.shape == (B,)
    n_max = int(lengths.max())

    root_logits = rng.normal(size=N)
    L_logits = cfg["lr_scale"] * rng.normal(size=(N, M))
    R_logits = cfg["lr_scale"] * rng.normal(size=(N, M))
    L = _softmax_rows(L_logits)
    R = _softmax_rows(R_logits)
    zf = float(cfg.get("zero_frac", 0.0))
    if zf > 0.0:  # structural zeros; rows are not renormalised (the path takes arbitrary non-negative weights)
        L = np.where(rng.random(L.shape) < zf, 0.0, L)
        R = np.where(rng.random(R.shape) < zf, 0.0, R)
    log_root = _log_softmax_rows(root_logits[None, :])[0]
    log_emis = _log_softmax_rows(rng.normal(size=(P, V)))  # [P, V]

    tokens = np.full((B, n_max), -1, dtype=np.int64)
    log_emit = np.full((B, n_max, P), pad_value, dtype=np.float32)
    for b in range(B):
        n = int(lengths[b])
        tok = zipf_tokens(rng, V, n)
        tokens[b, :n] = tok
        log_emit[b, :n, :] = log_emis[:, tok].T.astype(np.float32)

    return dict(name=name, seed=seed, B=B, N=N, P=P, V=V, n_max=n_max, precision=cfg["precision"],
                log_root=log_root.astype(np.float32), L=L.astype(np.float32), R=R.astype(np.float32),
                log_emit=log_emit, lengths=lengths, tokens=tokens)


def make_inputs_per_sentence(name="tiny", seed=None, pad_value=0.0, **overrides):
    """Like make_inputs, but every sentence has a grammar of its own (the setting of the compound variant,
    App. A, where rule probabilities depend on a per-sentence latent vector): log_root [B, N], L, R [B, N, N+P],
    and emissions drawn from a per-sentence table.  A shared random part plus a per-sentence perturbation of the
    logits, so the grammars are related but distinct."""
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    if seed is None:
        seed = BASE_SEED + 200 + _ORDER.index(name)
    rng = np.random.default_rng(seed)
    B, N, P, V = int(cfg["B"]), int(cfg["N"]), int(cfg["P"]), int(cfg["V"])
    M = N + P
    law = cfg["lengths"]
    lengths = draw_lengths(rng, law, B) if isinstance(law, tuple) else np.asarray(law, dtype=np.int32)
    assert lengths.shape == (B,)
    n_max = int(lengths.max())
    sc = cfg["lr_scale"]
    base = dict(root=rng.normal(size=N), L=sc * rng.normal(size=(N, M)), R=sc * rng.normal(size=(N, M)),
                E=rng.normal(size=(P, V)))
    log_root = np.empty((B, N), np.float32)
    L = np.empty((B, N, M), np.float32)
    R = np.empty((B, N, M), np.float32)
    tokens = np.full((B, n_max), -1, dtype=np.int64)
    log_emit = np.full((B, n_max, P), pad_value, dtype=np.float32)
    for b in range(B):
        log_root[b] = _log_softmax_rows((base["root"] + 0.5 * rng.normal(size=N))[None, :])[0]
        L[b] = _softmax_rows(base["L"] + 0.5 * sc * rng.normal(size=(N, M)))
        R[b] = _softmax_rows(base["R"] + 0.5 * sc * rng.normal(size=(N, M)))
        n = int(lengths[b])
        tok = zipf_tokens(rng, V, n)
        tokens[b, :n] = tok
        log_emis = _log_softmax_rows(base["E"][:, tok].T + 0.5 * rng.normal(size=(n, P)))  # only the columns in use
        log_emit[b, :n, :] = log_emis.astype(np.float32)
    return dict(name=name, seed=seed, B=B, N=N, P=P, V=V, n_max=n_max, precision="fp32", log_root=log_root, L=L, R=R,
                log_emit=log_emit, lengths=lengths, tokens=tokens)


def make_logits(name="tiny", seed=None, **overrides):
    """Scores for the rule-probability front-end of one named workload: root [N], L/R [N, N+P] (scaled like the
    workload's grammar), emission [P, V] logits, int32 tokens [B, n_max] (-1 on padding) and lengths."""
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    if seed is None:
        seed = BASE_SEED + 100 + _ORDER.index(name)
    rng = np.random.default_rng(seed)
    B, N, P, V = int(cfg["B"]), int(cfg["N"]), int(cfg["P"]), int(cfg["V"])
    law = cfg["lengths"]
    lengths = draw_lengths(rng, law, B) if isinstance(law, tuple) else np.asarray(law, dtype=np.int32)
    n_max = int(lengths.max())
    tokens = np.full((B, n_max), -1, dtype=np.int32)
    for b in range(B):
        tokens[b, : int(lengths[b])] = zipf_tokens(rng, V, int(lengths[b]))
    f = np.float32
    return dict(name=name, seed=seed, B=B, N=N, P=P, V=V, n_max=n_max, lengths=lengths, tokens=tokens,
                root_logits=rng.normal(size=N).astype(f),
                L_logits=(cfg["lr_scale"] * rng.normal(size=(N, N + P))).astype(f),
                R_logits=(cfg["lr_scale"] * rng.normal(size=(N, N + P))).astype(f),
                emis_logits=rng.normal(size=(P, V)).astype(f))


def work_counts(lengths, N, P):
    """Algorithmic work of one forward pass: projected spans, split terms, GEMM flop, split-reduction bytes."""
    n = np.asarray(lengths, dtype=np.int64)
    leaves = int(n.sum())
    proj_spans = int((n * (n - 1) // 2 - 1).sum())  # width >= 2, root excluded
    split_terms = int(((n - 1) * n * (n + 1) // 6).sum())
    flop_fwd = 4 * N * N * proj_spans + 4 * N * P * leaves
    split_bytes_fwd = 8 * N * split_terms
    return dict(leaves=leaves, proj_spans=proj_spans, split_terms=split_terms, flop_fwd=flop_fwd,
                flop_fwd_bwd=3 * flop_fwd, split_read_bytes_fwd=split_bytes_fwd)
