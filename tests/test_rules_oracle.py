"""Pins for the front-end oracle (softmaxes of App. A and their backward)."""
import numpy as np
import pytest

from oracle import rules_oracle as RO
from oracle import spcfg_oracle as O


def make(rng, N=5, P=4, V=9, lens=(3, 5, 2)):
    M = N + P
    B, n_max = len(lens), max(lens)
    tokens = np.full((B, n_max), -1, dtype=np.int64)
    for b, n in enumerate(lens):
        tokens[b, :n] = rng.integers(0, V, size=n)
    tokens[0, 1] = tokens[0, 0]  # a repeated token inside one sentence
    return dict(root_logits=rng.normal(size=N), L_logits=2 * rng.normal(size=(N, M)), R_logits=rng.normal(size=(N, M)),
                emis_logits=rng.normal(size=(P, V)), tokens=tokens, lengths=np.array(lens))


def test_outputs_are_normalised_distributions():
    d = make(np.random.default_rng(0))
    fw = RO.forward(**d)
    assert np.allclose(fw["L"].sum(1), 1) and np.allclose(fw["R"].sum(1), 1)
    assert np.isclose(np.exp(fw["log_root"]).sum(), 1)
    # gathered emissions are columns of a row-stochastic table
    table = np.exp(d["emis_logits"] - d["emis_logits"].max(1, keepdims=True))
    table /= table.sum(1, keepdims=True)
    b, i = 1, 3
    assert np.allclose(np.exp(fw["log_emit"][b, i]), table[:, d["tokens"][b, i]])
    assert np.all(fw["log_emit"][2, 2:] == 0.0)  # padding
    # shift invariance of every softmax
    d2 = dict(d, L_logits=d["L_logits"] + 3.0, root_logits=d["root_logits"] - 7.0, emis_logits=d["emis_logits"] + 1.5)
    fw2 = RO.forward(**d2)
    for k in fw:
        assert np.allclose(fw[k], fw2[k], atol=1e-12)


def test_backward_matches_finite_differences_and_zero_sum_rows():
    rng = np.random.default_rng(1)
    d = make(rng)
    fw = RO.forward(**d)
    gs = dict(grad_log_root=rng.normal(size=fw["log_root"].shape), grad_L=rng.normal(size=fw["L"].shape),
              grad_R=rng.normal(size=fw["R"].shape), grad_log_emit=rng.normal(size=fw["log_emit"].shape))
    for b, n in enumerate(d["lengths"]):
        gs["grad_log_emit"][b, n:] = 0.0
    bw = RO.backward(**d, **gs)

    def f(dd):
        o = RO.forward(**dd)
        return ((o["log_root"] * gs["grad_log_root"]).sum() + (o["L"] * gs["grad_L"]).sum()
                + (o["R"] * gs["grad_R"]).sum() + (o["log_emit"] * gs["grad_log_emit"]).sum())

    h = 1e-6
    for key, gkey in (("root_logits", "grad_root_logits"), ("L_logits", "grad_L_logits"),
                      ("R_logits", "grad_R_logits"), ("emis_logits", "grad_emis_logits")):
        for _ in range(3):
            dirn = rng.normal(size=d[key].shape)
            num = (f(dict(d, **{key: d[key] + h * dirn})) - f(dict(d, **{key: d[key] - h * dirn}))) / (2 * h)
            assert (bw[gkey] * dirn).sum() == pytest.approx(num, rel=1e-6, abs=1e-9)
        # a constant added to the logits of one softmax changes nothing: gradient rows sum to zero
        assert np.allclose(bw[gkey].sum(axis=-1), 0.0, atol=1e-12)


def test_composition_with_the_inside_oracle():
    """d log Z / d logits through front-end backward o inside backward equals finite differences of log Z."""
    rng = np.random.default_rng(2)
    d = make(rng, N=4, P=3, V=6, lens=(4, 3))

    def logZ_sum(dd):
        o = RO.forward(**dd)
        return O.inside(o["log_root"], o["L"], o["R"], o["log_emit"], dd["lengths"]).sum()

    fw = RO.forward(**d)
    ins = O.inside_backward(fw["log_root"], fw["L"], fw["R"], fw["log_emit"], d["lengths"])
    bw = RO.backward(**d, grad_log_root=ins["grad_log_root"], grad_L=ins["grad_L"], grad_R=ins["grad_R"],
                     grad_log_emit=ins["grad_log_emit"])
    h = 1e-6
    for key, gkey in (("root_logits", "grad_root_logits"), ("L_logits", "grad_L_logits"),
                      ("R_logits", "grad_R_logits"), ("emis_logits", "grad_emis_logits")):
        dirn = rng.normal(size=d[key].shape)
        num = (logZ_sum(dict(d, **{key: d[key] + h * dirn})) - logZ_sum(dict(d, **{key: d[key] - h * dirn}))) / (2 * h)
        assert (bw[gkey] * dirn).sum() == pytest.approx(num, rel=2e-6, abs=1e-9)
