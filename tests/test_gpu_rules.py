"""GPU parity of the rule-probability front-end (softmaxes + emission gather) and its backward against the
CPU oracle, and of the composed pipeline logits -> front-end -> inside -> backward -> logit gradients."""
import numpy as np
import pytest

from oracle import rules_oracle as RO
from oracle import spcfg_oracle as O
from paper_2310_14997_amd import binding as bd
from paper_2310_14997_amd import synth
from parity_util import check_grad

pytestmark = pytest.mark.gpu

FWD_RTOL = 2e-6   # fp32 exp / log / one row reduction per output
BWD_RTOL = 1e-4   # the gradient tolerance of the fp32 path


def run_gpu(d, grads=None):
    import torch
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    N, P, V, B, n_max = d["N"], d["P"], d["V"], d["B"], d["n_max"]
    M = N + P
    f = dict(dtype=torch.float32, device=dev)
    tin = {k: t(d[k]) for k in ("root_logits", "L_logits", "R_logits", "emis_logits", "tokens")}
    out = dict(log_root=torch.empty(N, **f), L=torch.empty(N, M, **f), R=torch.empty(N, M, **f),
               log_emit=torch.full((B, n_max, P), float("nan"), **f), emis_lse=torch.empty(P, **f))
    bd.spcfg_rules_forward(tin["root_logits"], tin["L_logits"], tin["R_logits"], tin["emis_logits"], tin["tokens"],
                           d["lengths"], out["log_root"], out["L"], out["R"], out["log_emit"], out["emis_lse"])
    res = {k: v.cpu().numpy().astype(np.float64) for k, v in out.items()}
    if grads is None:
        return res, out, tin
    g = {k: t(np.asarray(v, dtype=np.float32)) for k, v in grads.items()}
    go = dict(grad_root_logits=torch.empty(N, **f), grad_L_logits=torch.empty(N, M, **f),
              grad_R_logits=torch.empty(N, M, **f), grad_emis_logits=torch.empty(P, V, **f))
    bd.spcfg_rules_backward(out["log_root"], out["L"], out["R"], tin["emis_logits"], out["emis_lse"], tin["tokens"],
                            d["lengths"], g["grad_log_root"], g["grad_L"], g["grad_R"], g["grad_log_emit"],
                            go["grad_root_logits"], go["grad_L_logits"], go["grad_R_logits"], go["grad_emis_logits"],
                            torch.empty(32, P, **f))
    res.update({k: v.cpu().numpy().astype(np.float64) for k, v in go.items()})
    return res, out, tin


@pytest.mark.parametrize("name,kw", [
    ("tiny", {}),
    ("tiny", dict(N=70, P=45, V=333, B=5, lengths=[2, 9, 17, 5, 12])),
    ("small", dict(B=8)),
])
def test_frontend_forward_and_backward(name, kw):
    d = synth.make_logits(name, **kw)
    print("case rules", name, kw, flush=True)
    ref = RO.forward(d["root_logits"], d["L_logits"], d["R_logits"], d["emis_logits"], d["tokens"], d["lengths"])
    rng = np.random.default_rng(5)
    grads = dict(grad_log_root=rng.normal(size=ref["log_root"].shape), grad_L=rng.normal(size=ref["L"].shape),
                 grad_R=rng.normal(size=ref["R"].shape), grad_log_emit=rng.normal(size=ref["log_emit"].shape))
    for b, n in enumerate(d["lengths"]):
        grads["grad_log_emit"][b, int(n):] = 0.0
    got, _, _ = run_gpu(d, grads)
    for k in ("log_root", "L", "R", "log_emit"):
        check_grad(k, got[k], ref[k], FWD_RTOL)
    rb = RO.backward(d["root_logits"], d["L_logits"], d["R_logits"], d["emis_logits"], d["tokens"], d["lengths"],
                     **{k: np.asarray(v, dtype=np.float32) for k, v in grads.items()})
    for k in ("grad_root_logits", "grad_L_logits", "grad_R_logits", "grad_emis_logits"):
        check_grad(k, got[k], rb[k], BWD_RTOL)
    again, _, _ = run_gpu(d, grads)
    for k in got:
        assert np.array_equal(got[k], again[k]), f"{k}: two runs differ bitwise"


def test_logits_to_logit_gradients_through_the_inside_pass():
    """Whole chain on the GPU: front-end -> inside -> inside backward -> front-end backward, against the same
    chain of the two CPU oracles."""
    import torch
    d = synth.make_logits("tiny", N=96, P=80, V=400, B=6, lengths=[12, 5, 9, 3, 20, 7])
    print("case rules chain", flush=True)
    fw, out, tin = run_gpu(d)
    wl_in = dict(B=d["B"], N=d["N"], P=d["P"], n_max=d["n_max"], lengths=d["lengths"], log_root=fw["log_root"].astype(np.float32),
                 L=fw["L"].astype(np.float32), R=fw["R"].astype(np.float32), log_emit=fw["log_emit"].astype(np.float32))
    wl = bd.Workload(wl_in)
    wl.log_root, wl.L, wl.R, wl.log_emit = out["log_root"], out["L"], out["R"], out["log_emit"]
    wl.forward_backward()
    dev = torch.device("cuda:0")
    f = dict(dtype=torch.float32, device=dev)
    N, P, V = d["N"], d["P"], d["V"]
    go = dict(r=torch.empty(N, **f), l=torch.empty(N, N + P, **f), rr=torch.empty(N, N + P, **f), e=torch.empty(P, V, **f))
    bd.spcfg_rules_backward(out["log_root"], out["L"], out["R"], tin["emis_logits"], out["emis_lse"], tin["tokens"],
                            d["lengths"], wl.grad_log_root, wl.grad_L, wl.grad_R, wl.grad_log_emit, go["r"], go["l"],
                            go["rr"], go["e"], torch.empty(32, P, **f))
    torch.cuda.synchronize()
    rf = RO.forward(d["root_logits"], d["L_logits"], d["R_logits"], d["emis_logits"], d["tokens"], d["lengths"])
    ins = O.inside_backward(rf["log_root"], rf["L"], rf["R"], rf["log_emit"], d["lengths"])
    rb = RO.backward(d["root_logits"], d["L_logits"], d["R_logits"], d["emis_logits"], d["tokens"], d["lengths"],
                     ins["grad_log_root"], ins["grad_L"], ins["grad_R"], ins["grad_log_emit"])
    check_grad("logZ", wl.logZ.cpu().numpy(), ins["logZ"], 1e-5)
    check_grad("grad_root_logits", go["r"].cpu().numpy(), rb["grad_root_logits"], 2e-4)
    check_grad("grad_L_logits", go["l"].cpu().numpy(), rb["grad_L_logits"], 2e-4)
    check_grad("grad_R_logits", go["rr"].cpu().numpy(), rb["grad_R_logits"], 2e-4)
    check_grad("grad_emis_logits", go["e"].cpu().numpy(), rb["grad_emis_logits"], 2e-4)


def test_invalid_token_gives_nan_not_a_fault():
    d = synth.make_logits("tiny")
    d["tokens"] = d["tokens"].copy()
    d["tokens"][1, 2] = d["V"] + 5
    got, _, _ = run_gpu(d)
    assert np.all(np.isnan(got["log_emit"][1, 2])) and np.all(np.isfinite(got["log_emit"][1, 3]))
