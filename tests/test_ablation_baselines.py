"""The framework-op baselines of the Table-1 style ablation (log-sum-exp and log-einsum-exp inside passes written
with plain tensor ops, backward by automatic differentiation) against the oracle: log Z and all gradients.
Automatic differentiation of an independently written forward pass is also one more pin of the oracle's
hand-written reverse pass."""
import numpy as np
import pytest
import torch

from oracle import spcfg_oracle as O
from paper_2310_14997_amd import ablation, synth


@pytest.mark.parametrize("variant", ["logsumexp", "logeinsumexp"])
def test_torch_baselines_match_oracle(variant):
    d = synth.make_inputs("tiny", N=9, P=6, B=3, lengths=[7, 7, 7], V=40)
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).double().requires_grad_(True)
    lr, L, R, e = t(d["log_root"]), t(d["L"]), t(d["R"]), t(d["log_emit"])
    g = np.array([1.0, 0.5, 2.0])
    logZ = ablation.inside_torch(lr, L, R, e, variant)
    (logZ * torch.from_numpy(g)).sum().backward()
    ref = O.inside_backward(d["log_root"], d["L"], d["R"], d["log_emit"], d["lengths"], g)
    assert np.allclose(logZ.detach().numpy(), ref["logZ"], rtol=1e-12, atol=1e-12)
    for k, x in (("grad_L", L), ("grad_R", R), ("grad_log_root", lr), ("grad_log_emit", e)):
        assert np.allclose(x.grad.numpy(), ref[k], rtol=1e-9, atol=1e-12), k


@pytest.mark.gpu
def test_ablation_runs_and_variants_agree_on_the_gpu():
    print("case ablation", flush=True)
    out = ablation.one_config(64, 12, 4, 2, True)
    assert set(out["variants"]) == {"fused", "log-einsum-exp", "log-sum-exp"}
    for name, v in out["variants"].items():
        assert v["max_abs_logZ_diff_vs_fused"] < 2e-3, name   # the fp32 framework baselines carry their own rounding
        assert v["grad_L_rel_l2_vs_fused"] < 1e-3, name
        assert v["ms_per_step"] > 0 and v["peak_bytes"] > 0
