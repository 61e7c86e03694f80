"""The framework-op baselines of the Table-1 style ablation (log-sum-exp and log-einsum-exp inside passes written
with plain tensor ops, backward by automatic differentiation) against the oracle: log Z and all gradients.
Automatic differentiation of an independently written forward pass is also one more pin of the oracle's
hand-written reverse pass."""
import numpy as np
import pytest
import torch

from oracle import spcfg_oracle as O
import bench_ablation as ablation
from paper_2310_14997_amd import synth


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


@pytest.mark.gpu
def test_framework_baselines_match_the_oracle_at_table_size():
    """The two baselines at a size of the paper's Table 1 (|N| = |P| = 512, l = 20) against the oracle: they are fp32
    framework code (log-space, automatic differentiation), so log Z is held to the fp32 bar and the gradients to the
    gradient bar."""
    from parity_util import check_all
    d = synth.make_inputs("tiny", seed=synth.BASE_SEED + 300 + 512 + 20, pad_value=0.0, N=512, P=512, B=2, lengths=[20, 20],
                          V=2000)
    print("case ablation baselines vs oracle, N=512 l=20", flush=True)
    ref = O.inside_backward(d["log_root"], d["L"], d["R"], d["log_emit"], d["lengths"])
    for variant in ("logeinsumexp", "logsumexp"):
        got = ablation.run_torch(d, variant, 1)
        print(" ", variant, check_all(got, ref), flush=True)
