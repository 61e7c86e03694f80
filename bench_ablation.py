#!/usr/bin/env python3
"""Speed / memory ablation in the manner of the paper's Table 1, on this machine.

The paper compares three ways of running the same inside pass (Sec. 3.2, Table 1):
  * "log-sum-exp": every projection a[A] = logsumexp_B(log L[A,B] + o[B]) is evaluated by materialising the
    [spans, N, M] tensor of sums, framework ops, backward by automatic differentiation;
  * "log-einsum-exp": the same projection as x + log(exp(o - x) @ L^T) with x = max(o), framework ops and
    automatic differentiation (every intermediate of every width is kept for the backward pass);
  * the fused, recomputing implementation: here the HIP library (spcfg_inside_forward_backward).
The first two are written below with plain PyTorch tensor ops on the GPU, as the paper's baselines were; they
are comparison code beside the benchmark, not part of the library package, and double as an independent check of
log Z.  Sentences all have
length l; sizes follow the table (|N| = |P|).  Prints one JSON object per configuration with the time of a
forward+backward step and the peak device memory of each variant, and the ratios in the table's normalisation
(speed relative to the slowest variant, memory relative to the fused one).

    python bench_ablation.py --sizes 512:20,512:40 --batch 8
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import os

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def inside_torch(log_root, L, R, log_emit, variant):
    """log Z [B] of equal-length sentences with plain tensor ops.  L, R: [N, N+P] probabilities."""
    import torch
    B, n, P = log_emit.shape
    N = L.shape[0]
    logL, logR = L.log(), R.log()

    def project(o, W, logW):
        # o: [B, S, K] log inside scores of S spans; returns [B, S, N]
        if variant == "logsumexp":
            return torch.logsumexp(logW[None, None, :, :] + o[:, :, None, :], dim=-1)
        x = o.max(dim=-1, keepdim=True).values
        x = torch.where(torch.isfinite(x), x, torch.zeros_like(x))
        return x + torch.log(torch.einsum("bsk,ak->bsa", torch.exp(o - x), W))

    # a[w][b, i] = projection through L of span (i, i+w), b[w] through R
    a, b_ = {}, {}
    o = log_emit
    a[1] = project(o, L[:, N:], logL[:, N:])
    b_[1] = project(o, R[:, N:], logR[:, N:])
    for w in range(2, n + 1):
        terms = []
        for k in range(1, w):  # left child (i, i+k), right child (i+k, i+w)
            left = a[k][:, : n - w + 1]
            right = b_[w - k][:, k: k + n - w + 1]
            terms.append(left + right)
        o = torch.logsumexp(torch.stack(terms, dim=0), dim=0)  # [B, n-w+1, N]
        if w < n:
            a[w] = project(o, L[:, :N], logL[:, :N])
            b_[w] = project(o, R[:, :N], logR[:, :N])
    return torch.logsumexp(o[:, 0, :] + log_root[None, :], dim=-1)


def run_torch(d, variant, steps):
    import torch
    dev = torch.device("cuda:0")
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev).requires_grad_(True)
    log_root, L, R, log_emit = t(d["log_root"]), t(d["L"]), t(d["R"]), t(d["log_emit"])

    def step():
        for x in (log_root, L, R, log_emit):
            x.grad = None
        logZ = inside_torch(log_root, L, R, log_emit, variant)
        logZ.sum().backward()
        return logZ

    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    logZ = step()
    torch.cuda.synchronize()
    peak = torch.cuda.max_memory_allocated() - base
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    g = lambda x: x.grad.detach().cpu().numpy().astype(np.float64)
    return dict(ms=ms, peak_bytes=int(peak), logZ=logZ.detach().cpu().numpy().astype(np.float64),
                grad_L=g(L), grad_R=g(R), grad_log_root=g(log_root), grad_log_emit=g(log_emit))


def run_fused(d, steps):
    import torch
    from paper_2310_14997_amd import binding as bd
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    wl = bd.Workload(d)
    wl.forward_backward()
    torch.cuda.synchronize()
    inputs = sum(x.numel() * 4 for x in (wl.log_root, wl.L, wl.R, wl.log_emit))
    peak = torch.cuda.max_memory_allocated() - base - inputs  # like the others: memory beyond the inputs
    t0 = time.perf_counter()
    for _ in range(steps):
        wl.forward_backward()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    r = wl.results()
    return dict(ms=ms, peak_bytes=int(peak), logZ=r["logZ"], grad_L=r["grad_L"])


def one_config(N, l, batch, steps, with_logsumexp):
    from paper_2310_14997_amd import synth
    d = synth.make_inputs("tiny", seed=synth.BASE_SEED + 300 + N + l, N=N, P=N, B=batch, lengths=[l] * batch, V=2000)
    out = {"N": N, "P": N, "l": l, "batch": batch, "variants": {}}
    res = {"fused": run_fused(d, steps), "log-einsum-exp": run_torch(d, "logeinsumexp", steps)}
    if with_logsumexp:
        res["log-sum-exp"] = run_torch(d, "logsumexp", max(1, steps // 4))
    ref = res["fused"]
    slowest = max(v["ms"] for v in res.values())
    for name, v in res.items():
        out["variants"][name] = {
            "ms_per_step": v["ms"], "peak_bytes": v["peak_bytes"], "speed_vs_slowest": slowest / v["ms"],
            "memory_vs_fused": v["peak_bytes"] / ref["peak_bytes"],
            "max_abs_logZ_diff_vs_fused": float(np.max(np.abs(v["logZ"] - ref["logZ"]))),
            "grad_L_rel_l2_vs_fused": float(np.linalg.norm(v["grad_L"] - ref["grad_L"]) /
                                            max(np.linalg.norm(ref["grad_L"]), 1e-300))}
    return out


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--sizes", default="512:20,512:40", help="comma list of N:l (the paper's table: 512:20,8192:20,512:40,8192:40)")
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--logsumexp-max-n", type=int, default=1024,
                    help="largest N for which the materialising log-sum-exp variant is run (the paper omits it at 8192)")
    args = ap.parse_args(argv)
    for item in args.sizes.split(","):
        N, l = (int(x) for x in item.split(":"))
        print(json.dumps(one_config(N, l, args.batch, args.steps, N <= args.logsumexp_max_n)), flush=True)


if __name__ == "__main__":
    sys.exit(main())
