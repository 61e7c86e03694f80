#!/usr/bin/env python3
"""Benchmark of the simple-PCFG inside forward+backward pass on one MI355X.

A step is one spcfg_inside_forward_backward call (every kernel of the hot path) on one synthetic
PTB-shaped batch (N = P = 2048, B = 64, lengths <= 40) whose inputs are already resident in HBM.
Prints ONE JSON line: sentences/s, plus `roofline` for the dominant kernel (the stacked projection GEMM, whose
fp32 products are formed from six bf16 MFMA piece products each, timed with HIP events inside the library on
the launch stream) and `cpu_baseline` (the CPU oracle timed on
a bounded sample of the same batch on this machine's host cores).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
# fp32 operands, default path: every fp32 product costs six bf16 matrix-instruction products (three exact bf16
# pieces per operand, the six largest of the nine piece products), so the matrix cores can deliver at most
# a sixth of their bf16 rate in fp32-equivalent flop
SPLIT_PRODUCTS = 6
PEAK_SPLIT_TFLOPS = PEAK_BF16_MFMA_TFLOPS / SPLIT_PRODUCTS
PEAK_HBM_GBS = 8000.0


def cpu_baseline(d, max_sentences, budget_s=25.0):
    """Time the oracle (as it stands, fp64 numpy) on the first sentences of the batch; bounded by budget_s."""
    from oracle import spcfg_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    done, t0 = 0, time.perf_counter()
    for b in range(min(max_sentences, d["B"])):
        n = int(d["lengths"][b])
        if d["L"].ndim == 3:  # one grammar per sentence
            O.inside_backward_sentence(d["log_root"][b], d["L"][b], d["R"][b], d["log_emit"][b, :n])
        else:
            O.inside_backward_sentence(d["log_root"], d["L"], d["R"], d["log_emit"][b, :n])
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return dict(value=done / dt, unit="sentences/s", cores=int(cores), kind="oracle",
                sample=f"first {done} sentences of the batch (lengths {d['lengths'][:done].tolist()}), "
                       f"fp64 numpy oracle forward+backward, {dt:.1f} s")


def time_frontend(workload, wl, steps):
    """Front-end forward and backward on the workload's shape (HBM-bound passes over the logit matrices and the
    P x V emission table), timed with events on the launch stream; gradients fed from the inside pass's outputs."""
    import torch
    from paper_2310_14997_amd import binding as bd
    from paper_2310_14997_amd import synth
    d = synth.make_logits(workload)
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    N, P, V, B, n_max = d["N"], d["P"], d["V"], d["B"], d["n_max"]
    M = N + P
    f = dict(dtype=torch.float32, device=dev)
    tin = {k: t(d[k]) for k in ("root_logits", "L_logits", "R_logits", "emis_logits", "tokens")}
    o = dict(log_root=torch.empty(N, **f), L=torch.empty(N, M, **f), R=torch.empty(N, M, **f),
             log_emit=torch.empty(B, n_max, P, **f), lse=torch.empty(P, **f))
    g = dict(r=torch.empty(N, **f), l=torch.empty(N, M, **f), rr=torch.empty(N, M, **f), e=torch.empty(P, V, **f),
             s=torch.empty(32, P, **f))

    def fwd():
        bd.spcfg_rules_forward(tin["root_logits"], tin["L_logits"], tin["R_logits"], tin["emis_logits"], tin["tokens"],
                               d["lengths"], o["log_root"], o["L"], o["R"], o["log_emit"], o["lse"])

    def bwd():
        bd.spcfg_rules_backward(o["log_root"], o["L"], o["R"], tin["emis_logits"], o["lse"], tin["tokens"], d["lengths"],
                                wl.grad_log_root, wl.grad_L, wl.grad_R, wl.grad_log_emit, g["r"], g["l"], g["rr"], g["e"],
                                g["s"])

    res = {}
    for name, fn, byt in (("forward", fwd, 4.0 * (4 * N * M + P * V + 2 * B * n_max * P)),
                          ("backward", bwd, 4.0 * (6 * N * M + 2 * P * V + 2 * B * n_max * P))):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        res[name] = {"ms": ms, "algorithmic_GBps": byt / (ms * 1e-3) / 1e9}
    return res


def time_decode(wl, steps):
    """Span-posterior export and best-tree decoding on the workspace the last step left behind."""
    import torch
    from paper_2310_14997_amd import binding as bd
    dev = wl.logZ.device
    B, n_max = wl.B, wl.n_max
    mu = torch.empty(B, n_max, n_max, dtype=torch.float32, device=dev)
    lab = torch.empty(B, n_max, n_max, dtype=torch.int32, device=dev)
    spans = torch.empty(B, n_max - 1, 2, dtype=torch.int32, device=dev)
    score = torch.empty(B, dtype=torch.float32, device=dev)
    scratch = torch.empty(bd.spcfg_mbr_decode_scratch_bytes(B, n_max), dtype=torch.uint8, device=dev)
    n = wl.lengths.astype(np.int64)
    rows = int((n * (n + 1) // 2).sum())  # one root row per width-1 entry plus every wider span
    res = {}
    for name, fn, byt in (("span_marginals", lambda: bd.spcfg_span_marginals(wl.cfg, wl.lengths, n_max, wl.workspace,
                                                                             mu, lab), 8.0 * wl.N * rows),
                          ("mbr_decode", lambda: bd.spcfg_mbr_decode(mu, wl.lengths, spans, score, scratch), None)):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        res[name] = {"ms": ms}
        if byt:
            res[name]["algorithmic_GBps"] = byt / (ms * 1e-3) / 1e9
    return res


def mfma_sustained():
    """What a register-only loop of the products' matrix instruction sustains on this GPU right now (bench_mfma_ceiling.hip,
    built beside the library): the published peak assumes 2.4 GHz, and the chip lowers its clock under matrix load,
    the more the more the operands change.  Context for roofline.frac, which stays priced against the published peak."""
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2310_14997_amd", "mfma_ceiling.bin")
    try:
        res = subprocess.run([exe], capture_output=True, text=True, timeout=60, check=True)
        return json.loads(res.stdout.strip().splitlines()[-1])
    except Exception as e:  # the probe is optional: report why it is missing rather than fail the benchmark
        return {"error": repr(e)[:200]}


def measure(d, bf16, fp32_mfma, steps, warmup, profile_steps, graph=False, extra_flags=0):
    """Times `steps` forward+backward steps on the batch `d` (inputs resident in HBM), then repeats `profile_steps`
    steps with HIP events bound to every kernel's own dispatch for the per-class times."""
    import torch
    from paper_2310_14997_amd import binding as bd
    from paper_2310_14997_amd import synth
    wl = bd.Workload(d, precision=bd.PRECISION_BF16 if bf16 else bd.PRECISION_FP32,
                     flags=(bd.FLAG_FP32_MFMA if fp32_mfma else 0) | extra_flags)
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else (PEAK_FP32_MFMA_TFLOPS if fp32_mfma else PEAK_SPLIT_TFLOPS)
    if bf16:
        kernel_name, mfma = ("k_gemm_nt3 (forward: operands as two bf16 pieces, 3 bf16 MFMA products, not counted in "
                             "the flop) / k_gemm_nt16 (reverse: single bf16 operands", "bf16")
    elif fp32_mfma:
        kernel_name, mfma = "k_gemm_nt (fp32 MFMA", "f32"
    else:
        kernel_name, mfma = ("k_gemm_nt3 / k_gemm_nt (fp32 operands as 3 bf16 pieces, 6 bf16 MFMA products per fp32 "
                             "product; pre-cut planes for 128-row tiles, cut in the kernel for shorter ones"), "bf16 x6"
    wc = synth.work_counts(d["lengths"], d["N"], d["P"])
    stream = torch.cuda.current_stream()
    step = wl.forward_backward
    if graph:  # the step only enqueues kernels, so it can be captured once and replayed
        wl.forward_backward()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            wl.forward_backward()
        stream.wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            wl.forward_backward()
        step = g.replay
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    logz = wl.logZ.cpu().numpy()
    assert np.all(np.isfinite(logz)), "non-finite log Z in the benchmark batch"
    res = dict(wl=wl, wc=wc, ms_per_step=dt / steps * 1e3, sentences_per_s=d["B"] / (dt / steps), classes=None,
               roofline=None, gemm_grad=None, split_reduction=None)
    psteps = steps if profile_steps is None else profile_steps
    if psteps <= 0:
        return res
    # per-kernel-class device time: the same steps again, every launch carrying start/stop HIP events bound to
    # its own dispatch on the launch stream (kept out of the timed region above: the events perturb the schedule)
    bd.spcfg_profile_enable(True)
    for _ in range(psteps):
        wl.forward_backward()
    torch.cuda.synchronize()
    prof = bd.spcfg_profile_read()
    bd.spcfg_profile_enable(False)
    classes = {k: dict(ms_per_step=v["ms"] / psteps, launches_per_step=v["launches"] / psteps,
                       work_per_step=v["work"] / psteps) for k, v in prof.items()}
    proj_ms = classes["gemm_fwd"]["ms_per_step"] + classes["gemm_bwd"]["ms_per_step"]
    proj_flop = classes["gemm_fwd"]["work_per_step"] + classes["gemm_bwd"]["work_per_step"]
    proj_launches = classes["gemm_fwd"]["launches_per_step"] + classes["gemm_bwd"]["launches_per_step"]
    achieved = proj_flop / (proj_ms * 1e-3) / 1e12
    split_ms = classes["split_fwd"]["ms_per_step"] + classes["split_bwd"]["ms_per_step"]
    split_bytes = classes["split_fwd"]["work_per_step"] + classes["split_bwd"]["work_per_step"]
    gg = classes["gemm_grad"]
    gg_tflops = gg["work_per_step"] / (gg["ms_per_step"] * 1e-3) / 1e12
    res["classes"] = classes
    res["roofline"] = {"bound": "mfma", "kernel": kernel_name + "; stacked projection, forward + reverse)", "mfma": mfma,
                       "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                       "launches_per_step": proj_launches, "avg_launch_us": proj_ms * 1e3 / max(proj_launches, 1),
                       "flop_per_launch": proj_flop / max(proj_launches, 1)}
    res["gemm_grad"] = {"bound": "mfma", "kernel": "rule-gradient product (fp32 mode: k_gemm_tn3 on pre-cut bf16 planes incl. the kernel that scales and cuts the inside vectors; fp32 matrix instructions or per-sentence grammars: k_gemm_tn; bf16 mode: transposes + k_gemm_nt16)",
                        "mfma": mfma, "achieved": gg_tflops, "peak": peak, "unit": "TFLOP/s", "frac": gg_tflops / peak,
                        "ms_per_step": gg["ms_per_step"]}
    res["split_reduction"] = {"bound": "hbm", "achieved": split_bytes / (split_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                              "unit": "GB/s", "frac": split_bytes / (split_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                              "ms_per_step": split_ms}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="ptb", choices=["tiny", "small", "ptb", "scaled", "long"])
    ap.add_argument("--precision", default=None, choices=["fp32", "bf16"],
                    help="operand type of the projection GEMMs (default: the workload's own: bf16 for scaled)")
    ap.add_argument("--profile-steps", type=int, default=None,
                    help="steps repeated with HIP events around every kernel launch (default: as many as --steps)")
    ap.add_argument("--cpu-sentences", type=int, default=64,
                    help="sentences of the batch the CPU oracle is timed on (stops after about 25 s)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the short register-only matrix-instruction loop reported under \"mfma_sustained\"")
    ap.add_argument("--frontend", action="store_true",
                    help="also time the rule-probability front-end (softmaxes + emission gather) and its backward "
                         "at the workload's shape; reported under \"frontend\", not part of the step")
    ap.add_argument("--per-sentence", action="store_true",
                    help="one grammar per sentence (grouped projection products) at the workload's shape")
    ap.add_argument("--fp32-mfma", action="store_true",
                    help="fp32 matrix instructions instead of the split-bf16 products (SPCFG_FLAG_FP32_MFMA)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step into a HIP graph once and time its replays instead of eager launches")
    ap.add_argument("--decode", action="store_true",
                    help="also time the span-posterior export and the best-tree decoder on the step's workspace; "
                         "reported under \"decode\", not part of the step")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the extra measurements of the default run (fp32-matrix-instruction variant, other seeds "
                         "of the length law, the other configurations): for profiler runs")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain device copy of known size (1 GiB read + 1 GiB written per launch, 5 "
                         "launches): the reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (sharding over sentences with one all-reduce of the rule "
              "gradients is designed but not built); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2310_14997_amd import binding as bd
    from paper_2310_14997_amd import synth

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "copy", "bytes_read_per_launch": src.numel() * 4,
                          "bytes_written_per_launch": src.numel() * 4, "launches": 5}))
        return

    d = synth.make_inputs_per_sentence(args.workload) if args.per_sentence else synth.make_inputs(args.workload)
    precision = args.precision or d["precision"]
    bf16 = precision == "bf16"
    m = measure(d, bf16, args.fp32_mfma, args.steps, args.warmup, args.profile_steps, graph=args.graph)
    wl, wc, classes = m["wl"], m["wc"], m["classes"]
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get(args.workload + ("_bf16" if bf16 and args.workload != "scaled" else ""),
                                       {}).get("gemm_nt_bytes_per_launch")

    out = {
        # the headline metric's name for the headline workload; `value` is its sentences/s part, the two
        # fractions it also names are `roofline.frac` (MFMA) and `split_reduction.frac` (HBM)
        "metric": f"sentences/sec inside fwd+bwd at N=P={d['N']}, n<={d['n_max']}; % MFMA peak, % HBM peak",
        "value": m["sentences_per_s"], "unit": "sentences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic", "launch": "hip graph replay" if args.graph else "eager",
        "grammars": "one per sentence" if args.per_sentence else "shared",
        "config": {"workload": f"{args.workload}: B={d['B']}, N={d['N']}, P={d['P']}, n_max={d['n_max']}, "
                               f"sum_n={wc['leaves']}, projected_spans={wc['proj_spans']}, "
                               f"split_terms={wc['split_terms']}, seed={d['seed']}",
                   "flop_fwd_bwd": wc["flop_fwd_bwd"], "tflops_fwd_bwd": wc["flop_fwd_bwd"] / (m["ms_per_step"] * 1e-3) / 1e12},
        "roofline": dict(m["roofline"], traffic=traffic),
        "gemm_grad": m["gemm_grad"],
        "split_reduction": m["split_reduction"],
        "kernel_classes": classes,
    }
    if args.workload == "ptb" and not args.headline_only and not (bf16 or args.fp32_mfma or args.per_sentence or args.graph):
        # the same batch on fp32 matrix instructions (SPCFG_FLAG_FP32_MFMA), against that instruction's own peak
        v = measure(d, False, True, 5, 2, 5)
        out["variants"] = {"fp32_mfma": {"ms_per_step": v["ms_per_step"], "sentences_per_s": v["sentences_per_s"],
                                         "roofline": v["roofline"], "gemm_grad": v["gemm_grad"]}}
        del v
        # other draws of the same length law (the headline seed is one draw; its batch is lighter than the mean)
        vals, flops, toks = [], [], []
        for i in range(8):
            di = synth.make_inputs("ptb", seed=d["seed"] + 1000 + i)
            mi = measure(di, False, False, 5, 2, 0)
            vals.append(mi["sentences_per_s"]); flops.append(mi["wc"]["flop_fwd_bwd"]); toks.append(mi["wc"]["leaves"])
            del mi, di
        out["law_mean"] = {"seeds": 8, "sentences_per_s": float(np.mean(vals)), "sentences_per_s_min": float(np.min(vals)),
                           "sentences_per_s_max": float(np.max(vals)), "flop_fwd_bwd": float(np.mean(flops)),
                           "tokens_per_batch": float(np.mean(toks)),
                           "note": "mean over 8 further seeds of the PTB length law, 5 timed steps each"}
        # the other configurations, each in the launch configuration its parity test uses
        out["workloads"] = {}
        for name in ("small", "scaled", "long"):
            dn = synth.make_inputs(name)
            mn = measure(dn, dn["precision"] == "bf16", False, 5, 2, 5)
            out["workloads"][name] = {"dtype": "bf16" if dn["precision"] == "bf16" else "f32",
                                      "ms_per_step": mn["ms_per_step"], "sentences_per_s": mn["sentences_per_s"],
                                      "mfma_frac": mn["roofline"]["frac"], "mfma_peak": mn["roofline"]["peak"],
                                      "projection_tflops": mn["roofline"]["achieved"],
                                      "hbm_frac": mn["split_reduction"]["frac"],
                                      "split_GBps": mn["split_reduction"]["achieved"]}
            del mn
            if name == "scaled":  # the same with single bf16 operands in the forward products as well
                import paper_2310_14997_amd.binding as bd_
                m1 = measure(dn, True, False, 5, 2, 5, extra_flags=bd_.FLAG_BF16_SINGLE_FORWARD)
                out["workloads"]["scaled_single_bf16_forward"] = {
                    "dtype": "bf16", "ms_per_step": m1["ms_per_step"], "sentences_per_s": m1["sentences_per_s"],
                    "mfma_frac": m1["roofline"]["frac"], "mfma_peak": m1["roofline"]["peak"],
                    "projection_tflops": m1["roofline"]["achieved"], "hbm_frac": m1["split_reduction"]["frac"],
                    "split_GBps": m1["split_reduction"]["achieved"]}
                del m1
            del dn
    if args.frontend:
        out["frontend"] = time_frontend(args.workload, wl, args.steps)
    if args.decode:
        out["decode"] = time_decode(wl, args.steps)
    if args.workload == "ptb" and not args.no_mfma_probe:
        out["mfma_sustained"] = mfma_sustained()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(d, args.cpu_sentences)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
