"""Tolerances and comparison helpers for the GPU-vs-oracle parity tests.

fp32 path: log Z within 1e-5 relative; every gradient tensor within 1e-4 relative, read per tensor as
|x - y| <= 1e-4 |y| + 1e-4 mean|y| elementwise and a relative L2 error <= 1e-4.
"""
import numpy as np

LOGZ_RTOL_FP32 = 1e-5
GRAD_RTOL_FP32 = 1e-4


def check_logZ(got, ref, rtol=LOGZ_RTOL_FP32):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    fin = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), fin), f"finite pattern differs: {got} vs {ref}"
    assert np.all(got[~fin] == ref[~fin])
    err = np.abs(got[fin] - ref[fin])
    tol = rtol * np.abs(ref[fin])
    assert np.all(err <= tol), f"logZ max rel err {np.max(err / np.abs(ref[fin])):.3e} (tol {rtol})\n{got}\n{ref}"
    return float(np.max(err / np.abs(ref[fin]))) if fin.any() else 0.0


def check_grad(name, got, ref, rtol=GRAD_RTOL_FP32):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.all(np.isfinite(got)), f"{name}: non-finite entries"
    scale = np.mean(np.abs(ref))
    err = np.abs(got - ref)
    tol = rtol * np.abs(ref) + rtol * scale
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    l2 = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    assert np.all(err <= tol), (f"{name}: elementwise tolerance exceeded at {worst}: got {got[worst]:.8e} ref "
                                f"{ref[worst]:.8e} (mean|ref| {scale:.3e}, rel L2 {l2:.3e})")
    assert l2 <= rtol, f"{name}: relative L2 error {l2:.3e} > {rtol}"
    return float(l2)


def check_all(got, ref, logz_rtol=LOGZ_RTOL_FP32, grad_rtol=GRAD_RTOL_FP32):
    stats = {"logZ": check_logZ(got["logZ"], ref["logZ"], logz_rtol)}
    for k in ("grad_log_root", "grad_log_emit", "grad_L", "grad_R"):
        stats[k] = check_grad(k, got[k], ref[k], grad_rtol)
    return stats


def oracle_batch_parallel(d, grad_logZ=None, workers=4, sentences=None, timeout=900):
    """oracle.spcfg_oracle.inside_backward over a whole batch (or the listed sentences), the sentences dealt to a
    few worker processes (tests/oracle_worker.py: fresh interpreters that import numpy and the oracle only and
    never touch the GPU; inputs and results travel as .npz files in a temporary directory).
    Same result layout as the oracle's batched call; sentences that were not asked for keep NaN in logZ."""
    import os
    import subprocess
    import sys
    import tempfile
    lengths = np.asarray(d["lengths"])
    B, n_max, P = d["log_emit"].shape
    N = d["L"].shape[0]
    todo = list(range(B)) if sentences is None else list(sentences)
    # longest first, dealt round-robin: the cost of a sentence grows with the cube of its length
    order = sorted(todo, key=lambda b: -int(lengths[b]))
    chunks = [order[w::workers] for w in range(workers) if order[w::workers]]
    out = dict(logZ=np.full(B, np.nan), grad_L=np.zeros((N, N + P)), grad_R=np.zeros((N, N + P)),
               grad_log_root=np.zeros(N), grad_log_emit=np.zeros((B, n_max, P)))
    here = os.path.dirname(os.path.abspath(__file__))
    with tempfile.TemporaryDirectory() as tmp:
        inp = os.path.join(tmp, "in.npz")
        np.savez(inp, log_root=d["log_root"], L=d["L"], R=d["R"], log_emit=d["log_emit"], lengths=lengths,
                 grad_logZ=np.ones(B) if grad_logZ is None else np.asarray(grad_logZ, np.float64))
        procs = []
        # the workers share the host's cores: left at the default, every worker's BLAS would start a thread per core
        threads = str(max(1, min(os.cpu_count() or 1, 16) // len(chunks)))
        env = dict(os.environ, OMP_NUM_THREADS=threads, OPENBLAS_NUM_THREADS=threads, MKL_NUM_THREADS=threads)
        for w, c in enumerate(chunks):
            outp = os.path.join(tmp, f"out{w}.npz")
            cmd = [sys.executable, os.path.join(here, "oracle_worker.py"), inp, outp] + [str(b) for b in c]
            procs.append((subprocess.Popen(cmd, env=env), outp, c))
        for proc, outp, c in procs:
            rc = proc.wait(timeout=timeout)
            assert rc == 0, f"oracle worker failed with exit code {rc}"
            with np.load(outp) as res:
                for t, b in enumerate(c):
                    n = int(lengths[b])
                    out["logZ"][b] = res["logZ"][t]
                    out["grad_log_emit"][b, :n] = res[f"ge{t}"]
                out["grad_L"] += res["grad_L"]
                out["grad_R"] += res["grad_R"]
                out["grad_log_root"] += res["grad_log_root"]
    return out
