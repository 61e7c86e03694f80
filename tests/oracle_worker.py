"""Worker process of parity_util.oracle_batch_parallel: the CPU oracle over some sentences of a batch.

usage: oracle_worker.py IN.npz OUT.npz SENTENCE...   (imports numpy and the oracle only; never touches a GPU)
Parameter gradients are summed over the listed sentences; log Z and the emission gradients are kept per sentence.
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from oracle import spcfg_oracle as O  # noqa: E402


def main(argv):
    inp, outp, idx = argv[1], argv[2], [int(x) for x in argv[3:]]
    with np.load(inp) as z:
        log_root, L, R, log_emit, lengths, g = (z[k] for k in ("log_root", "L", "R", "log_emit", "lengths", "grad_logZ"))
    N, M = L.shape
    res = dict(logZ=np.zeros(len(idx)), grad_L=np.zeros((N, M)), grad_R=np.zeros((N, M)), grad_log_root=np.zeros(N))
    for t, b in enumerate(idx):
        n = int(lengths[b])
        lz, gL, gR, gr, ge = O.inside_backward_sentence(log_root, L, R, log_emit[b, :n], float(g[b]))
        res["logZ"][t] = lz
        res[f"ge{t}"] = ge
        res["grad_L"] += gL
        res["grad_R"] += gR
        res["grad_log_root"] += gr
    np.savez(outp, **res)


if __name__ == "__main__":
    main(sys.argv)
