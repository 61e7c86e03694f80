"""The library driven by a plain C program (no Python binding, no PyTorch): `paper_2310_14997_amd/abi_client.bin`,
built from csrc/abi_client.c with gcc, reads a batch from a file, calls spcfg_inside_forward_backward through the
C ABI and writes the results, which are compared with the oracle."""
import os
import subprocess

import numpy as np
import pytest

from oracle import spcfg_oracle as O
from paper_2310_14997_amd import synth
from parity_util import check_all

pytestmark = pytest.mark.gpu

CLIENT = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2310_14997_amd",
                      "abi_client.bin")


def test_c_program_through_the_abi(tmp_path):
    assert os.path.exists(CLIENT), "abi_client.bin is missing: run paper_2310_14997_amd/build.py"
    d = synth.make_inputs("tiny", N=70, P=45, B=5, lengths=[2, 9, 17, 5, 12])
    N, P, B, n_max = d["N"], d["P"], d["B"], d["n_max"]
    inp, out = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(inp, "wb") as f:
        np.array([N, P, B, n_max], dtype=np.int32).tofile(f)
        d["lengths"].astype(np.int32).tofile(f)
        for k in ("log_root", "L", "R", "log_emit"):
            np.ascontiguousarray(d[k], dtype=np.float32).tofile(f)
    print("case C client", flush=True)
    res = subprocess.run([CLIENT, str(inp), str(out)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    raw = np.fromfile(out, dtype=np.float32).astype(np.float64)
    M = N + P
    sizes = [("logZ", (B,)), ("grad_L", (N, M)), ("grad_R", (N, M)), ("grad_log_root", (N,)),
             ("grad_log_emit", (B, n_max, P))]
    got, at = {}, 0
    for name, shape in sizes:
        cnt = int(np.prod(shape))
        got[name] = raw[at:at + cnt].reshape(shape)
        at += cnt
    assert at == raw.size
    check_all(got, O.inside_backward(d["log_root"], d["L"], d["R"], d["log_emit"], d["lengths"]))
