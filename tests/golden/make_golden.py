"""Writes tests/golden/tiny_oracle.json from the CPU oracle alone (never from the HIP path).

The paper prints no worked example, so this fixture is not a value from the paper: it freezes what the
pinned oracle returns on the seeded Tiny workload (Sec. 3.1 recursion, B=4, n=10, N=30, P=60), so that a
later change to the oracle's arithmetic shows up as a diff.  Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import spcfg_oracle as O  # noqa: E402
from paper_2310_14997_amd import synth  # noqa: E402


def main():
    d = synth.make_inputs("tiny")
    out = O.inside_backward(d["log_root"], d["L"], d["R"], d["log_emit"], d["lengths"])
    fix = dict(
        source="oracle/spcfg_oracle.py on synth.make_inputs('tiny'); inside recursion of Sec. 3.1, root rule of Sec. 2",
        seed=d["seed"], logZ=[float(x) for x in out["logZ"]],
        grad_log_root=[float(x) for x in out["grad_log_root"]],
        grad_L_row0_first8=[float(x) for x in out["grad_L"][0, :8]],
        grad_R_col_sums_first8=[float(x) for x in out["grad_R"].sum(axis=0)[:8]],
        grad_log_emit_b0_i0_first8=[float(x) for x in out["grad_log_emit"][0, 0, :8]],
        expected_left_rule_count=float((d["L"].astype(np.float64) * out["grad_L"]).sum()),
    )
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.json")
    with open(path, "w") as f:
        json.dump(fix, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
