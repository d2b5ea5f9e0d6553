"""Writes tests/golden/tiny_oracle.json from the CPU oracle alone (never from the HIP path).

The paper prints no worked example of the attention forward, so this file is not a pin of
the oracle: it is a drift guard, so that an unintended change of the oracle's arithmetic or of
the seeded input generator shows up as a failing test.  Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import lot_oracle  # noqa: E402
from paper_2509_23436_amd import synth  # noqa: E402


def compute():
    w = synth.WORKLOADS["tiny"]
    x = synth.make_inputs(w)
    O, g1, g2, _ = lot_oracle.attention(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters,
                                        want_couplings=True)
    tok1, piv1, tok2, piv2 = lot_oracle.marginal_residuals(g1, g2, x["beta"])
    return {
        "workload": "tiny (B=1,H=1,n=64,d=32,r=8,f32 inputs,eps=0.1,T=20,seed=0)",
        "source": "oracle/lot_oracle.c via tests/golden/make_golden.py",
        "Q_first": [float(v) for v in x["Q"].ravel()[:4]],
        "beta": [float(v) for v in x["beta"].ravel()],
        "O_first_row": [float(v) for v in O[0, 0, 0, :8]],
        "O_sum": float(O.sum()),
        "O_abs_sum": float(np.abs(O).sum()),
        "tok1_max": float(np.abs(tok1).max()),
        "tok2_max": float(np.abs(tok2).max()),
        "gamma1_00": float(g1[0, 0, 0, 0]),
        "gamma2_00": float(g2[0, 0, 0, 0]),
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.json")
    with open(out, "w") as fh:
        json.dump(compute(), fh, indent=1)
    print("wrote", out)
