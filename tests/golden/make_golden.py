"""Writes tests/golden/oracle_small_cases.txt.

The paper prints no worked numeric example, so the stored values are the fp64
oracle's own (it calls nothing else), kept as a guard against an unnoticed
change of the oracle's arithmetic.  Run from the repository root:
    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import flurka_oracle as fo  # noqa: E402
from paper_2306_15799_amd import inputs  # noqa: E402

CASES = [
    ("performer_f32", inputs.Workload("g1", 1, 2, 48, 8, 6, 10, "f32", inputs.PHI_PERFORMER, True)),
    ("elu1_bf16", inputs.Workload("g2", 2, 1, 40, 8, 5, 8, "bf16", inputs.PHI_ELU1, True)),
]
ROWS = [0, 7, 39]


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_cases.txt")
    with open(path, "w") as f:
        f.write("# case, tensor, flat values (fp64 repr); inputs: make_inputs(workload, seed=3)\n")
        for name, w in CASES:
            t = inputs.make_inputs(w, seed=3)
            out = fo.flurka_attention(t["Q"], t["K"], t["V"], t["E"], t["F"], t["omega"], w.phi)
            g = fo.flurka_attention_bwd(t["Q"], t["K"], t["V"], t["E"], t["F"], t["omega"], t["dOut"], w.phi)
            rec = {"out": out[:, :, ROWS], "dQ": g[0][:, :, ROWS], "dK": g[1][:, :, ROWS],
                   "dV": g[2][:, :, ROWS], "dE": g[3][:, ROWS], "dF": g[4][:, ROWS]}
            for key, val in rec.items():
                f.write(f"{name} {key} " + " ".join(repr(float(v)) for v in np.ravel(val)) + "\n")


if __name__ == "__main__":
    main()
