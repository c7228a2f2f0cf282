"""Writes the stored expected values under tests/golden/ by calling ONLY the CPU oracle.

Run from the repository root:  python tests/golden/make_golden.py

tiny_trajectory.json: the "tiny" workload (n=256, T=2048, fp32 X ~ N(0,1) with 4 seeded
channels x50, Gaussian Z0, 10 steps of Alg. 1 with lr 1e-2, token-mean Whip): the loss of
every step, the Frobenius norm of the final latent and a few sampled entries of the final
rotation, all from the fp64 oracle.  The paper prints no worked numeric example, so these
values are the oracle's (itself pinned in tests/test_oracle_pins.py), not the paper's.
"""

import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import dartqr_oracle as orc  # noqa: E402
from paper_2511_04063_amd import synth  # noqa: E402


def main():
    inp = synth.make_inputs("tiny")
    cfg = inp["cfg"]
    X = inp["X"][0].astype(np.float64)
    Z0 = inp["Z0"][0].astype(np.float64)
    losses, Zf, Rf = orc.calibrate(X, Z0, cfg.steps, cfg.lr, "mean")
    idx = [(0, 0), (1, 7), (100, 200), (255, 255), (128, 3), (17, 254)]
    out = {
        "config": "tiny",
        "n": cfg.n, "T": cfg.T, "steps": cfg.steps, "lr": cfg.lr, "reduce": "mean",
        "losses": [float(v) for v in losses],
        "Z_final_fro": float(np.linalg.norm(Zf)),
        "R_final_samples": [{"i": i, "j": j, "value": float(Rf[i, j])} for i, j in idx],
        "source": "oracle/dartqr_oracle.py (fp64), written by tests/golden/make_golden.py",
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_trajectory.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path, "losses", out["losses"])


if __name__ == "__main__":
    main()
