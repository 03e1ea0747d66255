"""Writes tests/golden/oracle_tiny.json: the oracle's own outputs on a tiny seeded layer.

The paper prints no worked numeric example of a score, an index set or a compressed cache,
so there is no paper-given value to store.  This file only freezes the *oracle's* arithmetic
(a regression guard: a later edit that changes its numbers must be deliberate).  It calls
nothing but oracle/ and the input generator.   Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from ea_inputs import CONFIGS, make_layer, widen  # noqa: E402
from oracle import ea_oracle as O                  # noqa: E402


def build():
    cfg = CONFIGS["c1"].with_(head_dim=8)
    lay = make_layer(cfg, n=32, window=8, pos0=5000)
    res = O.compress_layer(widen(lay["q_win"]), widen(lay["k"]), widen(lay["v"]), lay["q_pos0"],
                           lay["inv_freq"], lay["t_next"], 16, T=512, epsilon=0.02)
    return {
        "recipe": "CONFIGS['c1'].with_(head_dim=8); make_layer(n=32, window=8, pos0=5000); "
                  "n_keep=16, T=512, eps=0.02, ddof=0, half-split",
        "mu": res["mu"].tolist(),
        "sigma_diag": np.diagonal(res["sigma"], axis1=-2, axis2=-1).tolist(),
        "sigma_fro": np.linalg.norm(res["sigma"], axis=(-2, -1)).tolist(),
        "scores": res["scores"].tolist(),
        "idx": res["idx"].tolist(),
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_tiny.json")
    with open(out, "w") as f:
        json.dump(build(), f, indent=1)
    print("wrote", out)
