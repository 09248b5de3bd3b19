"""Writes oracle_cfg1_digest.txt from the CPU oracle alone (never from the HIP path)."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import lstm_oracle as O  # noqa: E402
from paper_1604_01946_amd.inputs import CONFIGS, make_inputs  # noqa: E402


def digest():
    cfg = CONFIGS["cfg1"]
    d = make_inputs(cfg, 0)
    y, hT, cT, res = O.lstm_forward(*cfg.dims, d["x"], d["h0"], d["c0"], d["W"], d["R"], d["b"])
    g = O.lstm_backward(*cfg.dims, d["x"], d["h0"], d["c0"], d["W"], d["R"], res, d["dy"], d["dhT"], d["dcT"])
    out = {}
    for name, arr in zip(("y", "hT", "cT", "dx", "dh0", "dc0", "dW", "dR", "db"), (y, hT, cT) + tuple(g)):
        a = np.asarray(arr, np.float64).reshape(-1)
        w = np.cos(np.arange(a.size) * 0.37)  # position-sensitive weights
        out[name] = (float(a.sum()), float(np.abs(a).max()), float((a * w).sum()))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_cfg1_digest.txt")
    with open(path, "w") as f:
        f.write("# name sum maxabs cos-weighted-sum  (CPU oracle, config 1, seed 0; Section 2 equations)\n")
        for k, v in digest().items():
            f.write(f"{k} {v[0]:.15e} {v[1]:.15e} {v[2]:.15e}\n")
    print("wrote", path)
