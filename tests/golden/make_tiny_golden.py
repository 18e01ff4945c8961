"""Writes tests/golden/tiny_oracle.json: summary values of the fp64 oracle on the tiny
configuration (depth 4, width 64, batch 32, leaky slope 0.1, seed 0).

The values come from the oracle alone (oracle/ + the seeded generator); nothing here touches
the GPU library. The paper prints no worked numeric example for dense layers, so this file
pins the oracle and the generator against silent drift, while the mathematics is pinned in
tests/test_oracle_pins.py.

Run from the repository root:  python tests/golden/make_tiny_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import moonwalk_oracle as O      # noqa: E402
from workloads import make_config            # noqa: E402


def main():
    wl = make_config("tiny")
    bp = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    out = {
        "config": "tiny: L=4, d=64, B=32, alpha=0.1, seed=0",
        "loss": bp["loss"],
        "dW_fro": [float(np.linalg.norm(g)) for g in bp["dW"]],
        "db_fro": [float(np.linalg.norm(g)) for g in bp["db"]],
        "h0_fro": float(np.linalg.norm(bp["h"][0])),
        "mask_popcount": [int(m.sum()) for m in bp["masks"]],
        "mask_word0_hex": [format(int(O.pack_mask(m)[0]), "016x") for m in bp["masks"]],
        "W1_first_row_head": [float(v) for v in wl.W[0][0, :4]],
        "x_head": [float(v) for v in wl.x[0, :4]],
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
