"""Writes tests/golden/mlp_cfg1_oracle.json from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden_mlp.py
The stored values come from oracle/ and the seeded input generator only; no
GPU code is involved.  The paper prints no numeric worked example for the MLP
block, so these are regression anchors (generator and oracle did not drift),
not paper values.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import mst_inputs as mi  # noqa: E402
from oracle import mlp_oracle as orc  # noqa: E402


def main():
    inp = mi.make_mlp_inputs(1)
    r = orc.mlp(inp.f64("X"), inp.f64("Wg"), inp.f64("Wu"), inp.f64("Wd"), inp.f64("dO"))
    rng = np.random.default_rng(2)
    samples = {}
    for k in ("O", "dX", "dWg", "dWu", "dWd"):
        a = r[k]
        samples[k] = [(int(i), int(j), float(a[i, j])) for i, j in
                      zip(rng.integers(0, a.shape[0], 6), rng.integers(0, a.shape[1], 6))]
    gold = dict(
        source="oracle/mlp_oracle.py:mlp on mst_inputs.make_mlp_inputs(1)",
        samples=samples,
        frobenius={k: float(np.sqrt((r[k] ** 2).sum())) for k in r},
        bits_sum={n: int(getattr(inp, n + "_bits").astype(np.uint64).sum()) for n in ("X", "Wg", "Wu", "Wd", "dO")},
    )
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "mlp_cfg1_oracle.json"), "w") as f:
        json.dump(gold, f, indent=1)
    print("wrote mlp_cfg1_oracle.json")


if __name__ == "__main__":
    main()
