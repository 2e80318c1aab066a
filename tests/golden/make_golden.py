"""Writes tests/golden/cfg1_oracle.json from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden.py
The stored values come from oracle/ and the seeded input generator only; no
GPU code is involved.  The paper prints no numeric worked example for the LM
head, so these are regression anchors, not paper values.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import mst_inputs as mi  # noqa: E402
from oracle import lmhead_ce_oracle as orc  # noqa: E402


def main():
    inp = mi.make_inputs(1)
    r = orc.lmhead_ce(inp.H_f64(), inp.W_f64(), inp.labels)
    rng = np.random.default_rng(1)
    dH_s = [(int(s), int(k), float(r["dH"][s, k])) for s, k in
            zip(rng.integers(0, inp.cfg.S, 8), rng.integers(0, inp.cfg.d, 8))]
    dW_s = [(int(v), int(k), float(r["dW"][v, k])) for v, k in
            zip(rng.integers(0, inp.cfg.V, 8), rng.integers(0, inp.cfg.d, 8))]
    gold = dict(
        source="oracle/lmhead_ce_oracle.py:lmhead_ce on mst_inputs.make_inputs(1)",
        n_valid=r["n_valid"], loss=r["loss"], dH_samples=dH_s, dW_samples=dW_s,
        H_bits_sum=int(inp.H_bits.astype(np.uint64).sum()),
        W_bits_sum=int(inp.W_bits.astype(np.uint64).sum()),
        labels_sum=int(inp.labels.astype(np.int64).sum()),
    )
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_oracle.json"), "w") as f:
        json.dump(gold, f, indent=1)
    print("wrote cfg1_oracle.json: loss", r["loss"])


if __name__ == "__main__":
    main()
