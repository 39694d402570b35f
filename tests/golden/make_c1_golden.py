"""Writes tests/golden/c1_expected.json from the CPU oracle only (never from the GPU path).

Config c1 (single head, d=64, N=512, W=16, fp32, seed 0): the 128 kept indices per
score variant and the scores at 16 fixed positions.  The paper (arxiv 2510.07651)
prints no numeric example, so these are oracle outputs stored as a regression guard;
the pins in tests/test_oracle_pins.py are what tie the oracle to the paper.
Run:  python tests/golden/make_c1_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2510_07651_amd import synth  # noqa: E402


def main():
    wl = synth.config("c1")
    x = synth.make_inputs(wl)
    scores = oracle.score(x["q"], x["k"], x["v"])
    pos = [0, 1, 2, 3, 17, 64, 100, 255, 256, 300, 400, 495, 496, 500, 510, 511]
    out = {"workload": wl.name, "positions": pos}
    for name, s in zip(synth.VARIANTS, scores):
        keep = oracle.select(s.astype(np.float32), wl.budget)
        out[name] = {"scores_at_positions": [float(s[0, 0, p]) for p in pos],
                     "keep_idx": [int(i) for i in keep[0, 0]]}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_expected.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
