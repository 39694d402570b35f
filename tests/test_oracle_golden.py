"""The oracle reproduces its stored c1 outputs (regression guard; written by tests/golden/make_c1_golden.py)."""
import json
import os

import numpy as np

import oracle
from paper_2510_07651_amd import synth


def test_c1_golden():
    with open(os.path.join(os.path.dirname(__file__), "golden", "c1_expected.json")) as f:
        gold = json.load(f)
    wl = synth.config("c1")
    x = synth.make_inputs(wl)
    scores = oracle.score(x["q"], x["k"], x["v"])
    for name, s in zip(synth.VARIANTS, scores):
        np.testing.assert_allclose(s[0, 0, gold["positions"]], gold[name]["scores_at_positions"], rtol=1e-9)
        keep = oracle.select(s.astype(np.float32), wl.budget)
        assert keep[0, 0].tolist() == gold[name]["keep_idx"]
    # token 0 is the planted sink (key = 3 x mean window query): it must be kept by all variants
    for name in synth.VARIANTS:
        assert 0 in gold[name]["keep_idx"]
