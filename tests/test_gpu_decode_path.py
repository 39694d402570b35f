"""GPU parity of the decode-time scoring path (a window of one query row per head) against the fp64 oracle.

Section 3.2 / Appendix C: while decoding the scores of each new query row are accumulated onto the running
ones.  The library serves W = 1 on bf16 caches with kernels of their own; these cases cover their tiling
(1, 2, 4 and 8 query heads per KV head incl. a padded 7, both head dims, ranges merged inside the scoring kernel
and by the separate merge kernel with one and with several ranges per merging thread, ragged lengths down to one
token) and the cancellation guard for a row whose
attention sits on one key.  Tolerance: 1e-3 relative as everywhere for bf16 inputs.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_07651_amd import binding as obc
from paper_2510_07651_amd import synth

from parity_util import TOL, run_case, score_error, to_device

pytestmark = pytest.mark.gpu

W1 = dict(W=1, dtype="bf16")
CASES = {w.name: w for w in [
    synth.Workload("d_llama_1025", B=2, Hq=8, Hkv=2, d=128, N=1025, budget=100, seed=51, sinks=4, outlier_channels=4, **W1),
    synth.Workload("d_qwen_g7", B=1, Hq=14, Hkv=2, d=128, N=777, budget=64, seed=52, sinks=4, outlier_channels=4, **W1),
    synth.Workload("d_mha_d64", B=2, Hq=3, Hkv=3, d=64, N=300, budget=30, seed=53, sinks=1, **W1),
    synth.Workload("d_g2_ragged", B=5, Hq=4, Hkv=2, d=128, N=2000, budget=1, seed=54, sinks=1, ragged=(1, 2000),
                   pad_nan=True, **W1),
    synth.Workload("d_g3", B=2, Hq=6, Hkv=2, d=128, N=400, budget=40, seed=62, sinks=1, ragged=(100, 400), **W1),
    synth.Workload("d_g5_d64", B=1, Hq=10, Hkv=2, d=64, N=700, budget=70, seed=63, sinks=2, outlier_channels=2, **W1),
    synth.Workload("d_g6", B=1, Hq=12, Hkv=2, d=128, N=130, budget=13, seed=64, sinks=1, **W1),
    synth.Workload("d_g8_d64", B=1, Hq=8, Hkv=1, d=64, N=500, budget=50, seed=55, sinks=2, **W1),
    synth.Workload("d_long_separate_merge", B=2, Hq=8, Hkv=2, d=128, N=9000, budget=500, seed=56, sinks=4,
                   outlier_channels=4, ragged=(3000, 9000), pad_nan=True, **W1),
    synth.Workload("d_one_key_takes_all", B=1, Hq=8, Hkv=2, d=128, N=1200, budget=100, seed=57, sinks=1, sink_gain=1.0,
                   shared_query=1.0, **W1),
    synth.Workload("d_one_key_takes_all_harder", B=1, Hq=8, Hkv=2, d=128, N=1200, budget=100, seed=60, sinks=1,
                   sink_gain=1.5, shared_query=1.0, **W1),
    synth.Workload("d_many_ranges", B=1, Hq=2, Hkv=1, d=128, N=133000, budget=2000, seed=61, sinks=4, outlier_channels=4,
                   needles=8, **W1),
    synth.Workload("d_three_tokens", B=2, Hq=4, Hkv=1, d=128, N=3, budget=2, seed=58, **W1),
    synth.Workload("d_one_token", B=1, Hq=4, Hkv=2, d=128, N=1, budget=1, seed=59, **W1),
]}


@pytest.mark.parametrize("name", list(CASES))
def test_decode_scores_select_compact_match_oracle(name, score_path):
    score_path("decode")      # whatever the size (long caches go to the matrix cores otherwise)
    worst = run_case(CASES[name])
    print(name, {k: "%.2e" % v for k, v in worst.items()})


def test_attention_mass_of_the_dominant_case():
    """The guard case is only a test of the guard if one key really takes almost all of some row's attention."""
    x = synth.make_inputs(CASES["d_one_key_takes_all"])
    _, A, _ = oracle.window_attention(x["q"], x["k"], x["v"])
    top = A.max(axis=-1)
    assert top.min() > 0.98 and top.max() > 0.999 and top.max() < 1.0


@pytest.mark.parametrize("name", ["d_llama_1025", "d_qwen_g7", "d_g2_ragged", "d_long_separate_merge", "d_mha_d64"])
def test_decode_attention_only_and_vatp_match_oracle(name, score_path):
    score_path("decode")
    wl = CASES[name]
    x = synth.make_inputs(wl)
    dev = to_device(x)
    lens = x["seq_lens"]
    for variant, ref in (("attn", oracle.attn_score(x["q"], x["k"], x["v"], seq_lens=lens)),
                         ("vatp", oracle.vatp_score(x["q"], x["k"], x["v"], seq_lens=lens))):
        g = obc.obc_score(dev["q"], dev["k"], dev["v"], variant, seq_lens=lens).cpu().numpy()
        assert np.isfinite(g).all() and (g >= 0).all()
        err, where = score_error(g, ref, wl.budget, lens, TOL["bf16"])
        assert err <= TOL["bf16"], "%s %s: err %.3g at %s" % (name, variant, err, where)


@pytest.mark.parametrize("name", ["d_llama_1025", "d_long_separate_merge"])
def test_decode_accumulate_adds_and_leaves_padding_alone(name, score_path):
    score_path("decode")
    wl = CASES[name]
    x = synth.make_inputs(wl)
    dev = to_device(x)
    lens = x["seq_lens"]
    for variant in ("all", "joint", "attn"):
        inc = obc.obc_score(dev["q"], dev["k"], dev["v"], variant, seq_lens=lens)
        run = torch.full_like(inc, 2.5)
        obc.obc_score(dev["q"], dev["k"], dev["v"], variant, seq_lens=lens, scores=run, accumulate=True)
        for b in range(wl.B):
            L = wl.N if lens is None else lens[b]
            assert torch.equal(run[..., b, :, :L], inc[..., b, :, :L] + 2.5), variant
            assert torch.all(run[..., b, :, L:] == 2.5), variant
        again = obc.obc_score(dev["q"], dev["k"], dev["v"], variant, seq_lens=lens)
        assert torch.equal(again, inc), "decode scoring must be bit-reproducible"


def test_matrix_core_path_still_serves_one_row_windows(score_path):
    """The matrix-core pin keeps W = 1 on the matrix-core kernels; both paths must meet the oracle."""
    score_path("mfma")
    run_case(CASES["d_llama_1025"])
    run_case(CASES["d_one_key_takes_all"])
    run_case(CASES["d_one_key_takes_all_harder"])


def test_long_caches_take_the_matrix_core_path_by_default():
    """Past the measured crossover a one-row window goes to the matrix-core kernels; both routes meet the oracle."""
    run_case(CASES["d_many_ranges"])
