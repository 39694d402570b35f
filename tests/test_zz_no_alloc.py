"""The entry point that allocates nothing (obc_score_static) against the entry points it is a variant of.

Through the C ABI: two calls in a row on the library's static scratch, the second on a smaller input, each compared
with obc_score / obc_score_accumulate on a caller-provided workspace (same kernels, so the bits must agree), and with
the oracle on the small case.  A shape beyond the scratch is refused before anything is launched.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2510_07651_amd import binding as obc
from paper_2510_07651_amd import synth

from parity_util import TOL, score_error, to_device

pytestmark = pytest.mark.gpu


def _inputs(name):
    wl = {w.name.split("_")[0] if w.name[0] == "c" else w.name: w for w in synth.small_cases() + synth.paper_configs()[:2]}[name]
    x = synth.make_inputs(wl)
    return wl, x, to_device(x)


def test_static_scratch_matches_workspace_calls_twice_in_a_row():
    obc.obc_init()
    big_wl, big_x, big = _inputs("c2")                  # 8 KV heads x 8192 tokens: several splits and ranges
    small_wl, small_x, small = _inputs("s_bf16_ragged")  # smaller, ragged: the scratch still holds the first call's data
    for variant in ("joint", "all"):
        for wl, x, dev in ((big_wl, big_x, big), (small_wl, small_x, small)):
            lens = x["seq_lens"]
            want = obc.obc_score(dev["q"], dev["k"], dev["v"], variant, seq_lens=lens)
            got = torch.full_like(want, -7.0)
            obc.obc_score_static(dev["q"], dev["k"], dev["v"], variant, got, seq_lens=lens)
            torch.cuda.synchronize()
            assert torch.equal(got, want), (wl.name, variant)
            # accumulate form: adds to what the tensor holds, padding untouched
            run_a = torch.full_like(want, 1.5)
            run_b = run_a.clone()
            obc.obc_score(dev["q"], dev["k"], dev["v"], variant, seq_lens=lens, scores=run_a, accumulate=True)
            obc.obc_score_static(dev["q"], dev["k"], dev["v"], variant, run_b, seq_lens=lens, accumulate=True)
            torch.cuda.synchronize()
            assert torch.equal(run_a, run_b), (wl.name, variant)
    # and against the oracle on the small case
    ref = oracle.score(small_x["q"], small_x["k"], small_x["v"], seq_lens=small_x["seq_lens"])
    got = torch.empty((3, small_wl.B, small_wl.Hkv, small_wl.N), dtype=torch.float32, device="cuda")
    obc.obc_score_static(small["q"], small["k"], small["v"], "all", got, seq_lens=small_x["seq_lens"])
    for vi in range(3):
        err, where = score_error(got[vi].cpu().numpy(), ref[vi], small_wl.budget, small_x["seq_lens"], TOL["bf16"])
        assert err <= TOL["bf16"], (vi, err, where)


def test_static_scratch_serves_decode_steps_and_the_plain_path():
    """A one-row window on a short cache (decode kernels) and an fp32 case (plain kernels) use the same scratch."""
    for name in ("s_bf16_w1", "c1"):
        wl, x, dev = _inputs(name)
        want = obc.obc_score(dev["q"], dev["k"], dev["v"], "all", seq_lens=x["seq_lens"])
        got = torch.empty_like(want)
        obc.obc_score_static(dev["q"], dev["k"], dev["v"], "all", got, seq_lens=x["seq_lens"])
        torch.cuda.synchronize()
        assert torch.equal(got, want), name


def test_static_scratch_refuses_shapes_beyond_its_size():
    B, Hq, Hkv, d, N, W = 1, 28, 4, 128, 131072, 64      # needs ~54 MiB of workspace: more than the static scratch
    assert obc.obc_score_workspace_bytes(B, N, W, Hq, Hkv, d, obc.OBC_BF16, obc.OBC_ALL) > obc.OBC_STATIC_SCRATCH_BYTES
    q = torch.zeros(B, Hq, W, d, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(B, Hkv, N, d, dtype=torch.bfloat16, device="cuda")
    scores = torch.full((3, B, Hkv, N), 3.0, dtype=torch.float32, device="cuda")
    with pytest.raises(obc.ObcError) as e:
        obc.obc_score_static(q, k, k, "all", scores)
    assert e.value.status == obc.OBC_EWORKSPACE
    torch.cuda.synchronize()
    assert torch.all(scores == 3.0)                      # nothing ran
    lib = obc.load_library()
    assert lib.obc_score_static(q.data_ptr(), k.data_ptr(), k.data_ptr(), N, W, Hq, Hkv, d, obc.OBC_ALL,
                                scores.data_ptr(), B, obc.OBC_BF16, None, 2, None) == obc.OBC_EINVAL   # accumulate flag
