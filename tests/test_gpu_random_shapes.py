"""GPU parity on randomly drawn (but seeded) shapes: a sweep over the corners that hand-picked cases miss.

Every draw stays inside the documented limits of the C ABI (W <= 64, G*W <= 512, W <= len_b <= N, budget <= len_b);
the comparison is the one of test_gpu_parity_small: scores within the dtype's tolerance of the fp64 oracle, kept
indices bit-exact given the same fp32 scores.  The budget of every draw is one eighth of the shortest sequence (the
regime of the paper's 10-40 % budgets): the comparison floor is tied to the budget-th largest score, and a tiny budget
would lift that floor to the scale of a head's top scores.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_07651_amd import binding as obc
from paper_2510_07651_amd import synth

from parity_util import TOL, score_error, to_device

pytestmark = pytest.mark.gpu


def _draw(seed, decode=False):
    rng = np.random.default_rng((5000 if decode else 1000) + seed)
    G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8] if decode else [1, 2, 3, 4, 7, 8]))
    Hkv = int(rng.integers(1, 4))
    W = 1 if decode else int(rng.integers(1, min(64, 512 // G) + 1))
    dtype, d = [("bf16", 128), ("bf16", 128), ("bf16", 128), ("bf16", 64), ("fp32", 64), ("fp32", 128)][int(rng.integers(0, 6))]
    N = int(rng.integers(W, 2600))
    B = int(rng.integers(1, 4))
    ragged = (int(rng.integers(W, N + 1)), N) if rng.random() < 0.5 else None
    min_len = ragged[0] if ragged else N
    sinks = int(rng.integers(0, min(5, min_len - W + 1))) if min_len > W else 0
    room = min_len - W - sinks
    needles = int(rng.integers(0, min(6, room) + 1)) if room > 8 and rng.random() < 0.4 else 0
    return synth.Workload("rnd%d" % seed, B=B, Hq=G * Hkv, Hkv=Hkv, d=d, N=N, W=W, dtype=dtype,
                          budget=max(1, min_len // 8), seed=7000 + seed, sinks=sinks,
                          outlier_channels=int(rng.integers(0, 5)), needles=needles, ragged=ragged,
                          pad_nan=bool(ragged) and rng.random() < 0.5,
                          shared_query=float(rng.choice([0.0, 0.0, 0.5, 1.0])))


@pytest.mark.parametrize("seed", range(40))
def test_random_shape(seed):
    _check(_draw(seed))


@pytest.mark.parametrize("seed", range(24))
def test_random_decode_shape(seed):
    """One-row windows (the decoding setting): the bf16 draws run on the decode kernels, the fp32 ones on the plain path."""
    _check(_draw(seed, decode=True))


def _draw_long(seed):
    """Caches of several sequence splits and many tiles on the matrix-core path (bf16, d = 128)."""
    rng = np.random.default_rng(9000 + seed)
    G = int(rng.choice([1, 2, 4, 7]))
    Hkv = int(rng.integers(1, 3))
    W = int(rng.integers(1, 49))
    N = int(rng.integers(2600, 24000))
    B = int(rng.integers(1, 3))
    ragged = (int(rng.integers(max(W, N // 4), N + 1)), N) if rng.random() < 0.6 else None
    min_len = ragged[0] if ragged else N
    sinks = int(rng.integers(0, 5))
    return synth.Workload("long%d" % seed, B=B, Hq=G * Hkv, Hkv=Hkv, d=128, N=N, W=W, dtype="bf16",
                          budget=max(1, min_len // 8), seed=9500 + seed, sinks=sinks,
                          outlier_channels=int(rng.integers(0, 5)), needles=int(rng.integers(0, 9)), ragged=ragged,
                          pad_nan=bool(ragged) and rng.random() < 0.5,
                          shared_query=float(rng.choice([0.0, 0.0, 0.5, 1.0])))


@pytest.mark.parametrize("seed", range(10))
def test_random_long_shape(seed):
    _check(_draw_long(seed))


def _check(wl):
    x = synth.make_inputs(wl)
    dev = to_device(x)
    lens = x["seq_lens"]
    tol = TOL[wl.dtype]
    label = "%s B%d Hq%d Hkv%d d%d N%d W%d %s lens=%s budget=%d" % (wl.name, wl.B, wl.Hq, wl.Hkv, wl.d, wl.N, wl.W,
                                                                    wl.dtype, lens, wl.budget)
    ref = list(oracle.score(x["q"], x["k"], x["v"], seq_lens=lens))
    ref.append(oracle.attn_score(x["q"], x["k"], x["v"], seq_lens=lens))
    ref.append(oracle.vatp_score(x["q"], x["k"], x["v"], seq_lens=lens))
    all3 = obc.obc_score(dev["q"], dev["k"], dev["v"], "all", seq_lens=lens)
    gpu = [all3[0], all3[1], all3[2],
           obc.obc_score(dev["q"], dev["k"], dev["v"], "attn", seq_lens=lens),
           obc.obc_score(dev["q"], dev["k"], dev["v"], "vatp", seq_lens=lens)]
    torch.cuda.synchronize()
    for name, g, r in zip(("value", "key", "joint", "attn", "vatp"), gpu, ref):
        gn = g.cpu().numpy()
        assert np.isfinite(gn).all() and (gn >= 0).all(), (label, name)
        err, where = score_error(gn, np.asarray(r), wl.budget, lens, tol)
        assert err <= tol, "%s %s: err %.3g at %s" % (label, name, err, where)
    joint = gpu[2].contiguous()
    keep = obc.obc_select(joint, wl.budget, seq_lens=lens).cpu().numpy()
    np.testing.assert_array_equal(keep, oracle.select(joint.cpu().numpy(), wl.budget, lens), err_msg=label)
