"""GPU parity of the matrix-core scoring path on hand-built rows whose attention sits on one or a few keys.

Eq. 5 and 6 contain v_p - o_i, which for a key that holds nearly all of row i's attention is a difference of
nearly equal vectors.  The matrix-core path keeps, per row, the key that may end up dominant out of its running
sums and forms that difference directly; these inputs drive every branch of that bookkeeping on bf16 caches with
d = 128 and several sequence splits:

* a staircase of keys, each clearing the previous maximum by three nats or more, seven of them inside one split (more
  than a lane can park: some are added back on the spot), ending in a key that dominates the row; shorter
  staircases over a quiet background that end in a key with about two thirds or one third of the attention;
* two keys with exactly the same logit (same K row, different V rows) sharing a row half and half, in the same
  block of 32 tokens, in different blocks, in different splits;
* every row dominated by its own token (the last key it may see, inside the causally masked blocks) with a
  sink at token 0 that holds a third;
* the dominant key in the last split while an earlier split holds a strong runner-up;
* a ragged batch whose dominant keys sit on the last token of a partial block;
* staircases whose direction differs from row to row, so that the rows of one wave meet their candidates
  in different steps.

All inputs are seeded and synthetic.  Tolerance: 1e-3 relative as everywhere for bf16 inputs; the fp64 oracle
evaluates the dominant key's difference without cancellation (see its header).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_07651_amd import binding as obc

from parity_util import TOL, score_error

D = 128
VARIANTS = ("value", "key", "joint")


def _base(seed, B, Hq, Hkv, N, W):
    """Background: unit-variance keys and values; queries = sqrt(d) u + 0.3 noise with u a unit vector per KV head,
    so that a key c u has logit c (+ small noise) for every row of the head and a background key about N(0, 1)."""
    g = torch.Generator().manual_seed(seed)
    k = torch.randn(B, Hkv, N, D, generator=g, dtype=torch.float64)
    v = torch.randn(B, Hkv, N, D, generator=g, dtype=torch.float64)
    u = torch.randn(B, Hkv, D, generator=g, dtype=torch.float64)
    u = u / u.norm(dim=-1, keepdim=True)
    G = Hq // Hkv
    q = 0.3 * torch.randn(B, Hq, W, D, generator=g, dtype=torch.float64)
    q = q + np.sqrt(D) * u.repeat_interleave(G, dim=1)[:, :, None, :]
    return q, k, v, u


def _plant(k, u, b, h, tok, c):
    k[b, h, tok] = c * u[b, h]


def _finish(q, k, v, lens=None):
    to = lambda t: t.to(torch.float32).to(torch.bfloat16)
    return {"q": to(q), "k": to(k), "v": to(v), "seq_lens": lens}


def _staircase(stairs, background=1.0):
    q, k, v, u = _base(11, 1, 4, 1, 6000, 32)
    k *= background
    for j, c in enumerate(stairs):
        _plant(k, u, 0, 0, 20 + 70 * j, c)                 # all inside the first 512 tokens
    return _finish(q, k, v)


def _ties(tok_a, tok_b):
    q, k, v, u = _base(12, 1, 8, 2, 5000, 32)
    for h in range(2):
        _plant(k, u, 0, h, tok_a, 24.0)
        _plant(k, u, 0, h, tok_b, 24.0)
    return _finish(q, k, v)


def _diagonal():
    B, Hq, Hkv, N, W = 1, 4, 1, 4100, 32
    q, k, v, u = _base(13, B, Hq, Hkv, N, W)
    # row i of every query head attends to its own token N - W + i: that key is aligned with the row's own noise
    # direction (shared by the four heads of the group), the sink at token 0 with the common direction
    g = torch.Generator().manual_seed(130)
    own = torch.randn(W, D, generator=g, dtype=torch.float64)
    own = own - (own @ u[0, 0])[:, None] * u[0, 0][None, :]
    own = own / own.norm(dim=-1, keepdim=True)
    q[0] += 14.0 * own[None, :, :]
    for i in range(W):
        k[0, 0, N - W + i] = (np.sqrt(D) * 13.0 / 14.0) * own[i]       # logit ~13 for row i, ~0 for the others
    _plant(k, u, 0, 0, 0, 12.3)                                           # sink: about a third of every row
    return _finish(q, k, v)


def _late_split():
    q, k, v, u = _base(14, 1, 4, 1, 6000, 32)
    _plant(k, u, 0, 0, 3, 15.0)            # runner-up in the first split: e^-1 of the winner
    _plant(k, u, 0, 0, 5900, 16.0)         # winner in the last split
    return _finish(q, k, v)


def _ragged():
    lens = [2600, 3999, 5000]
    q, k, v, u = _base(15, 3, 4, 1, 5000, 32)
    for b, L in enumerate(lens):
        # the last key every window row of the sequence may see is L - 32; end it on a partial block
        _plant(k, u, b, 0, L - 32, 21.0)
        _plant(k, u, b, 0, 1, 12.0)
        k[b, 0, L:] = float("nan")
        v[b, 0, L:] = float("nan")
    return _finish(q, k, v, lens)


def _staggered():
    """Every row has a staircase of its own direction and its own token positions inside the first two splits."""
    B, Hq, Hkv, N, W = 1, 4, 1, 4500, 32
    q, k, v, u = _base(16, B, Hq, Hkv, N, W)
    g = torch.Generator().manual_seed(160)
    own = torch.randn(W, D, generator=g, dtype=torch.float64)
    own = own / own.norm(dim=-1, keepdim=True)
    q[0] += 14.0 * own[None, :, :]
    for i in range(W):
        for j in range(6):
            tok = 5 + 31 * i + 7 * j * (1 + i % 3)            # rows meet their candidates in different steps
            k[0, 0, tok] = (np.sqrt(D) / 14.0) * (5.0 + 3.0 * j + 0.1 * i + (4.0 if j == 5 else 0.0)) * own[i]
    return _finish(q, k, v)


CASES = {
    "staircase_dominant": lambda: _staircase((4.0, 7.0, 10.0, 13.0, 16.0, 19.0, 27.0)),
    # (a quiet background, 6000 keys of logit ~N(0, 0.1): its weight is e^8.75, its largest logit ~1.2)
    "staircase_two_thirds": lambda: _staircase((1.9, 4.4, 6.9, 9.45), background=0.3),
    "staircase_one_third": lambda: _staircase((0.5, 3.0, 5.5, 8.05), background=0.3),
    "ties_same_block": lambda: _ties(100, 117),
    "ties_other_block": lambda: _ties(100, 300),
    "ties_other_split": lambda: _ties(100, 4000),
    "diagonal_and_sink": _diagonal,
    "winner_in_last_split": _late_split,
    "ragged_partial_block": _ragged,
    "staggered_staircases": _staggered,
}


@pytest.mark.gpu
@pytest.mark.parametrize("name", list(CASES))
def test_dominant_rows_match_oracle(name, score_path):
    score_path("mfma")
    x = CASES[name]()
    lens = x["seq_lens"]
    ref = oracle.score(x["q"], x["k"], x["v"], seq_lens=lens)
    dev = {n: x[n].cuda() for n in ("q", "k", "v")}
    all3 = obc.obc_score(dev["q"], dev["k"], dev["v"], "all", seq_lens=lens)
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    worst = {}
    for vi, variant in enumerate(VARIANTS):
        gpu = all3[vi].cpu().numpy()
        assert np.isfinite(gpu).all() and (gpu >= 0).all(), variant
        worst[variant], where = score_error(gpu, ref[vi], 64, lens, tol)
        assert worst[variant] <= tol, "%s %s: err %.3g at %s" % (name, variant, worst[variant], where)
        one = obc.obc_score(dev["q"], dev["k"], dev["v"], variant, seq_lens=lens)
        if variant == "value":
            torch.testing.assert_close(one, all3[vi], rtol=2e-5, atol=0.0)
        else:
            assert torch.equal(one, all3[vi]), variant
    print(name, {k: "%.2e" % e for k, e in worst.items()})


def test_the_cases_are_what_they_claim():
    """Top shares per row from the oracle's attention: the staircases end where they should, ties split in half."""
    def top_share(x):
        _, A, _ = oracle.window_attention(x["q"], x["k"], x["v"], seq_lens=x["seq_lens"])
        return np.sort(A, axis=-1)[..., ::-1]
    s = top_share(CASES["staircase_dominant"]())
    assert s[..., 0].min() > 0.999
    s = top_share(CASES["staircase_two_thirds"]())
    assert 0.5 < np.median(s[..., 0]) < 0.85
    s = top_share(CASES["staircase_one_third"]())
    assert 0.15 < np.median(s[..., 0]) < 0.5
    s = top_share(CASES["ties_other_split"]())
    assert np.abs(s[..., 0] - 0.5).max() < 1e-3 and np.abs(s[..., 1] - 0.5).max() < 1e-3
    s = top_share(CASES["diagonal_and_sink"]())
    assert np.median(s[..., 0]) > 0.5 and np.median(s[..., 1]) > 0.15
    s = top_share(CASES["winner_in_last_split"]())
    assert 0.6 < np.median(s[..., 0]) < 0.8 and 0.2 < np.median(s[..., 1]) < 0.35
