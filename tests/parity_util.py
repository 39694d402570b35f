"""Helpers shared by the GPU parity tests (test infrastructure only)."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2510_07651_amd import binding as obc
from paper_2510_07651_amd import synth

TOL = {"fp32": 1e-5, "bf16": 1e-3}   # relative tolerance on scores, per storage dtype
FP32_SCORE_FLOOR = 1e-30             # scale below which fp32 scores are not compared relative to themselves


def kth_largest(s: np.ndarray, k: int, length: int) -> float:
    return float(np.partition(s[:length], length - k)[length - k])


def score_error(gpu: np.ndarray, ref: np.ndarray, budget: int, lens, tol: float):
    """Worst |gpu - ref| / max(|ref|, floor) over all head-tokens.

    floor = tol * (the head's budget-th largest oracle score), at least FP32_SCORE_FLOOR:
    scores far below the selection threshold are compared on the
    threshold's scale, because that is the scale on which they can influence which tokens
    are kept; everything at or above the threshold is compared relative to itself.
    """
    B, H, N = ref.shape
    worst, where = 0.0, None
    for b in range(B):
        L = N if lens is None else lens[b]
        for h in range(H):
            # An fp32 pipeline flushes attention weights (or their squares) below its smallest normal number, 1.2e-38,
            # before they meet norms of up to ~1e8: oracle scores below ~1e-30 are out of its reach and are compared
            # on that scale (such a token has less than 1e-15 of any row's attention)
            floor = max(tol * kth_largest(ref[b, h], budget, L), FP32_SCORE_FLOOR)
            err = np.abs(gpu[b, h, :L] - ref[b, h, :L]) / np.maximum(np.abs(ref[b, h, :L]), floor)
            i = int(np.argmax(err))
            if err[i] > worst:
                worst, where = float(err[i]), (b, h, i, float(gpu[b, h, i]), float(ref[b, h, i]))
            assert np.all(gpu[b, h, L:] == 0.0), "scores at padded positions must be exactly 0"
    return worst, where


def raw_relative_error(gpu: np.ndarray, ref: np.ndarray, lens):
    """(max, 99.9th percentile) of |gpu - ref| / |ref| over the live head-tokens with a nonzero oracle score: no floor.
    Reported beside the floored error, not asserted (scores far below the selection threshold may sit at the edge of
    what fp32 resolves)."""
    B, H, N = ref.shape
    errs = []
    for b in range(B):
        L = N if lens is None else lens[b]
        r = ref[b, :, :L]
        nz = r != 0
        errs.append((np.abs(gpu[b, :, :L] - r)[nz] / np.abs(r[nz])).ravel())
    e = np.concatenate(errs)
    return (float(e.max()), float(np.quantile(e, 0.999))) if e.size else (0.0, 0.0)


def check_selection_against_oracle_scores(keep: np.ndarray, ref: np.ndarray, budget: int, lens, tol: float):
    """End-to-end index parity: outside a band of +-2*tol around the head's budget-th
    largest oracle score the kept set is unique; inside it either choice is valid."""
    B, H, N = ref.shape
    in_band_total = 0
    for b in range(B):
        L = N if lens is None else lens[b]
        for h in range(H):
            s = ref[b, h, :L]
            tau = kth_largest(s, budget, L)
            kept = np.zeros(L, dtype=bool)
            kept[keep[b, h]] = True
            must = s > tau * (1 + 2 * tol)
            must_not = s < tau * (1 - 2 * tol)
            assert kept[must].all(), "a token clearly above the threshold was dropped (b=%d h=%d)" % (b, h)
            assert not kept[must_not].any(), "a token clearly below the threshold was kept (b=%d h=%d)" % (b, h)
            in_band_total += int((~must & ~must_not).sum())
    return in_band_total


def check_keep_idx_valid(keep: np.ndarray, budget: int, lens, N: int):
    B, H, K = keep.shape
    assert K == budget
    for b in range(B):
        L = N if lens is None else lens[b]
        for h in range(H):
            row = keep[b, h]
            assert row.min() >= 0 and row.max() < L
            assert np.all(np.diff(row) > 0), "kept indices must be strictly ascending"


def to_device(x):
    return {k: (v.cuda() if torch.is_tensor(v) else v) for k, v in x.items()}


def oracle_scores(x, heads=None):
    """Oracle scores for all heads, or for a list of (b, g) KV heads (full-size sampling)."""
    if heads is None:
        return oracle.score(x["q"], x["k"], x["v"], seq_lens=x["seq_lens"])
    q, k, v = x["q"], x["k"], x["v"]
    G = q.shape[1] // k.shape[1]
    out = []
    for b, g in heads:
        lens = None if x["seq_lens"] is None else [x["seq_lens"][b]]
        out.append(oracle.score(q[b:b + 1, g * G:(g + 1) * G], k[b:b + 1, g:g + 1], v[b:b + 1, g:g + 1],
                                seq_lens=lens))
    return out


def run_case(wl):
    """Scores (all variants), selection and compaction of one workload through the C ABI against the oracle;
    returns the worst score error per variant."""
    x = synth.make_inputs(wl)
    dev = to_device(x)
    lens = x["seq_lens"]
    tol = TOL[wl.dtype]
    ref = oracle_scores(x)
    all3 = obc.obc_score(dev["q"], dev["k"], dev["v"], "all", seq_lens=lens)
    torch.cuda.synchronize()
    assert all3.shape == (3, wl.B, wl.Hkv, wl.N)
    worst = {}
    for vi, name in enumerate(synth.VARIANTS):
        gpu = all3[vi].cpu().numpy()
        assert np.isfinite(gpu).all() and (gpu >= 0).all(), name
        worst[name], where = score_error(gpu, ref[vi], wl.budget, lens, tol)
        assert worst[name] <= tol, "%s %s: err %.3g at %s" % (wl.name, name, worst[name], where)
        # single-variant calls agree with the all-variant call (the value-only call skips the
        # attention outputs, and with them the refinement of dominant rows, so bits may differ)
        one = obc.obc_score(dev["q"], dev["k"], dev["v"], name, seq_lens=lens)
        if name == "value":
            torch.testing.assert_close(one, all3[vi], rtol=2e-5, atol=0.0)
        else:
            assert torch.equal(one, all3[vi]), name
        # selection: bit-exact vs the oracle's select on the very same fp32 scores
        keep = obc.obc_select(all3[vi].contiguous(), wl.budget, seq_lens=lens)
        keep_np = keep.cpu().numpy()
        check_keep_idx_valid(keep_np, wl.budget, lens, wl.N)
        np.testing.assert_array_equal(keep_np, oracle.select(gpu, wl.budget, lens))
        # and consistent with the oracle's own scores outside the tolerance band
        check_selection_against_oracle_scores(keep_np, ref[vi], wl.budget, lens, tol)
    # compaction: byte-exact gather
    k_out, v_out = obc.obc_compact(dev["k"], dev["v"], keep)
    as_bits = (lambda t: t.view(torch.int16)) if wl.dtype == "bf16" else (lambda t: t.view(torch.int32))
    kref, vref = oracle.compact(as_bits(x["k"]).numpy(), as_bits(x["v"]).numpy(), keep_np)
    np.testing.assert_array_equal(as_bits(k_out).cpu().numpy(), kref)
    np.testing.assert_array_equal(as_bits(v_out).cpu().numpy(), vref)
    return worst
