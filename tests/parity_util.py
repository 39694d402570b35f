"""Helpers shared by the GPU parity tests (test infrastructure only)."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2510_07651_amd import synth

TOL = {"fp32": 1e-5, "bf16": 1e-3}   # relative tolerance on scores, per storage dtype


def kth_largest(s: np.ndarray, k: int, length: int) -> float:
    return float(np.partition(s[:length], length - k)[length - k])


def score_error(gpu: np.ndarray, ref: np.ndarray, budget: int, lens, tol: float):
    """Worst |gpu - ref| / max(|ref|, floor) over all head-tokens.

    floor = tol * (the head's budget-th largest oracle score): scores far below the
    selection threshold are compared on the threshold's scale, because that is the scale
    on which they can influence which tokens are kept; everything at or above the
    threshold is compared relative to itself.
    """
    B, H, N = ref.shape
    worst, where = 0.0, None
    for b in range(B):
        L = N if lens is None else lens[b]
        for h in range(H):
            floor = tol * kth_largest(ref[b, h], budget, L)
            err = np.abs(gpu[b, h, :L] - ref[b, h, :L]) / np.maximum(np.abs(ref[b, h, :L]), floor)
            i = int(np.argmax(err))
            if err[i] > worst:
                worst, where = float(err[i]), (b, h, i, float(gpu[b, h, i]), float(ref[b, h, i]))
            assert np.all(gpu[b, h, L:] == 0.0), "scores at padded positions must be exactly 0"
    return worst, where


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
