"""GPU selection family on seeded random scores, sizes and parameters: every kept index bit-exact against the oracle.

The draws mix what hand-picked cases keep apart: head lengths from a handful of tokens to 140000 (single block,
streamed and sliced kernels), ragged batches, scores with heavy ties, a wide dynamic range, NaN / inf / -0 / subnormal
entries, protected sinks and recent windows of any size, every pooling width, safeguards from 0 to the whole budget;
each result is then pushed through the in-place compaction and compared with the oracle's gather.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_07651_amd import binding as obc

pytestmark = pytest.mark.gpu


def _scores(rng, shape):
    kind = int(rng.integers(0, 4))
    if kind == 0:
        s = rng.random(shape)
    elif kind == 1:
        s = np.floor(rng.random(shape) * rng.integers(2, 40))                 # heavy ties
    elif kind == 2:
        s = np.exp(rng.normal(0.0, 12.0, shape))                              # many binades
    else:
        s = rng.normal(0.0, 1.0, shape)                                       # negative scores too
    s = s.astype(np.float32)
    flat = s.reshape(-1)
    n_special = int(rng.integers(0, max(2, flat.size // 50)))
    for v in (np.nan, np.inf, -np.inf, -0.0, 1e-42, -1e-42):
        idx = rng.integers(0, flat.size, size=n_special // 6 + 1)
        if rng.random() < 0.5:
            flat[idx] = v
    return s


def _shape(rng):
    r = rng.random()
    if r < 0.35:
        N = int(rng.integers(1, 300))
    elif r < 0.85:
        N = int(rng.integers(300, 9000))
    else:
        N = int(rng.integers(33000, 140000))
    B = int(rng.integers(1, 5))
    Hkv = int(rng.integers(1, 5)) if N < 33000 else int(rng.integers(1, 3))
    return B, Hkv, N


def _lens(rng, B, N, floor):
    if rng.random() < 0.5 or floor >= N:
        return None
    return [int(rng.integers(floor, N + 1)) for _ in range(B)]


def _check_inplace(rng, keep, N):
    """The kept rows through obc_compact_inplace against the oracle's gather (short rows: the indices are the point)."""
    B, Hkv, budget = keep.shape
    d = 8
    k = rng.integers(-2 ** 31, 2 ** 31, size=(B, Hkv, N, d), dtype=np.int64).astype(np.int32)
    v = rng.integers(-2 ** 31, 2 ** 31, size=(B, Hkv, N, d), dtype=np.int64).astype(np.int32)
    kd = torch.from_numpy(k).cuda().view(torch.float32)
    vd = torch.from_numpy(v).cuda().view(torch.float32)
    obc.obc_compact_inplace(kd, vd, torch.from_numpy(keep).cuda())
    kref, vref = oracle.compact(k, v, keep)
    np.testing.assert_array_equal(kd.view(torch.int32).cpu().numpy()[:, :, :budget], kref)
    np.testing.assert_array_equal(vd.view(torch.int32).cpu().numpy()[:, :, :budget], vref)
    np.testing.assert_array_equal(kd.view(torch.int32).cpu().numpy()[:, :, budget:], k[:, :, budget:])


@pytest.mark.parametrize("seed", range(30))
def test_random_select_protected_and_pooled(seed):
    rng = np.random.default_rng(300 + seed)
    B, Hkv, N = _shape(rng)
    s = _scores(rng, (B, Hkv, N))
    sinks = int(rng.integers(0, min(6, N)))
    recent = int(rng.integers(0, min(300, N - sinks) + 1))
    coming = int(rng.integers(0, recent + 1)) if recent else 0
    tail = recent - coming
    lens = _lens(rng, B, N, max(1, sinks + tail))
    shortest = min(lens) if lens else N
    room = shortest - sinks - tail
    hh = int(rng.integers(0 if sinks + tail > 0 else 1, room + 1)) if room >= 1 else 0
    if sinks + hh + tail < 1:
        hh = 1
    pool = int(rng.choice([1, 1, 3, 5, 7, 15]))
    dev = torch.from_numpy(s).cuda()
    label = "seed %d B%d Hkv%d N%d lens=%s hh=%d sinks=%d recent=%d coming=%d pool=%d" % (
        seed, B, Hkv, N, lens, hh, sinks, recent, coming, pool)
    want = oracle.select_pooled(s, hh, pool=pool, num_sinks=sinks, num_recent=recent, num_coming=coming, seq_lens=lens)
    for use_ws in (None, False):                     # with the optional scratch (sliced kernels on long heads), and without
        got = obc.obc_select_pooled(dev, hh, pool=pool, num_sinks=sinks, num_recent=recent, num_coming=coming,
                                    seq_lens=lens, workspace=use_ws).cpu().numpy()
        np.testing.assert_array_equal(got, want, err_msg=label)
    if pool == 1:
        got = obc.obc_select_protected(dev, hh, sinks, recent, coming, seq_lens=lens).cpu().numpy()
        np.testing.assert_array_equal(got, oracle.select_protected(s, hh, sinks, recent, coming, lens), err_msg=label)
        if sinks == 0 and recent == 0:
            got = obc.obc_select(dev, hh, seq_lens=lens).cpu().numpy()
            np.testing.assert_array_equal(got, oracle.select(s, hh, lens), err_msg=label)
    if N <= 9000:
        _check_inplace(rng, want, N)


@pytest.mark.parametrize("seed", range(16))
def test_random_select_adaptive(seed):
    rng = np.random.default_rng(700 + seed)
    B, Hkv, N = _shape(rng)
    N = min(N, 40000)
    s = _scores(rng, (B, Hkv, N))
    lens = _lens(rng, B, N, 1)
    shortest = min(lens) if lens else N
    budget = int(rng.integers(1, shortest + 1))
    n_safe = int(rng.choice([0, budget, int(rng.integers(0, budget + 1)), budget // 5]))
    label = "seed %d B%d Hkv%d N%d lens=%s budget=%d n_safe=%d" % (seed, B, Hkv, N, lens, budget, n_safe)
    want_idx, want_cnt = oracle.select_adaptive(s, budget, n_safe, seq_lens=lens)
    got_idx, got_cnt = obc.obc_select_adaptive(torch.from_numpy(s).cuda(), budget, n_safe, seq_lens=lens)
    np.testing.assert_array_equal(got_cnt.cpu().numpy(), want_cnt, err_msg=label)
    np.testing.assert_array_equal(got_idx.cpu().numpy(), want_idx, err_msg=label)
    if N <= 9000:
        _check_inplace(rng, want_idx, N)
