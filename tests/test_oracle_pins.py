"""Pins of the fp64 CPU oracle against what the paper and the mathematics fix.

The paper (arxiv 2510.07651) prints no worked numeric example of a score, so the
oracle is pinned to: the definition the closed forms approximate (Definition 4.1 /
Eq. 1 and its windowed form Eq. 9, evaluated by brute force here, in numpy, with
code independent of the oracle), exact identities from the derivation in
Appendix A, closed forms of special cases, a library attention routine, and
invariances.  Each test names the plausible oracle mistake it would catch.
"""
import numpy as np
import pytest
import torch

import oracle


# ----------------------------------------------------------------------------
# Independent brute-force helpers (numpy, fp64).  They implement Section 3's
# attention for the window rows only; nothing here calls the oracle.
# ----------------------------------------------------------------------------
def window_outputs(q, K, V, length=None):
    """q [W,d], K,V [N,d] -> O [W,d]; row r sits at position len-W+r, causal."""
    W, d = q.shape
    N = K.shape[0] if length is None else length
    out = np.zeros((W, d))
    for r in range(W):
        n_vis = N - W + r + 1
        z = K[:n_vis] @ q[r] / np.sqrt(d)
        e = np.exp(z - z.max())
        a = e / e.sum()
        out[r] = a @ V[:n_vis]
    return out


def group_window_outputs(q, K, V, length=None):
    """q [G,W,d] (query heads sharing one KV head) -> O [G,W,d]."""
    return np.stack([window_outputs(q[h], K, V, length) for h in range(q.shape[0])])


def rand_case(seed, B=1, Hq=2, Hkv=1, N=24, W=5, d=8, scale=1.0):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, Hq, W, d)) * scale
    k = rng.standard_normal((B, Hkv, N, d))
    v = rng.standard_normal((B, Hkv, N, d))
    return q, k, v


# ----------------------------------------------------------------------------
# P1  softmax rows: sum to 1, non-negative, invisible entries absent
# ----------------------------------------------------------------------------
def test_softmax_rows_and_mask():
    q, k, v = rand_case(1, B=2, Hq=4, Hkv=2, N=30, W=6, d=16)
    lens = [30, 17]
    Z, A, O = oracle.window_attention(q, k, v, seq_lens=lens)
    for b in range(2):
        for r in range(6):
            n_vis = lens[b] - 6 + r + 1
            row = A[b, :, r, :]
            np.testing.assert_allclose(row.sum(-1), 1.0, rtol=0, atol=1e-14)
            assert (row >= 0).all()
            assert (row[:, n_vis:] == 0).all() and (row[:, :n_vis] > 0).all()
            assert np.isnan(Z[b, :, r, n_vis:]).all() and np.isfinite(Z[b, :, r, :n_vis]).all()


# ----------------------------------------------------------------------------
# P8  A, Z, O against a library routine (torch SDPA, fp64, explicit mask)
# ----------------------------------------------------------------------------
def test_attention_matches_torch_sdpa():
    B, Hq, Hkv, N, W, d = 2, 6, 2, 41, 9, 16
    q, k, v = rand_case(2, B, Hq, Hkv, N, W, d)
    lens = [41, 29]
    Z, A, O = oracle.window_attention(q, k, v, seq_lens=lens)
    G = Hq // Hkv
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    tk = tk.repeat_interleave(G, dim=1)            # consecutive grouping: head h reads KV head h // G
    tv = tv.repeat_interleave(G, dim=1)
    mask = torch.zeros(B, 1, W, N, dtype=torch.bool)
    for b in range(B):
        for r in range(W):
            mask[b, 0, r, : lens[b] - W + r + 1] = True
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)
    np.testing.assert_allclose(O, ref.numpy(), rtol=1e-12, atol=1e-13)
    zref = (tq @ tk.transpose(-1, -2) / np.sqrt(d)).numpy()
    vis = mask.expand(B, Hq, W, N).numpy()
    np.testing.assert_allclose(Z[vis], zref[vis], rtol=1e-13, atol=1e-13)


# ----------------------------------------------------------------------------
# P2 / P3  signs, and Eq. 6 literal == completed square
# ----------------------------------------------------------------------------
def test_scores_nonnegative_and_joint_forms_agree():
    q, k, v = rand_case(3, B=2, Hq=4, Hkv=2, N=50, W=8, d=16, scale=2.0)
    lens = [50, 31]
    sv, sk, sj = oracle.score(q, k, v, seq_lens=lens, joint_form=0)
    _, _, sj_lit = oracle.score(q, k, v, seq_lens=lens, joint_form=1)
    assert (sv >= 0).all() and (sk >= 0).all() and (sj >= 0).all()
    np.testing.assert_allclose(sj_lit, sj, rtol=1e-12, atol=1e-15)
    # padded positions score exactly zero
    assert (sv[1, :, 31:] == 0).all() and (sk[1, :, 31:] == 0).all() and (sj[1, :, 31:] == 0).all()
    # the cross term is not identically zero: joint differs from value + key
    assert np.abs(sj - (sv + sk)).max() > 1e-3


# ----------------------------------------------------------------------------
# P4  value score is EXACT (Appendix A.2: the objective is quadratic in dV):
#     zero v_p, recompute the window outputs, squared Frobenius change == S^value_p.
#     Catches: wrong window rows, wrong causal bound, missing group sum, A vs A^2.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (3, 1), (4, 2)])
def test_value_score_equals_bruteforce_zeroing(Hq, Hkv):
    B, N, W, d = 1, 26, 6, 8
    q, k, v = rand_case(4 + Hq, B, Hq, Hkv, N, W, d, scale=1.5)
    sv, _, _ = oracle.score(q, k, v)
    G = Hq // Hkv
    for g in range(Hkv):
        qg = q[0, g * G:(g + 1) * G]
        base = group_window_outputs(qg, k[0, g], v[0, g])
        for p in range(N):
            V2 = v[0, g].copy()
            V2[p] = 0.0
            err = ((group_window_outputs(qg, k[0, g], V2) - base) ** 2).sum()
            np.testing.assert_allclose(sv[0, g, p], err, rtol=1e-10, atol=1e-18)


# ----------------------------------------------------------------------------
# P5  key and joint scores are the squared directional derivative of the window
#     outputs along (dV, dK) = (-v_p, -k_p) on row p (Theorem 4.2 with the
#     Gauss-Newton Hessians of Appendix A.3-A.4): central differences, brute force.
#     Catches: dropped / mis-signed cross term, Z shifted by the max, o_i of the
#     wrong row, ||v-o|| vs ||v||, transposed operands.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("seed,Hq,Hkv", [(10, 1, 1), (11, 2, 1), (12, 4, 2)])
def test_key_and_joint_scores_equal_squared_directional_derivative(seed, Hq, Hkv):
    B, N, W, d = 1, 22, 5, 8
    q, k, v = rand_case(seed, B, Hq, Hkv, N, W, d, scale=1.3)
    _, sk, sj = oracle.score(q, k, v)
    G = Hq // Hkv
    t = 1e-4
    for g in range(Hkv):
        qg = q[0, g * G:(g + 1) * G]
        K0, V0 = k[0, g], v[0, g]
        for p in range(N):
            for which, ref in (("key", sk), ("joint", sj)):
                def out(sign):
                    K2, V2 = K0.copy(), V0.copy()
                    K2[p] = K0[p] * (1.0 - sign * t)          # K + (sign t) dK, dK_p = -k_p
                    if which == "joint":
                        V2[p] = V0[p] * (1.0 - sign * t)
                    return group_window_outputs(qg, K2, V2)
                D = (out(+1) - out(-1)) / (2 * t)
                np.testing.assert_allclose(ref[0, g, p], (D ** 2).sum(), rtol=2e-6, atol=1e-16)


# ----------------------------------------------------------------------------
# P6  Definition 4.1 itself (row p of K and V set to zero, softmax recomputed)
#     converges to the closed forms as the logits shrink (q scaled by eps).
# ----------------------------------------------------------------------------
def test_full_zeroing_converges_to_closed_form():
    B, Hq, Hkv, N, W, d = 1, 2, 1, 20, 4, 8
    q, k, v = rand_case(20, B, Hq, Hkv, N, W, d)
    ratios = {}
    for eps in (1e-2, 1e-3):
        qe = q * eps
        _, sk, sj = oracle.score(qe, k, v)
        base = group_window_outputs(qe[0], k[0, 0], v[0, 0])
        worst = 0.0
        for p in range(N):
            K2, V2 = k[0, 0].copy(), v[0, 0].copy()
            K2[p] = 0.0
            Lk = ((group_window_outputs(qe[0], K2, v[0, 0]) - base) ** 2).sum()
            V2[p] = 0.0
            Lj = ((group_window_outputs(qe[0], K2, V2) - base) ** 2).sum()
            worst = max(worst, abs(Lk / sk[0, 0, p] - 1), abs(Lj / sj[0, 0, p] - 1))
        ratios[eps] = worst
    assert ratios[1e-3] < 1e-2
    assert ratios[1e-3] < ratios[1e-2] / 5          # first-order convergence in eps


# ----------------------------------------------------------------------------
# P7  closed form at q = 0: Z = 0, A_rp = 1/(len-W+r+1)
# ----------------------------------------------------------------------------
def test_zero_queries_closed_form():
    B, Hq, Hkv, N, W, d = 1, 3, 1, 19, 4, 8
    _, k, v = rand_case(30, B, Hq, Hkv, N, W, d)
    q = np.zeros((B, Hq, W, d))
    sv, sk, sj = oracle.score(q, k, v)
    vv = (v[0, 0] ** 2).sum(-1)
    expect = np.zeros(N)
    for r in range(W):
        n_vis = N - W + r + 1
        expect[:n_vis] += Hq * vv[:n_vis] / n_vis ** 2
    np.testing.assert_allclose(sv[0, 0], expect, rtol=1e-13)
    np.testing.assert_allclose(sj[0, 0], expect, rtol=1e-13)
    assert np.abs(sk).max() == 0.0


# ----------------------------------------------------------------------------
# P9  permuting tokens of the prefix (visible to every window row) permutes scores
# ----------------------------------------------------------------------------
def test_prefix_permutation_equivariance():
    B, Hq, Hkv, N, W, d = 1, 4, 2, 40, 6, 8
    q, k, v = rand_case(40, B, Hq, Hkv, N, W, d)
    perm = np.arange(N)
    perm[: N - W] = np.random.default_rng(0).permutation(N - W)
    a = oracle.score(q, k, v)
    b = oracle.score(q, k[:, :, perm], v[:, :, perm])
    for x, y in zip(a, b):
        np.testing.assert_allclose(y, x[:, :, perm], rtol=1e-11, atol=1e-18)


# ----------------------------------------------------------------------------
# P10  GQA (Appendix A.5): group score == sum of MHA scores with K,V repeated;
#      W = 1 is the single-row case; attention-only score (Eq. 8) sums |A|.
# ----------------------------------------------------------------------------
def test_gqa_is_sum_of_mha_heads_and_w1():
    B, Hq, Hkv, N, W, d = 2, 6, 2, 33, 5, 8
    q, k, v = rand_case(50, B, Hq, Hkv, N, W, d)
    G = Hq // Hkv
    grouped = oracle.score(q, k, v)
    mha = oracle.score(q, np.repeat(k, G, axis=1), np.repeat(v, G, axis=1))
    for x, y in zip(grouped, mha):
        np.testing.assert_allclose(x, y.reshape(B, Hkv, G, N).sum(2), rtol=1e-12)
    # W = 1: scores of the last query row alone
    q1 = q[:, :, -1:, :]
    sv1, _, _ = oracle.score(q1, k, v)
    Z, A, O = oracle.window_attention(q1, k, v)
    vv = (v ** 2).sum(-1)
    np.testing.assert_allclose(sv1, (A[:, :, 0, :] ** 2).reshape(B, Hkv, G, N).sum(2) * vv, rtol=1e-12)
    sa = oracle.attn_score(q, k, v)
    _, Aw, _ = oracle.window_attention(q, k, v)
    np.testing.assert_allclose(sa, Aw.sum(2).reshape(B, Hkv, G, N).sum(2), rtol=1e-12)
    np.testing.assert_allclose(sa.sum(-1), G * W, rtol=1e-12)      # every row of A sums to 1


# ----------------------------------------------------------------------------
# P11  plumbing identity: dropping token p from the softmax changes o_i by
#      -A_ip (v_p - o_i) / (1 - A_ip)  (exact; follows from Section 3's softmax)
# ----------------------------------------------------------------------------
def test_token_removal_identity():
    B, Hq, Hkv, N, W, d = 1, 1, 1, 18, 3, 8
    q, k, v = rand_case(60, B, Hq, Hkv, N, W, d)
    Z, A, O = oracle.window_attention(q, k, v)
    p = 4                                            # in the prefix: visible to all rows
    keep = [i for i in range(N) if i != p]
    O2 = window_outputs(q[0, 0], k[0, 0][keep], v[0, 0][keep])
    for r in range(W):
        a = A[0, 0, r, p]
        pred = O[0, 0, r] - a * (v[0, 0, p] - O[0, 0, r]) / (1 - a)
        np.testing.assert_allclose(O2[r], pred, rtol=1e-11, atol=1e-14)


# ----------------------------------------------------------------------------
# Independent second formulation: the expanded-norm recipe of Appendix E
# (||v-o||^2 = ||o||^2 + ||v||^2 - 2 v.o, sums over the query axis), assembled in
# torch from torch's own softmax.  Different algebra, different library.
# ----------------------------------------------------------------------------
def test_expanded_norm_recipe_agrees():
    B, Hq, Hkv, N, W, d = 2, 4, 2, 37, 7, 16
    q, k, v = rand_case(70, B, Hq, Hkv, N, W, d, scale=1.2)
    G = Hq // Hkv
    tq = torch.from_numpy(q)
    tk = torch.from_numpy(k).repeat_interleave(G, 1)
    tv = torch.from_numpy(v).repeat_interleave(G, 1)
    Z = tq @ tk.transpose(-1, -2) / d ** 0.5
    vis = torch.ones(W, N, dtype=torch.bool).tril(N - W)
    A = torch.softmax(Z.masked_fill(~vis, float("-inf")), -1)
    Zm = Z.masked_fill(~vis, 0.0)
    O = A @ tv
    v2 = tv.pow(2).sum(-1)
    o2 = O.pow(2).sum(-1)
    vo = torch.einsum("bhqd,bhpd->bhqp", O, tv)
    s_value = A.pow(2).sum(-2) * v2
    s_key = ((A * Zm).pow(2) * (o2.unsqueeze(-1) + v2.unsqueeze(-2) - 2 * vo)).sum(-2)
    s_joint = (2 * A.pow(2) * Zm * (v2.unsqueeze(-2) - vo)).sum(-2) + s_value + s_key
    sv, sk, sj = oracle.score(q, k, v)
    for mine, ref in ((sv, s_value), (sk, s_key), (sj, s_joint)):
        np.testing.assert_allclose(mine, ref.view(B, Hkv, G, N).sum(2).numpy(), rtol=1e-10, atol=1e-16)


# ----------------------------------------------------------------------------
# P12  selection and compaction
# ----------------------------------------------------------------------------
def _select_ref(scores, budget, lens=None):
    B, H, N = scores.shape
    out = np.empty((B, H, budget), dtype=np.int32)
    for b in range(B):
        L = N if lens is None else lens[b]
        for h in range(H):
            s = scores[b, h, :L].astype(np.float64)
            s = np.where(np.isnan(s), -np.inf, s)
            order = np.argsort(-s, kind="stable")      # ties keep index order -> lowest index first
            out[b, h] = np.sort(order[:budget])
    return out


def test_select_matches_stable_sort_random_and_ties():
    rng = np.random.default_rng(80)
    s = rng.random((3, 4, 257)).astype(np.float32)
    lens = [257, 100, 64]
    np.testing.assert_array_equal(oracle.select(s, 50, lens), _select_ref(s, 50, lens))
    np.testing.assert_array_equal(oracle.select(s, 257), _select_ref(s, 257))
    # quantised scores: many ties, k-th value repeated across the cut
    t = np.floor(s * 6).astype(np.float32)
    for budget in (1, 7, 64):
        np.testing.assert_array_equal(oracle.select(t, budget, lens), _select_ref(t, budget, lens))
    # all equal -> the first `budget` indices
    e = np.full((1, 1, 90), 2.5, dtype=np.float32)
    np.testing.assert_array_equal(oracle.select(e, 13)[0, 0], np.arange(13))
    # zeros of both signs tie; duplicated maxima
    z = np.zeros((1, 1, 16), dtype=np.float32)
    z[0, 0, [3, 9]] = -0.0
    z[0, 0, [12, 5]] = 7.0
    np.testing.assert_array_equal(oracle.select(z, 5)[0, 0], [0, 1, 2, 5, 12])
    # NaN ranks below everything, -inf included? no: below every number including -inf is not required;
    # NaN is never preferred over a number
    n = np.array([[[np.nan, 1.0, -1.0, np.nan, 0.5]]], dtype=np.float32)
    np.testing.assert_array_equal(oracle.select(n, 3)[0, 0], [1, 2, 4])
    np.testing.assert_array_equal(oracle.select(n, 4)[0, 0], [0, 1, 2, 4])


def test_select_rejects_bad_budget():
    s = np.zeros((1, 1, 8), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.select(s, 9)
    with pytest.raises(ValueError):
        oracle.select(s, 5, [4])


def test_compact_matches_fancy_indexing():
    rng = np.random.default_rng(90)
    k = rng.integers(0, 2 ** 16, (2, 3, 50, 8)).astype(np.uint16)    # bf16 payloads are just bytes
    v = rng.integers(0, 2 ** 16, (2, 3, 50, 8)).astype(np.uint16)
    idx = np.sort(rng.permuted(np.tile(np.arange(50), (2, 3, 1)), axis=-1)[..., :11], axis=-1).astype(np.int32)
    ko, vo = oracle.compact(k, v, idx)
    np.testing.assert_array_equal(ko, np.take_along_axis(k, idx[..., None], axis=2))
    np.testing.assert_array_equal(vo, np.take_along_axis(v, idx[..., None], axis=2))
    kf = rng.standard_normal((1, 1, 9, 4)).astype(np.float32)
    ko, _ = oracle.compact(kf, kf, np.array([[[0, 8]]], dtype=np.int32))
    np.testing.assert_array_equal(ko[0, 0], kf[0, 0, [0, 8]])


# ---- selection with protected regions (Appendix E, Algorithm 2; sinks as in the decoding setup of Appendix C) ----

def test_select_protected_is_topk_below_cutoff_plus_recent_tail():
    """Distinct scores: library top-k over S[..., :cutoff], sorted, recent rows appended (Algorithm 2's semantics)."""
    g = torch.Generator().manual_seed(81)
    S = torch.rand(2, 3, 200, generator=g)
    num_hh, num_recent, num_coming = 17, 32, 5
    cutoff = 200 - num_recent + num_coming
    hh = torch.topk(S[..., :cutoff], num_hh, dim=-1).indices.sort(dim=-1).values
    tail = torch.arange(cutoff, 200).expand(2, 3, -1)
    want = torch.cat([hh, tail], dim=-1).numpy().astype(np.int32)
    got = oracle.select_protected(S.numpy(), num_hh, 0, num_recent, num_coming)
    np.testing.assert_array_equal(got, want)
    # compaction with these indices == gather of the heavy hitters followed by the recent rows
    k = torch.randn(2, 3, 200, 4, generator=g)
    ko, _ = oracle.compact(k.numpy(), k.numpy(), got)
    k_hh = torch.gather(k[..., :cutoff, :], 2, hh.unsqueeze(-1).expand(-1, -1, -1, 4))
    np.testing.assert_array_equal(ko, torch.cat([k_hh, k[..., cutoff:, :]], dim=2).numpy())


def test_select_protected_reduces_to_plain_select():
    rng = np.random.default_rng(82)
    s = np.floor(rng.random((2, 2, 300)) * 9).astype(np.float32)         # ties everywhere
    lens = [300, 123]
    np.testing.assert_array_equal(oracle.select_protected(s, 40, 0, 0, 0, lens), oracle.select(s, 40, lens))
    np.testing.assert_array_equal(oracle.select_protected(s, 40, 0, 7, 7, lens), oracle.select(s, 40, lens))


def test_select_protected_sinks_ties_and_ragged():
    rng = np.random.default_rng(83)
    s = np.floor(rng.random((3, 2, 150)) * 5).astype(np.float32)
    s[0, 0, :4] = -1.0                                                   # sinks are kept whatever they score
    lens = [150, 61, 97]
    num_hh, sinks, recent, coming = 20, 4, 16, 3
    tail = recent - coming
    got = oracle.select_protected(s, num_hh, sinks, recent, coming, lens)
    assert got.shape == (3, 2, sinks + num_hh + tail)
    for b in range(3):
        L = lens[b]
        cutoff = L - tail
        for h in range(2):
            row = got[b, h]
            assert np.all(np.diff(row) > 0)
            np.testing.assert_array_equal(row[:sinks], np.arange(sinks))
            np.testing.assert_array_equal(row[-tail:], np.arange(cutoff, L))
            cand = np.arange(sinks, cutoff)
            order = cand[np.argsort(-s[b, h, cand].astype(np.float64), kind="stable")]
            np.testing.assert_array_equal(row[sinks:sinks + num_hh], np.sort(order[:num_hh]))
    # budget consumes every candidate; no heavy hitters at all
    np.testing.assert_array_equal(oracle.select_protected(s[:1, :1, :20], 20 - 4 - 5, 4, 5, 0)[0, 0], np.arange(20))
    np.testing.assert_array_equal(oracle.select_protected(s[:1, :1, :20], 0, 2, 3, 0)[0, 0], [0, 1, 17, 18, 19])
    with pytest.raises(ValueError):
        oracle.select_protected(s, 140, 4, 16, 3, lens)                  # does not fit the shortest sequence
    with pytest.raises(ValueError):
        oracle.select_protected(s, 5, 0, 2, 3)                           # num_coming > num_recent


# ---- pooled selection (Appendix C, SnapKV paragraph: average pooling, kernel size 5, before eviction) ----

def test_select_pooled_matches_library_avg_pool():
    """Scores that are small integers: every window sum is exact, so the library's average pooling
    (zero padding, stride 1) followed by the pinned select must give the same indices."""
    g = torch.Generator().manual_seed(84)
    S = torch.randint(0, 1000, (2, 3, 400), generator=g).to(torch.float32)
    for pool in (3, 5, 7):
        pooled = torch.nn.functional.avg_pool1d(S.double(), kernel_size=pool, stride=1, padding=pool // 2) * pool
        want = oracle.select(pooled.to(torch.float32).numpy(), 60)
        np.testing.assert_array_equal(oracle.select_pooled(S.numpy(), 60, pool=pool), want)
    np.testing.assert_array_equal(oracle.select_pooled(S.numpy(), 60, pool=1), oracle.select(S.numpy(), 60))


def test_select_pooled_window_stays_inside_candidates_and_hand_case():
    s = np.zeros((1, 1, 12), dtype=np.float32)
    s[0, 0, [0, 1]] = 100.0          # sinks: huge, but outside the candidate range -> must not leak into token 2
    s[0, 0, 5] = 9.0                 # window sums (pool 3): tokens 4,5,6 -> 9 each; token 5's neighbours tie with it
    s[0, 0, [10, 11]] = 50.0         # recent tail: always kept, must not leak into token 9
    got = oracle.select_pooled(s, 2, pool=3, num_sinks=2, num_recent=2, num_coming=0)[0, 0]
    np.testing.assert_array_equal(got, [0, 1, 4, 5, 10, 11])     # ties 4,5,6 -> lowest indices
    # ragged: the window also stops at the true length
    t = np.zeros((2, 1, 10), dtype=np.float32)
    t[1, 0, 6] = 5.0                 # beyond len 6 of sequence 1: never read
    t[:, 0, 2] = 1.0
    got = oracle.select_pooled(t, 3, pool=5, seq_lens=[10, 6])
    np.testing.assert_array_equal(got[1, 0], [0, 1, 2])          # sums: p0..p4 = 1, p5 = 0
    with pytest.raises(ValueError):
        oracle.select_pooled(t, 3, pool=4)


# ---- decoding-time accumulation (Section 4.2 closing remark; Eq. 9) ----

def test_window_score_is_sum_of_single_row_steps_with_growing_cache():
    """Eq. 9 sums independent per-row terms: a W-row causal window equals W decode steps (one query row each,
    cache length = the row's position + 1) added up.  Pins the causal mask row by row and is what
    obc_score_accumulate relies on."""
    rng = np.random.default_rng(85)
    B, Hq, Hkv, N, W, d = 2, 4, 2, 90, 6, 8
    q = rng.standard_normal((B, Hq, W, d)); k = rng.standard_normal((B, Hkv, N, d)); v = rng.standard_normal((B, Hkv, N, d))
    lens = [90, 41]
    whole = np.asarray(oracle.score(q, k, v, seq_lens=lens))
    acc = np.zeros_like(whole)
    for r in range(W):
        step_lens = [L - W + r + 1 for L in lens]
        acc += np.asarray(oracle.score(q[:, :, r:r + 1, :], k, v, seq_lens=step_lens))
    np.testing.assert_allclose(acc, whole, rtol=1e-12, atol=1e-300)


# ---- attention-only score (Eq. 8) and its l1-weighted form (Appendix C, VATP paragraph) ----

def test_attention_score_is_the_l11_change_when_a_column_of_A_is_zeroed():
    """Eq. 8 by brute force: zero column p of the window rows of A (library softmax) and take the (1,1)-norm
    of the change."""
    g = torch.Generator().manual_seed(86)
    N, W, d = 40, 5, 8
    q = torch.randn(1, 1, W, d, generator=g, dtype=torch.float64)
    k = torch.randn(1, 1, N, d, generator=g, dtype=torch.float64)
    v = torch.randn(1, 1, N, d, generator=g, dtype=torch.float64)
    Z = (q[0, 0] @ k[0, 0].T) / d ** 0.5
    vis = torch.arange(N)[None, :] <= (N - W + torch.arange(W))[:, None]
    A = torch.softmax(Z.masked_fill(~vis, float("-inf")), dim=-1)
    want = np.empty(N)
    for p in range(N):
        Ap = A.clone(); Ap[:, p] = 0.0
        want[p] = float((Ap - A).abs().sum())
    np.testing.assert_allclose(oracle.attn_score(q.numpy(), k.numpy(), v.numpy())[0, 0], want, rtol=1e-12)


def test_vatp_is_attention_score_times_l1_norm_and_ties_to_the_value_score():
    rng = np.random.default_rng(87)
    B, Hq, Hkv, N, W, d = 2, 4, 2, 60, 3, 16
    q = rng.standard_normal((B, Hq, W, d)); k = rng.standard_normal((B, Hkv, N, d)); v = rng.standard_normal((B, Hkv, N, d))
    lens = [60, 33]
    sa = oracle.attn_score(q, k, v, seq_lens=lens)
    sp = oracle.vatp_score(q, k, v, seq_lens=lens)
    l1 = np.linalg.norm(v, ord=1, axis=-1)                         # library norm
    np.testing.assert_allclose(sp, sa * l1, rtol=1e-13)
    assert np.all(sp[1, :, 33:] == 0.0)
    # scaling one value row scales only that token's score, by |alpha| (A does not depend on V)
    v2 = v.copy(); v2[0, 1, 7] *= -2.5
    sp2 = oracle.vatp_score(q, k, v2, seq_lens=lens)
    np.testing.assert_allclose(sp2[0, 1, 7], 2.5 * sp[0, 1, 7], rtol=1e-13)
    sp2[0, 1, 7] = sp[0, 1, 7]
    np.testing.assert_array_equal(sp2, sp)
    # one query head, one row, values in {-1, 0, 1}: ||v||_1 == ||v||_2^2 =: n, so VATP^2 == S^value * n
    q1 = rng.standard_normal((1, 1, 1, d)); k1 = rng.standard_normal((1, 1, N, d))
    v1 = rng.integers(-1, 2, (1, 1, N, d)).astype(np.float64)
    n = np.abs(v1).sum(-1)
    sv = oracle.score(q1, k1, v1)[0]
    np.testing.assert_allclose(oracle.vatp_score(q1, k1, v1) ** 2, sv * n, rtol=1e-12)
    # padded rows may hold NaN
    v3 = v.copy(); v3[1, :, 33:] = np.nan; k3 = k.copy(); k3[1, :, 33:] = np.nan
    np.testing.assert_array_equal(oracle.vatp_score(q, k3, v3, seq_lens=lens), sp)


# ---- head-adaptive selection (Appendix C, AdaKV paragraph: global ranking across heads, safeguard) ----

def _split_flat(flat_sorted, Hkv, N, cap):
    keep = np.full((Hkv, cap), -1, dtype=np.int32)
    counts = np.zeros(Hkv, dtype=np.int32)
    for f in flat_sorted:
        g, p = divmod(int(f), N)
        keep[g, counts[g]] = p
        counts[g] += 1
    return keep, counts


def test_select_adaptive_without_safeguard_is_a_global_topk():
    """Distinct scores, n_safe = 0: library top-k over the concatenated heads of each sequence."""
    g = torch.Generator().manual_seed(88)
    B, Hkv, N, budget = 2, 4, 150, 30
    S = torch.rand(B, Hkv, N, generator=g)
    S[:, 1] *= 3.0                                           # one head attracts most of the budget
    cap = oracle.adaptive_cap(Hkv, budget, 0, N)
    keep, counts = oracle.select_adaptive(S.numpy(), budget, 0, cap)
    for b in range(B):
        flat = torch.topk(S[b].reshape(-1), Hkv * budget).indices.sort().values.numpy()
        want_keep, want_counts = _split_flat(flat, Hkv, N, cap)
        np.testing.assert_array_equal(keep[b], want_keep)
        np.testing.assert_array_equal(counts[b], want_counts)
    assert counts[:, 1].min() > budget                       # the budget really moved between heads


def test_select_adaptive_full_safeguard_is_the_per_head_select_and_invariants():
    rng = np.random.default_rng(89)
    B, Hkv, N, budget = 3, 3, 120, 20
    s = np.floor(rng.random((B, Hkv, N)) * 7).astype(np.float32)         # ties everywhere
    lens = [120, 45, 77]
    keep, counts = oracle.select_adaptive(s, budget, budget, budget, lens)
    np.testing.assert_array_equal(keep, oracle.select(s, budget, lens))
    assert np.all(counts == budget)
    n_safe = 4                                                            # floor(0.2 * budget)
    cap = oracle.adaptive_cap(Hkv, budget, n_safe, max(lens))
    keep, counts = oracle.select_adaptive(s, budget, n_safe, cap, lens)
    safe = oracle.select(s, n_safe, lens)
    for b in range(B):
        L = lens[b]
        assert counts[b].sum() == Hkv * budget and counts[b].min() >= n_safe
        kept = np.zeros((Hkv, N), dtype=bool)
        for h in range(Hkv):
            row = keep[b, h]
            c = counts[b, h]
            assert np.all(np.diff(row[:c]) > 0) and np.all(row[c:] == -1) and row[:c].max() < L
            kept[h, row[:c]] = True
            assert kept[h, safe[b, h]].all()                              # the safeguard set is inside
        # global threshold: no dropped live non-safeguard token beats a kept non-safeguard one, ties to lower (head, index)
        issafe = np.zeros((Hkv, N), dtype=bool)
        for h in range(Hkv):
            issafe[h, safe[b, h]] = True
        live = np.zeros((Hkv, N), dtype=bool); live[:, :L] = True
        order = [(-float(s[b, h, p]), h, p) for h in range(Hkv) for p in range(L) if not issafe[h, p]]
        order.sort()
        want = set((h, p) for _, h, p in order[:Hkv * (budget - n_safe)])
        got = set(zip(*np.nonzero(kept & ~issafe & live)))
        assert got == want
    with pytest.raises(ValueError):
        oracle.select_adaptive(s, budget, budget + 1, cap, lens)
    with pytest.raises(ValueError):
        oracle.select_adaptive(s, budget, 0, 10, lens)                    # cap too small for the worst case


def test_compact_pads_negative_indices_with_zero_rows():
    rng = np.random.default_rng(91)
    k = rng.integers(1, 2 ** 16, (1, 2, 9, 8)).astype(np.uint16)
    v = rng.integers(1, 2 ** 16, (1, 2, 9, 8)).astype(np.uint16)
    idx = np.array([[[0, 3, 8, -1], [2, -1, -1, -1]]], dtype=np.int32)
    ko, vo = oracle.compact(k, v, idx)
    np.testing.assert_array_equal(ko[0, 0, :3], k[0, 0, [0, 3, 8]])
    np.testing.assert_array_equal(vo[0, 1, :1], v[0, 1, [2]])
    assert np.all(ko[0, 0, 3:] == 0) and np.all(ko[0, 1, 1:] == 0) and np.all(vo[0, 1, 1:] == 0)


def _fifty_digit_scores(mp, qn, kn, vn, lens):
    """Eq. 4-6 term by term in 50-digit arithmetic, window sum (Eq. 9) and sum over the group's query heads
    (Appendix A.5): per (sequence, KV head, token) the three scores, and the least 1 - max_p A_ip over all rows."""
    B, Hq, W, d = qn.shape
    Hkv, N = kn.shape[1], kn.shape[2]
    G = Hq // Hkv
    M = lambda a: [mp.mpf(float(x)) for x in a]
    ref = {name: [[[mp.mpf(0)] * N for _ in range(Hkv)] for _ in range(B)] for name in ("value", "key", "joint")}
    least_rest, most_rest = mp.mpf(1), mp.mpf(0)
    for b in range(B):
        L = N if lens is None else lens[b]
        for h in range(Hq):
            g = h // G
            for r in range(W):
                n_vis = L - W + r + 1
                z = [sum(a * c for a, c in zip(M(qn[b, h, r]), M(kn[b, g, p]))) / mp.sqrt(d) for p in range(n_vis)]
                zmax = max(z)
                e = [mp.exp(x - zmax) for x in z]
                tot = sum(e)
                A = [x / tot for x in e]
                least_rest = min(least_rest, 1 - max(A))
                most_rest = max(most_rest, 1 - max(A))
                o = [sum(A[p] * mp.mpf(float(vn[b, g, p, j])) for p in range(n_vis)) for j in range(d)]
                for p in range(n_vis):
                    vp = M(vn[b, g, p])
                    ref["value"][b][g][p] += A[p] ** 2 * sum(x * x for x in vp)
                    ref["key"][b][g][p] += A[p] ** 2 * z[p] ** 2 * sum((x - y) ** 2 for x, y in zip(vp, o))
                    ref["joint"][b][g][p] += A[p] ** 2 * sum(((1 + z[p]) * x - z[p] * y) ** 2 for x, y in zip(vp, o))
    return ref, least_rest, most_rest


FIFTY_DIGIT_SHAPES = {
    # name: (B, Hq, Hkv, N, W, d, true lengths)
    "mha_pair": (1, 2, 1, 24, 2, 8, None),
    "gqa4_w5_ragged_d16": (2, 8, 2, 40, 5, 16, [40, 29]),
}


@pytest.mark.parametrize("shape", list(FIFTY_DIGIT_SHAPES))
@pytest.mark.parametrize("gain", [2.0, 4.0, 6.0, 8.0])
def test_scores_of_a_key_that_takes_nearly_all_attention_match_50_digit_arithmetic(gain, shape):
    """Eq. 4-6 evaluated term by term in 50-digit arithmetic (mpmath) from the same inputs.  One key is aligned with
    every window query, so that it holds 1 - 1e-4 .. 1 - 1e-16 of each row's weight and v_p - o_i is the difference of
    two nearly equal vectors: plain fp64 loses eps / (1 - A) of that difference, the oracle must not.  Shapes: two
    query heads on one KV head; and a group of four query heads per KV head, a five-row window, a ragged batch and
    head_dim 16 (group sum, row-wise causal mask and padding all in play)."""
    import mpmath as mp                                   # (a plain import: without the module this pin must fail, not skip)
    mp.mp.dps = 50
    B, Hq, Hkv, N, W, d, lens = FIFTY_DIGIT_SHAPES[shape]
    g = torch.Generator().manual_seed(91)
    q = torch.randn(B, Hq, W, d, generator=g, dtype=torch.float64)
    k = torch.randn(B, Hkv, N, d, generator=g, dtype=torch.float64)
    v = torch.randn(B, Hkv, N, d, generator=g, dtype=torch.float64)
    u = torch.randn(d, generator=g, dtype=torch.float64)
    q = q + 3.0 * u / u.norm() * d ** 0.5              # a direction all queries share
    k[:, :, 5] = gain * u / u.norm() * d ** 0.5         # key 5 of every head points along it
    qn, kn, vn = q.numpy(), k.numpy(), v.numpy()
    sv, sk, sj = oracle.score(qn, kn, vn, seq_lens=lens)
    _, _, sj_literal = oracle.score(qn, kn, vn, seq_lens=lens, joint_form=1)
    ref, least_rest, _ = _fifty_digit_scores(mp, qn, kn, vn, lens)
    assert least_rest < mp.mpf(10) ** (-2 * gain + 1), "the case must be as lopsided as it claims (1 - A = %s)" % least_rest
    for name, got in (("value", sv), ("key", sk), ("joint", sj), ("joint", sj_literal)):
        for b in range(B):
            L = N if lens is None else lens[b]
            for h in range(Hkv):
                for p in range(N):
                    want = ref[name][b][h][p] if p < L else mp.mpf(0)
                    assert abs(mp.mpf(float(got[b, h, p])) - want) <= mp.mpf("1e-9") * want, (name, b, h, p, float(got[b, h, p]), float(want))


@pytest.mark.parametrize("gain", [0.26, 0.29, 0.32])
def test_largest_weight_branch_agrees_with_the_plain_branch_where_fp64_resolves_both(gain):
    """The oracle forms v_p - o_i of each row's largest-weight key as sum_q A_iq (v_p - v_q) (Section 3: a softmax row
    sums to one) and of every other key as the plain difference.  Where the largest weight is moderate (0.2 .. 0.6 of
    the row) fp64 resolves both forms: the same C function with the special case switched off (test-only flag) must
    then agree to 1e-12 on every token, for all three scores and both joint forms; and the 50-digit evaluation sits
    beside both."""
    import mpmath as mp
    mp.mp.dps = 50
    B, Hq, Hkv, N, W, d, lens = 2, 8, 2, 40, 5, 16, [40, 29]
    g = torch.Generator().manual_seed(92)
    q = torch.randn(B, Hq, W, d, generator=g, dtype=torch.float64)
    k = torch.randn(B, Hkv, N, d, generator=g, dtype=torch.float64)
    v = torch.randn(B, Hkv, N, d, generator=g, dtype=torch.float64)
    u = torch.randn(d, generator=g, dtype=torch.float64)
    q = 0.3 * q + 3.0 * u / u.norm() * d ** 0.5
    k = 0.3 * k
    k[:, :, 7] = gain * u / u.norm() * d ** 0.5
    qn, kn, vn = q.numpy(), k.numpy(), v.numpy()
    _, A, _ = oracle.window_attention(qn, kn, vn, seq_lens=lens)
    top = np.nanmax(np.where(np.isfinite(A), A, np.nan), axis=-1)
    assert top.min() > 0.2 and top.max() < 0.6, (top.min(), top.max())     # the case is what it claims
    ref, _, _ = _fifty_digit_scores(mp, qn, kn, vn, lens)
    for form in (0, 1):
        special = oracle.score(qn, kn, vn, seq_lens=lens, joint_form=form)
        plain = oracle.score(qn, kn, vn, seq_lens=lens, joint_form=form + 2)
        for name, a, b_ in zip(("value", "key", "joint"), special, plain):
            np.testing.assert_allclose(a, b_, rtol=1e-12, atol=0.0, err_msg="%s form %d" % (name, form))
            for b in range(B):
                for h in range(Hkv):
                    for p in range(lens[b]):
                        want = ref[name][b][h][p]
                        assert abs(mp.mpf(float(a[b, h, p])) - want) <= mp.mpf("1e-11") * want, (name, form, b, h, p)
