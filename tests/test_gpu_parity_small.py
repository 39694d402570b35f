"""GPU parity, element by element, against the fp64 CPU oracle on oracle-sized inputs.

Every call goes through the C ABI (ctypes binding).  Tolerances: scores rel 1e-5 (fp32
inputs) / 1e-3 (bf16 inputs, fp32 accumulation) measured as in parity_util.score_error;
indices bit-exact given the same fp32 scores; byte-exact compaction.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_07651_amd import binding as obc
from paper_2510_07651_amd import synth

from parity_util import TOL, run_case as _run_case, score_error, to_device

pytestmark = pytest.mark.gpu

CASES = {w.name: w for w in synth.small_cases() + synth.paper_configs()[:2]}


@pytest.mark.parametrize("name", list(CASES))
def test_score_select_compact_match_oracle(name):
    worst = _run_case(CASES[name])
    print(name, {k: "%.2e" % v for k, v in worst.items()})


@pytest.mark.parametrize("name", ["s_bf16_llama", "s_bf16_ragged", "s_bf16_strong_sink", "s_bf16_tiny", "s_bf16_max_rows",
                                  "c2_llama8b_8k"])
def test_narrow_second_sweep_matches_oracle_too(name, score_path):
    """Shapes whose second sweep runs 64 rows per wave by default, forced through the 32-rows-per-wave kernel."""
    obc.obc_set_sweep2_form(1)
    worst = _run_case(CASES[name])
    print(name, {k: "%.2e" % v for k, v in worst.items()})


def test_deterministic_bits():
    wl = CASES["s_bf16_llama"]
    dev = to_device(synth.make_inputs(wl))
    a = obc.obc_score(dev["q"], dev["k"], dev["v"], "all")
    b = obc.obc_score(dev["q"], dev["k"], dev["v"], "all")
    assert torch.equal(a, b)


def test_plain_path_switch(score_path):
    """The vector-ALU path serves bf16 head_dim-128 inputs too when asked to; it must agree with the oracle."""
    score_path("plain")
    _run_case(CASES["s_bf16_ragged"])


def test_environment_change_between_size_query_and_call(monkeypatch):
    """A workspace of exactly the queried size is accepted whatever the process environment does in between."""
    wl = CASES["s_bf16_llama"]
    x = synth.make_inputs(wl)
    dev = to_device(x)
    need = obc.obc_score_workspace_bytes(wl.B, wl.N, wl.W, wl.Hq, wl.Hkv, wl.d, obc.OBC_BF16, obc.OBC_JOINT)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    first = obc.obc_score(dev["q"], dev["k"], dev["v"], "joint", seq_lens=x["seq_lens"], workspace=ws).clone()
    for name, value in (("OBC_SCORE_PATH", "plain"), ("OBC_TUNE_SPLITS", "1"), ("OBC_TUNE_RANGE", "8192")):
        monkeypatch.setenv(name, value)
    again = obc.obc_score(dev["q"], dev["k"], dev["v"], "joint", seq_lens=x["seq_lens"], workspace=ws)
    assert torch.equal(first, again)


def test_select_crafted_ties_and_specials():
    dev = torch.device("cuda")
    rng = np.random.default_rng(5)
    cases = []
    s = np.floor(rng.random((2, 3, 5000)) * 7).astype(np.float32)            # heavy ties across the cut
    cases.append((s, 777, [5000, 4100]))
    cases.append((np.full((1, 2, 4097), 3.25, np.float32), 1000, None))       # all equal
    z = np.zeros((1, 1, 9000), np.float32); z[0, 0, ::7] = -0.0; z[0, 0, [11, 4999, 8999]] = 1.0
    cases.append((z, 10, None))                                               # zeros of both signs
    n = rng.standard_normal((1, 2, 3000)).astype(np.float32); n[0, :, ::5] = np.nan; n[0, 0, 7] = -np.inf
    cases.append((n, 2500, None))                                             # NaN below -inf, negatives
    e = rng.random((2, 2, 64)).astype(np.float32)
    cases.append((e, 64, None))                                               # budget == N
    cases.append((e, 1, [64, 1]))                                             # budget 1, len 1
    big = rng.random((1, 1, 200000)).astype(np.float32) ** 8                  # long head, tiny values
    cases.append((big, 4096, None))
    d = rng.random((1, 1, 70000)).astype(np.float32); d[0, 0, 1000:60000] = d[0, 0, 1000]
    cases.append((d, 30000, None))                                            # 59000 duplicates straddling the cut
    for s, budget, lens in cases:
        keep = obc.obc_select(torch.from_numpy(s).to(dev), budget, seq_lens=lens).cpu().numpy()
        np.testing.assert_array_equal(keep, oracle.select(s, budget, lens))


def test_select_protected_matches_oracle():
    """Algorithm 2's recent tail and cutoff, plus always-kept sinks: bit-exact indices, then the compacted rows."""
    dev = torch.device("cuda")
    rng = np.random.default_rng(6)
    cases = []
    s = rng.random((2, 3, 5000)).astype(np.float32)
    cases.append((s, dict(num_hh=700, num_sinks=4, num_recent=256, num_coming=1), [5000, 3111]))
    cases.append((s, dict(num_hh=700, num_sinks=0, num_recent=64, num_coming=0), None))
    cases.append((s, dict(num_hh=40, num_sinks=0, num_recent=0, num_coming=0), None))      # plain select
    t = np.floor(rng.random((1, 2, 9000)) * 5).astype(np.float32)                          # ties across the cut
    t[0, 0, :4] = -3.0                                                                     # sinks kept whatever they score
    t[0, 1, -20:] = np.nan                                                                 # so is the recent tail
    cases.append((t, dict(num_hh=1000, num_sinks=4, num_recent=20, num_coming=0), None))
    cases.append((t, dict(num_hh=0, num_sinks=2, num_recent=3, num_coming=1), None))       # no heavy hitters
    cases.append((t[:, :, :64], dict(num_hh=64 - 4 - 7, num_sinks=4, num_recent=8, num_coming=1), None))  # keep all
    big = rng.random((1, 2, 100000)).astype(np.float32)                                    # streamed (non-resident) kernel
    cases.append((big, dict(num_hh=764, num_sinks=4, num_recent=256, num_coming=0), [99000]))
    for s, kw, lens in cases:
        keep = obc.obc_select_protected(torch.from_numpy(s).to(dev), seq_lens=lens, **kw).cpu().numpy()
        np.testing.assert_array_equal(keep, oracle.select_protected(s, seq_lens=lens, **kw))
    # evict_kv of Algorithm 2 end to end: gather with these indices == [heavy hitters ; recent rows]
    g = torch.Generator().manual_seed(4)
    k = torch.randn(2, 3, 5000, 128, generator=g).to(torch.bfloat16); v = torch.randn(2, 3, 5000, 128, generator=g).to(torch.bfloat16)
    s, kw, lens = cases[0]
    keep = obc.obc_select_protected(torch.from_numpy(s).to(dev), seq_lens=lens, **kw)
    ko, vo = obc.obc_compact(k.to(dev), v.to(dev), keep)
    kref, vref = oracle.compact(k.view(torch.int16).numpy(), v.view(torch.int16).numpy(), keep.cpu().numpy())
    np.testing.assert_array_equal(ko.view(torch.int16).cpu().numpy(), kref)
    np.testing.assert_array_equal(vo.view(torch.int16).cpu().numpy(), vref)
    tail = kw["num_recent"] - kw["num_coming"]
    assert torch.equal(ko[0, 0, -tail:].cpu(), k[0, 0, 5000 - tail:])                      # the recent rows, in order


def test_select_pooled_matches_oracle():
    """Average-pooled ranking (window sums in fp32, fixed order): indices bit-exact against the oracle."""
    dev = torch.device("cuda")
    rng = np.random.default_rng(7)
    s = (rng.random((2, 3, 6000)).astype(np.float32)) ** 6                 # spread over many binades: sums do round
    s[0, 0, 100:140] = np.nan                                              # NaN poisons its neighbours' windows on both sides alike
    big = rng.random((1, 1, 70001)).astype(np.float32)                     # streamed kernel, odd length (scalar tail loads)
    cases = [
        (s, dict(num_hh=600, pool=5), None),
        (s, dict(num_hh=600, pool=5, num_sinks=4, num_recent=64, num_coming=0), [6000, 2501]),
        (s, dict(num_hh=50, pool=3, num_sinks=1, num_recent=7, num_coming=2), [5999, 64]),
        (s, dict(num_hh=333, pool=15), None),
        (s, dict(num_hh=333, pool=1, num_sinks=2, num_recent=5), None),
        (np.floor(s * 50).astype(np.float32), dict(num_hh=777, pool=7), None),   # heavy ties
        (big, dict(num_hh=4096, pool=5, num_sinks=4, num_recent=64), None),
    ]
    for s_, kw, lens in cases:
        keep = obc.obc_select_pooled(torch.from_numpy(s_).to(dev), seq_lens=lens, **kw).cpu().numpy()
        np.testing.assert_array_equal(keep, oracle.select_pooled(s_, seq_lens=lens, **kw))


def test_compact_fp32_and_edge_rows():
    dev = torch.device("cuda")
    g = torch.Generator().manual_seed(3)
    k = torch.randn(2, 3, 100, 64, generator=g); v = torch.randn(2, 3, 100, 64, generator=g)
    idx = torch.stack([torch.stack([torch.randperm(100, generator=g)[:17].sort().values for _ in range(3)])
                       for _ in range(2)]).to(torch.int32)
    idx[0, 0, 0] = 0; idx[0, 0, -1] = 99
    ko, vo = obc.obc_compact(k.to(dev), v.to(dev), idx.to(dev))
    kref, vref = oracle.compact(k.numpy(), v.numpy(), idx.numpy())
    np.testing.assert_array_equal(ko.cpu().numpy(), kref)
    np.testing.assert_array_equal(vo.cpu().numpy(), vref)


def test_runtime_errors_surface():
    dev = torch.device("cuda")
    q = torch.zeros(1, 2, 4, 128, device=dev, dtype=torch.bfloat16)
    k = torch.zeros(1, 1, 64, 128, device=dev, dtype=torch.bfloat16)
    with pytest.raises(obc.ObcError) as e:
        obc.obc_score(q, k, k.clone(), "joint", seq_lens=[3])        # W > len
    assert e.value.status == obc.OBC_EINVAL
    with pytest.raises(obc.ObcError):
        obc.obc_select(torch.zeros(1, 1, 8, device=dev), 9)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_decode_accumulation_matches_oracle(dtype):
    """Prefill scores, then T decode steps (W = 1, cache one token longer each step) accumulated in place."""
    wl = synth.Workload("decode_" + dtype, B=2, Hq=8, Hkv=2, d=128, N=700, W=16, dtype=dtype, budget=64, seed=31,
                        sinks=2, outlier_channels=2)
    x = synth.make_inputs(wl)
    dev = to_device(x)
    T, L0 = 24, [600, 333]                                # prefill lengths; the cache grows to L0 + T
    tol = TOL[dtype]
    g = torch.Generator().manual_seed(32)
    qd = torch.randn(T, wl.B, wl.Hq, 1, wl.d, generator=g).to(x["q"].dtype)
    ref = np.asarray(oracle.score(x["q"], x["k"], x["v"], seq_lens=L0))
    run = obc.obc_score(dev["q"], dev["k"], dev["v"], "all", seq_lens=L0)
    sentinel = 123.0
    for b in range(wl.B):
        run[:, b, :, L0[b] + T:] = sentinel               # positions no step reaches must stay untouched
    for t in range(T):
        lens_t = [L + t + 1 for L in L0]
        ref += np.asarray(oracle.score(qd[t], x["k"], x["v"], seq_lens=lens_t))
        obc.obc_score(qd[t].cuda(), dev["k"], dev["v"], "all", seq_lens=lens_t, scores=run, accumulate=True)
    torch.cuda.synchronize()
    final = [L + T for L in L0]
    for vi, name in enumerate(synth.VARIANTS):
        gpu = run[vi].cpu().numpy()
        for b in range(wl.B):
            assert np.all(gpu[b, :, final[b]:] == sentinel), name
            gpu[b, :, final[b]:] = 0.0
        err, where = score_error(gpu, ref[vi], wl.budget, final, tol)
        assert err <= tol, "%s: err %.3g at %s" % (name, err, where)
    # single-variant accumulation takes the same path as the all-variant one
    one = obc.obc_score(dev["q"], dev["k"], dev["v"], "joint", seq_lens=L0)
    obc.obc_score(qd[0].cuda(), dev["k"], dev["v"], "joint", seq_lens=[L + 1 for L in L0], scores=one, accumulate=True)
    two = obc.obc_score(dev["q"], dev["k"], dev["v"], "joint", seq_lens=L0)
    inc = obc.obc_score(qd[0].cuda(), dev["k"], dev["v"], "joint", seq_lens=[L + 1 for L in L0])
    for b in range(wl.B):
        n = L0[b] + 1
        assert torch.equal(one[b, :, :n], two[b, :, :n] + inc[b, :, :n])


def test_accumulate_onto_zeros_equals_plain_call_with_several_row_chunks():
    """G*W = 448 window rows: four row chunks whose planes are summed by a second kernel; that path accumulates too."""
    wl = CASES["s_bf16_qwen"]
    dev = to_device(synth.make_inputs(wl))
    plain = obc.obc_score(dev["q"], dev["k"], dev["v"], "all")
    run = torch.zeros_like(plain)
    obc.obc_score(dev["q"], dev["k"], dev["v"], "all", scores=run, accumulate=True)
    assert torch.equal(run, plain)
    obc.obc_score(dev["q"], dev["k"], dev["v"], "all", scores=run, accumulate=True)
    assert torch.equal(run, plain + plain)


@pytest.mark.parametrize("in_place", [False, True, "one call"])
def test_decode_eviction_loop_matches_oracle(in_place):
    """The decoding setup of Appendix C in miniature: every step appends a token, accumulates its scores, and once the
    cache is over budget evicts one token per head with sinks and a recent window protected.  The oracle runs the same
    loop in fp64; eviction decisions are taken on the same fp32 running scores on both sides and must be identical."""
    B, Hq, Hkv, d = 2, 8, 2, 128
    sinks, recent, hh = 4, 24, 36
    budget = sinks + recent + hh                                  # 64 cache slots after an eviction
    cap = budget + 1
    T = 150
    g = torch.Generator().manual_seed(41)
    qs = torch.randn(T, B, Hq, 1, d, generator=g).to(torch.bfloat16)
    ks = torch.randn(T, B, Hkv, d, generator=g).to(torch.bfloat16); ks[:, :, :, :3] *= 6.0
    vs = torch.randn(T, B, Hkv, d, generator=g).to(torch.bfloat16)
    dev = torch.device("cuda")
    k = torch.zeros(B, Hkv, cap, d, dtype=torch.bfloat16, device=dev); v = torch.zeros_like(k)
    run = torch.zeros(B, Hkv, cap, dtype=torch.float32, device=dev)
    k_ref = np.zeros((B, Hkv, cap, d), np.float64); v_ref = np.zeros_like(k_ref)
    run_ref = np.zeros((B, Hkv, cap), np.float64)
    one_call = in_place == "one call"
    if one_call:
        kf, vf, runf = k.clone(), v.clone(), run.clone()
    length, evictions = 0, 0
    for t in range(T):
        k[:, :, length] = ks[t].to(dev); v[:, :, length] = vs[t].to(dev)
        k_ref[:, :, length] = ks[t].double().numpy(); v_ref[:, :, length] = vs[t].double().numpy()
        length += 1
        lens = [length] * B
        if one_call:
            # The same step through obc_decode_step on a cache of its own: one call accumulates, drops one token per
            # head and closes the gap.  The three-call path below is held to the oracle; the one call must agree with it
            # bit for bit, and report the position it dropped.
            kf[:, :, length - 1] = ks[t].to(dev); vf[:, :, length - 1] = vs[t].to(dev)
            if length > budget:
                evicted = obc.obc_decode_step(qs[t].to(dev), kf, vf, runf, "joint", sinks, recent, seq_lens=lens).cpu().numpy()
            else:
                obc.obc_score(qs[t].to(dev), kf, vf, "joint", seq_lens=lens, scores=runf, accumulate=True)
        obc.obc_score(qs[t].to(dev), k, v, "joint", seq_lens=lens, scores=run, accumulate=True)
        run_ref += np.asarray(oracle.score(qs[t].double().numpy(), k_ref, v_ref, seq_lens=lens))[2]
        if length > budget:
            keep = obc.obc_select_protected(run, hh, sinks, recent, 0, seq_lens=lens)
            keep_np = keep.cpu().numpy()
            np.testing.assert_array_equal(keep_np, oracle.select_protected(run.cpu().numpy(), hh, sinks, recent, 0, lens))
            if one_call:
                for b in range(B):
                    for h in range(Hkv):
                        gone = np.setdiff1d(np.arange(length), keep_np[b, h])
                        assert gone.tolist() == [int(evicted[b, h])], (t, b, h, gone, evicted[b, h])
            if in_place:
                obc.obc_compact_inplace(k, v, keep, scores=run)
                k[:, :, budget:] = 0; v[:, :, budget:] = 0        # stale rows; cleared only to compare whole caches below
            else:
                ko, vo = obc.obc_compact(k, v, keep)
                new_run = obc.obc_compact_scores(run, keep, n_out=cap)
                k = torch.zeros_like(k); v = torch.zeros_like(v)
                k[:, :, :budget] = ko; v[:, :, :budget] = vo
                run = new_run
            idx = keep_np[..., None]
            k_new = np.zeros_like(k_ref); v_new = np.zeros_like(v_ref); r_new = np.zeros_like(run_ref)
            k_new[:, :, :budget] = np.take_along_axis(k_ref, idx, axis=2)
            v_new[:, :, :budget] = np.take_along_axis(v_ref, idx, axis=2)
            r_new[:, :, :budget] = np.take_along_axis(run_ref, keep_np, axis=2)
            k_ref, v_ref, run_ref = k_new, v_new, r_new
            length = budget
            evictions += 1
            np.testing.assert_array_equal(k.double().cpu().numpy(), k_ref)         # the caches stay identical
            assert np.all(run.cpu().numpy()[:, :, budget:] == 0.0)
            if one_call:
                assert torch.equal(kf[:, :, :budget], k[:, :, :budget]) and torch.equal(vf[:, :, :budget], v[:, :, :budget])
                assert torch.equal(runf, run), "step %d" % t
        if t % 10 == 9 or t == T - 1:
            err, where = score_error(run.cpu().numpy(), run_ref, min(hh, length), [length] * B, TOL["bf16"])
            assert err <= TOL["bf16"], "step %d: err %.3g at %s" % (t, err, where)
    assert evictions == T - budget


@pytest.mark.parametrize("name", ["s_fp32_gqa_ragged", "s_bf16_llama", "s_bf16_ragged", "s_bf16_qwen", "s_bf16_w1",
                                  "s_bf16_strong_sink", "s_bf16_d64", "s_bf16_max_batch", "c1_single_head_fp32"])
def test_attention_only_and_vatp_scores_match_oracle(name):
    """Eq. 8 (sum of attention weights) and the l1-weighted form the paper reproduces VATP with."""
    wl = CASES[name]
    x = synth.make_inputs(wl)
    dev = to_device(x)
    lens = x["seq_lens"]
    tol = TOL[wl.dtype]
    for variant, ref in (("attn", oracle.attn_score(x["q"], x["k"], x["v"], seq_lens=lens)),
                         ("vatp", oracle.vatp_score(x["q"], x["k"], x["v"], seq_lens=lens))):
        gpu = obc.obc_score(dev["q"], dev["k"], dev["v"], variant, seq_lens=lens)
        assert gpu.shape == (wl.B, wl.Hkv, wl.N)
        g = gpu.cpu().numpy()
        assert np.isfinite(g).all() and (g >= 0).all()
        err, where = score_error(g, ref, wl.budget, lens, tol)
        assert err <= tol, "%s %s: err %.3g at %s" % (name, variant, err, where)
        keep = obc.obc_select(gpu, wl.budget, seq_lens=lens).cpu().numpy()
        np.testing.assert_array_equal(keep, oracle.select(g, wl.budget, lens))


def test_select_sliced_and_single_block_paths_agree_with_oracle():
    """Few long heads take the sliced five-kernel path when scratch is available; the one-block-per-head path
    (workspace=False) must return the same indices, and both the oracle's."""
    dev = torch.device("cuda")
    rng = np.random.default_rng(8)
    cases = [
        (rng.random((1, 4, 131072)).astype(np.float32) ** 10, dict(num_hh=4096), None),
        (np.floor(rng.random((2, 3, 50000)) * 3).astype(np.float32), dict(num_hh=20000), [50000, 20001]),   # ties everywhere
        (rng.standard_normal((1, 1, 32769)).astype(np.float32), dict(num_hh=1, num_sinks=0), None),
        (rng.random((3, 2, 40000)).astype(np.float32), dict(num_hh=764, num_sinks=4, num_recent=256, pool=5),
         [40000, 8193, 1024]),
        (np.zeros((1, 2, 33000), np.float32), dict(num_hh=32999), None),                                     # all equal
    ]
    for s, kw, lens in cases:
        B, H, N = s.shape
        assert obc.obc_select_workspace_bytes(B, H, N) > 0
        st = torch.from_numpy(s).to(dev)
        a = obc.obc_select_pooled(st, seq_lens=lens, **kw).cpu().numpy()
        b = obc.obc_select_pooled(st, seq_lens=lens, workspace=False, **kw).cpu().numpy()
        want = oracle.select_pooled(s, seq_lens=lens, **kw)
        np.testing.assert_array_equal(a, want)
        np.testing.assert_array_equal(b, want)
    assert obc.obc_select_workspace_bytes(4, 8, 32768) == 0        # fits one block's registers


def test_compact_scores_matches_indexing():
    dev = torch.device("cuda")
    rng = np.random.default_rng(9)
    s = rng.standard_normal((3, 2, 1000)).astype(np.float32)
    idx = np.sort(rng.permuted(np.tile(np.arange(1000), (3, 2, 1)), axis=-1)[..., :77], axis=-1).astype(np.int32)
    for n_out in (77, 78, 300):
        out = obc.obc_compact_scores(torch.from_numpy(s).to(dev), torch.from_numpy(idx).to(dev), n_out=n_out).cpu().numpy()
        np.testing.assert_array_equal(out[..., :77], np.take_along_axis(s, idx, axis=-1))
        assert np.all(out[..., 77:] == 0.0) and out.shape == (3, 2, n_out)
    with pytest.raises(obc.ObcError):
        obc.obc_compact_scores(torch.from_numpy(s).to(dev), torch.from_numpy(idx).to(dev), n_out=10)


def test_select_on_scores_that_start_off_a_16_byte_boundary():
    """A view into a larger buffer: only 4-byte aligned, so the kernels must not use their 128-bit loads."""
    dev = torch.device("cuda")
    rng = np.random.default_rng(10)
    for shape, budget in (((2, 3, 5001), 300), ((1, 2, 40003), 4000)):
        s = rng.random(shape).astype(np.float32)
        buf = torch.zeros(s.size + 3, dtype=torch.float32, device=dev)
        for off in (1, 3):
            view = buf[off:off + s.size].view(shape)
            view.copy_(torch.from_numpy(s))
            assert view.data_ptr() % 16 != 0
            keep = obc.obc_select(view, budget).cpu().numpy()
            np.testing.assert_array_equal(keep, oracle.select(s, budget))


def test_select_adaptive_matches_oracle_and_compacts_ragged_lists():
    """Head-adaptive budgets (global ranking across the KV heads with a per-head safeguard): counts and index lists
    bit-exact against the oracle; obc_compact turns the -1 padding into zero rows."""
    dev = torch.device("cuda")
    rng = np.random.default_rng(11)
    skew = rng.random((2, 4, 3000)).astype(np.float32) ** 4
    skew[:, 2] *= 20.0                                                     # one head attracts the budget
    ties = np.floor(rng.random((3, 3, 700)) * 4).astype(np.float32)
    long_heads = rng.random((1, 8, 32768)).astype(np.float32) ** 8         # the flattened row takes the sliced path
    nanny = rng.standard_normal((1, 2, 500)).astype(np.float32); nanny[0, :, ::7] = np.nan
    cases = [
        (skew, 300, 60, None),
        (skew, 300, 0, [3000, 1234]),
        (skew, 300, 300, [3000, 1234]),                                    # full safeguard == per-head select
        (ties, 100, 20, [700, 100, 333]),
        (long_heads, 2048, 409, None),
        (nanny, 200, 40, None),
        (ties[:, :1], 50, 10, None),                                       # a single KV head
    ]
    for s, budget, n_safe, lens in cases:
        st = torch.from_numpy(s).to(dev)
        keep, counts = obc.obc_select_adaptive(st, budget, n_safe, seq_lens=lens)
        want_keep, want_counts = oracle.select_adaptive(s, budget, n_safe, keep.shape[-1], lens)
        np.testing.assert_array_equal(counts.cpu().numpy(), want_counts)
        np.testing.assert_array_equal(keep.cpu().numpy(), want_keep)
    # ragged lists through the gather: padded entries give zero rows
    s, budget, n_safe, lens = cases[0]
    g = torch.Generator().manual_seed(5)
    k = torch.randn(2, 4, 3000, 128, generator=g).to(torch.bfloat16); v = torch.randn(2, 4, 3000, 128, generator=g).to(torch.bfloat16)
    keep, counts = obc.obc_select_adaptive(torch.from_numpy(s).to(dev), budget, n_safe)
    ko, vo = obc.obc_compact(k.to(dev), v.to(dev), keep)
    kref, vref = oracle.compact(k.view(torch.int16).numpy(), v.view(torch.int16).numpy(), keep.cpu().numpy())
    np.testing.assert_array_equal(ko.view(torch.int16).cpu().numpy(), kref)
    np.testing.assert_array_equal(vo.view(torch.int16).cpu().numpy(), vref)
    c = int(counts[0, 0])
    assert c < keep.shape[-1] and torch.all(ko[0, 0, c:] == 0)


@pytest.mark.parametrize("dtype,d,N", [("bf16", 128, 1000), ("bf16", 64, 1000), ("fp32", 128, 1000), ("fp32", 20, 1000),
                                       ("bf16", 128, 9000)])
def test_compact_inplace_matches_oracle_gather(dtype, d, N):
    """Appendix D's "specialised kernel for cache eviction": the in-place form must leave exactly what the oracle's
    gather gives in rows [0, budget), leave the rows behind untouched, move the scores along and zero their tail.
    The longest case spans several chunks of the kernel's walk and its search for the first row that moves."""
    B, Hkv = 3, 2
    g = torch.Generator().manual_seed(61)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    k = torch.randn(B, Hkv, N, d, generator=g).to(dt); v = torch.randn(B, Hkv, N, d, generator=g).to(dt)
    s = torch.rand(B, Hkv, N, generator=g)
    bits = (lambda t: t.view(torch.int16)) if dtype == "bf16" else (lambda t: t.view(torch.int32))
    lists = {
        "evict_one": lambda n: np.delete(np.arange(n), n // 3),
        "evict_first": lambda n: np.arange(1, n),
        "evict_last": lambda n: np.arange(n - 1),
        "keep_everything": lambda n: np.arange(n),
        "keep_tail": lambda n: np.arange(n - 130, n),
        "random_third": lambda n: np.sort(np.random.default_rng(62).choice(n, n // 3, replace=False)),
        "random_most": lambda n: np.sort(np.random.default_rng(64).choice(n, n - n // 10, replace=False)),
        "evict_late": lambda n: np.delete(np.arange(n), n - 7),
        "one_row": lambda n: np.array([n - 1]),
    }
    for name, make in lists.items():
        base = make(N)
        keep = np.stack([np.stack([base if (b + h) % 2 == 0 or name != "random_third" else
                                   np.sort(np.random.default_rng(63 + b).choice(N, len(base), replace=False))
                                   for h in range(Hkv)]) for b in range(B)]).astype(np.int32)
        budget = keep.shape[-1]
        kd, vd, sd = k.cuda(), v.cuda(), s.cuda()
        obc.obc_compact_inplace(kd, vd, torch.from_numpy(keep).cuda(), scores=sd)
        kref, vref = oracle.compact(bits(k).numpy(), bits(v).numpy(), keep)
        np.testing.assert_array_equal(bits(kd).cpu().numpy()[:, :, :budget], kref, err_msg=name)
        np.testing.assert_array_equal(bits(vd).cpu().numpy()[:, :, :budget], vref, err_msg=name)
        np.testing.assert_array_equal(bits(kd).cpu().numpy()[:, :, budget:], bits(k).numpy()[:, :, budget:], err_msg=name)
        np.testing.assert_array_equal(bits(vd).cpu().numpy()[:, :, budget:], bits(v).numpy()[:, :, budget:], err_msg=name)
        np.testing.assert_array_equal(sd.cpu().numpy()[:, :, :budget], np.take_along_axis(s.numpy(), keep, axis=2))
        assert np.all(sd.cpu().numpy()[:, :, budget:] == 0.0), name
        # without scores the cache moves all the same
        kd2, vd2 = k.cuda(), v.cuda()
        obc.obc_compact_inplace(kd2, vd2, torch.from_numpy(keep).cuda())
        assert torch.equal(bits(kd2), bits(kd)) and torch.equal(bits(vd2), bits(vd)), name
    # a ragged list padded with -1 (what obc_select_adaptive returns) gives zero rows and zero scores
    keep = np.full((B, Hkv, 40), -1, np.int32)
    keep[:, :, :25] = np.arange(5, 30)
    kd, vd, sd = k.cuda(), v.cuda(), s.cuda()
    obc.obc_compact_inplace(kd, vd, torch.from_numpy(keep).cuda(), scores=sd)
    kref, vref = oracle.compact(bits(k).numpy(), bits(v).numpy(), keep)
    np.testing.assert_array_equal(bits(kd).cpu().numpy()[:, :, :40], kref)
    np.testing.assert_array_equal(bits(vd).cpu().numpy()[:, :, :40], vref)
    assert np.all(sd.cpu().numpy()[:, :, 25:] == 0.0)
    np.testing.assert_array_equal(sd.cpu().numpy()[:, :, :25], s.numpy()[:, :, 5:30])


@pytest.mark.parametrize("variant,Hq,Hkv,d,dtype", [("key", 8, 2, 128, torch.bfloat16), ("value", 8, 2, 128, torch.bfloat16),
                                                    ("joint", 8, 2, 128, torch.bfloat16), ("joint", 7, 1, 128, torch.bfloat16),
                                                    ("joint", 4, 2, 64, torch.bfloat16), ("joint", 4, 2, 64, torch.float32),
                                                    ("attn", 8, 2, 128, torch.bfloat16)])
def test_decode_step_on_a_ragged_batch_with_ties(variant, Hq, Hkv, d, dtype):
    """obc_decode_step on sequences of different lengths, one of them with every candidate tied (zero query, equal
    value rows: Eq. 4-6 then give every token the same score): the accumulated scores equal obc_score's own, the
    dropped position is the oracle's choice on those fp32 scores (lowest score, the later position among equals, sinks
    and the recent window exempt), and K, V and scores close the gap exactly."""
    B, N = 3, 200
    sinks, recent = 4, 16
    lens = [200, 77, 131]
    g = torch.Generator().manual_seed(97)
    q = torch.randn(B, Hq, 1, d, generator=g).to(dtype)
    k = torch.randn(B, Hkv, N, d, generator=g).to(dtype)
    v = torch.randn(B, Hkv, N, d, generator=g).to(dtype)
    run = torch.rand(B, Hkv, N, generator=g) * 0.01
    q[1] = 0; v[1] = v[1, :, :1]; run[1] = 0.25                       # sequence 1: all tied
    for b, L in enumerate(lens):
        run[b, :, L:] = 0
    dev = torch.device("cuda")
    q, k, v, run = q.to(dev), k.to(dev), v.to(dev), run.to(dev)
    acc = run.clone()
    obc.obc_score(q, k, v, variant, seq_lens=lens, scores=acc, accumulate=True)
    k0, v0 = k.clone(), v.clone()
    evicted = obc.obc_decode_step(q, k, v, run, variant, sinks, recent, seq_lens=lens).cpu().numpy()
    acc_np = acc.cpu().numpy()
    for b, L in enumerate(lens):
        keep = oracle.select_protected(acc_np[b:b + 1], L - sinks - recent - 1, sinks, recent, 0, [L])[0]     # [Hkv, L-1]
        for h in range(Hkv):
            gone = np.setdiff1d(np.arange(L), keep[h])
            assert gone.tolist() == [int(evicted[b, h])], (b, h, gone, evicted[b, h])
            if b == 1:
                assert evicted[b, h] == L - recent - 1
            idx = torch.from_numpy(keep[h]).long().to(dev)
            assert torch.equal(k[b, h, :L - 1], k0[b, h].index_select(0, idx))
            assert torch.equal(v[b, h, :L - 1], v0[b, h].index_select(0, idx))
            assert torch.equal(run[b, h, :L - 1], acc[b, h].index_select(0, idx))
            assert (run[b, h, L - 1:] == 0).all()
            assert torch.equal(k[b, h, L:], k0[b, h, L:])             # rows past the sequence are left alone
