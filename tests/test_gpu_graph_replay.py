"""The hot path under HIP graph capture: a captured score -> select -> compact step replays to the eager bits.

Serving loops capture their per-layer work once and replay it; the library's entry points only launch kernels on the
caller's stream (no allocation, no memset, no synchronisation), so a step can be captured as it is.  Every replay is
checked against the eager result, with eager work and synchronisations between the replays, on the matrix-core
route (prefill window) and on the decode route (one-row window, accumulate + in-place compaction).
"""
import pytest
import torch

from paper_2510_07651_amd import binding as obc
from paper_2510_07651_amd import synth

pytestmark = pytest.mark.gpu


def _capture(fn):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()                                   # first call outside the capture: one-time function attributes are set here
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        fn()
    torch.cuda.synchronize()
    return g


def test_prefill_step_replays_bit_exact():
    wl = synth.Workload("g_prefill", B=2, Hq=8, Hkv=2, d=128, N=3000, W=32, dtype="bf16", budget=300, seed=71, sinks=4,
                        outlier_channels=4, shared_query=0.7, sink_gain=2.0)
    x = synth.make_inputs(wl)
    q, k, v = (x[n].cuda() for n in ("q", "k", "v"))
    var = obc.VARIANT_CODES["joint"]
    ws = torch.empty(obc.obc_score_workspace_bytes(wl.B, wl.N, wl.W, wl.Hq, wl.Hkv, wl.d, obc.OBC_BF16, var),
                     dtype=torch.uint8, device="cuda")
    scores = torch.empty(wl.B, wl.Hkv, wl.N, dtype=torch.float32, device="cuda")
    keep = torch.empty(wl.B, wl.Hkv, wl.budget, dtype=torch.int32, device="cuda")
    k_out = torch.empty(wl.B, wl.Hkv, wl.budget, wl.d, dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)

    def step():
        obc.obc_score(q, k, v, var, scores=scores, workspace=ws)
        obc.obc_select(scores, wl.budget, keep_idx=keep)
        obc.obc_compact(k, v, keep, k_out=k_out, v_out=v_out)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (scores, keep, k_out, v_out)]
    g = _capture(step)
    for rep in range(4):
        for t in (scores, keep, k_out, v_out):
            t.zero_()
        ws.random_(0, 255)                      # stale workspace contents must not matter
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, (scores, keep, k_out, v_out)):
            assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.int16) if b.dtype == torch.bfloat16 else b), "replay %d" % rep
        step()                                  # eager work between the replays
        torch.cuda.synchronize()


def test_decode_step_replays_bit_exact():
    B, Hq, Hkv, d, N = 2, 8, 2, 128, 700
    gen = torch.Generator().manual_seed(72)
    q = torch.randn(B, Hq, 1, d, generator=gen).to(torch.bfloat16).cuda()
    k0 = torch.randn(B, Hkv, N, d, generator=gen).to(torch.bfloat16).cuda()
    v0 = torch.randn(B, Hkv, N, d, generator=gen).to(torch.bfloat16).cuda()
    run0 = torch.rand(B, Hkv, N, generator=gen).cuda()
    var = obc.VARIANT_CODES["joint"]
    ws = torch.empty(obc.obc_score_workspace_bytes(B, N, 1, Hq, Hkv, d, obc.OBC_BF16, var), dtype=torch.uint8,
                     device="cuda")
    k, v, run = k0.clone(), v0.clone(), run0.clone()
    keep = torch.empty(B, Hkv, N - 1, dtype=torch.int32, device="cuda")

    def step():
        obc.obc_score(q, k, v, var, scores=run, workspace=ws, accumulate=True)
        obc.obc_select_protected(run, N - 1 - 4 - 64, 4, 64, 0, keep_idx=keep)
        obc.obc_compact_inplace(k, v, keep, scores=run)

    def reset():
        k.copy_(k0); v.copy_(v0); run.copy_(run0)

    reset()
    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (k.view(torch.int16), v.view(torch.int16), run, keep)]
    reset()
    g = _capture(step)
    for rep in range(4):
        reset()
        keep.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, (k.view(torch.int16), v.view(torch.int16), run, keep)):
            assert torch.equal(a, b), "replay %d" % rep
        reset()
        step()
        torch.cuda.synchronize()
