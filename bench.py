#!/usr/bin/env python3
"""Benchmark of the OBCache hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch already resident in HBM:
obc_score (joint variant) -> obc_select -> obc_compact, through the C ABI.  The default
workload is the one the headline metric is quoted on: c3, one LLaMA-3.1-8B-shaped layer
(32 query / 8 KV heads, d=128, W=32, bf16), batch 4, N=32768, budget 2048.

Prints ONE JSON line: whole-path throughput in scored KV tokens/s, the HBM roofline of the
scoring call (algorithmic bytes: K and V once, Q, scores) from its duration inside the timed
region (events on the launch stream), per-kernel durations, and the fp64 CPU oracle timed on a
bounded sample of the same workload (a reported baseline, not a target).

Order of a run: the oracle on the CPU; the side measurements (streaming-read probe, sink-dominated
inputs, two streams, per-stage loops); W untimed steps; exactly K timed steps between two
synchronisations; parity diagnostics against the oracle's sample.  Steps and stage loops alternate
between two input sets and share one workspace and one set of outputs (a stage loop re-runs one
stage on whatever the workspace holds: fine for its duration, which does not depend on the values).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # Defaults: ~0.1 s of untimed steps first.  The GPU's clock management needs tens of milliseconds of load to
    # settle (the first 30 steps after idle run ~15 % slower than the 100th); the metric is steady-state throughput.
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--variant", default="joint")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plain", action="store_true",
                    help="skip the side measurements (two streams, sink-dominated inputs): for runs under a profiler, whose "
                         "per-kernel durations they would blur")
    ap.add_argument("--timed-first", action="store_true",
                    help="run the timed region before the side measurements instead of after them")
    ap.add_argument("--cpu-seqs", type=int, default=0, help="sequences the oracle is timed on (0 = the whole batch)")
    ap.add_argument("--decode", action="store_true",
                    help="time one decoding step per layer instead (W=1 accumulate, evict one token, compact); "
                         "a side measurement, not the headline metric")
    ap.add_argument("--cache", type=int, default=1025, help="--decode: tokens in the cache when the step starts")
    ap.add_argument("--batch", type=int, default=1, help="--decode: sequences")
    return ap.parse_args()


def decode_step_bench(args, torch, obc):
    """One decoding step of a Llama-3.1-8B-shaped layer in the paper's decoding setup (Appendix C: 4 sinks, 256
    recent tokens, the rest heavy hitters): accumulate the new row's scores, evict one token per head, move the
    cache and the scores.  Prints one JSON line of per-layer latencies in microseconds."""
    dev = torch.device("cuda:0")
    B, N, Hq, Hkv, d = args.batch, args.cache, 32, 8, 128
    g = torch.Generator().manual_seed(7)
    q = torch.randn(B, Hq, 1, d, generator=g).to(torch.bfloat16).to(dev)
    k = torch.randn(B, Hkv, N, d, generator=g).to(torch.bfloat16).to(dev)
    v = torch.randn(B, Hkv, N, d, generator=g).to(torch.bfloat16).to(dev)
    var = obc.VARIANT_CODES[args.variant]
    ws = torch.empty(obc.obc_score_workspace_bytes(B, N, 1, Hq, Hkv, d, obc.OBC_BF16, var), dtype=torch.uint8, device=dev)
    run = torch.zeros(B, Hkv, N, dtype=torch.float32, device=dev)
    keep = torch.empty(B, Hkv, N - 1, dtype=torch.int32, device=dev)
    k_out = torch.empty(B, Hkv, N - 1, d, dtype=torch.bfloat16, device=dev)
    v_out = torch.empty_like(k_out)
    s_out = torch.empty(B, Hkv, N, dtype=torch.float32, device=dev)
    sinks, recent = 4, 256
    hh = N - 1 - sinks - recent

    def score(i):
        obc.obc_score(q, k, v, var, scores=run, workspace=ws, accumulate=True)

    def step_gather(i):
        score(i)
        obc.obc_select_protected(run, hh, sinks, recent, 0, keep_idx=keep)
        obc.obc_compact(k, v, keep, k_out=k_out, v_out=v_out)
        obc.obc_compact_scores(run, keep, n_out=N, scores_out=s_out)

    def step_inplace(i):
        score(i)
        obc.obc_select_protected(run, hh, sinks, recent, 0, keep_idx=keep)
        obc.obc_compact_inplace(k, v, keep, scores=run)

    ws_step = torch.empty(obc.obc_decode_step_workspace_bytes(B, N, Hq, Hkv, d, obc.OBC_BF16, var), dtype=torch.uint8, device=dev)
    evicted = torch.empty(B, Hkv, dtype=torch.int32, device=dev)

    def step_one_call(i):
        obc.obc_decode_step(q, k, v, run, var, sinks, recent, evicted=evicted, workspace=ws_step)

    for i in range(args.warmup):
        step_gather(i)
        step_inplace(i)
        step_one_call(i)
    torch.cuda.synchronize()
    it = max(args.steps, 50)
    out = {"metric": "decode step latency per layer (W=1 accumulate + evict one + compact)", "unit": "us", "n_gpus": 1,
           "steps": it, "warmup": args.warmup, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "decode_llama8b_layer", "B": B, "Hq": Hq, "Hkv": Hkv, "d": d, "cache": N,
                      "sinks": sinks, "recent": recent, "variant": args.variant},
           "score_accumulate_us": round(timed(score, it, torch) * 1e3, 2),
           "step_gather_us": round(timed(step_gather, it, torch) * 1e3, 2),
           "step_inplace_us": round(timed(step_inplace, it, torch) * 1e3, 2),
           "step_one_call_us": round(timed(step_one_call, it, torch) * 1e3, 2)}
    out["value"] = out["step_one_call_us"]
    print(json.dumps(out))


def timed(fn, iters, torch):
    """Average milliseconds per call of fn(i), events on the current (launch) stream."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        fn(i)
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


def parity_diagnostics(torch, np, oracle, ref, keep_ref, vi, nb, sub_lens, wl, N, Hkv, nvar, scores, keep, score, select):
    """GPU scores of input set 0 against the oracle's on the sampled sequences, and the GPU's kept indices against the
    oracle's selection on the oracle's own scores (outside every timed region)."""
    if keep_ref is None:
        keep_ref = oracle.select(ref.astype("float32"), wl.budget, sub_lens)
    score(0)
    select(0)
    torch.cuda.synchronize()
    g_scores = (scores[vi] if nvar == 3 else scores)[:nb].cpu().numpy()
    g_keep = keep[:nb].cpu().numpy()
    tol = 1e-3 if wl.dtype == "bf16" else 1e-5
    rel, in_band, out_band = [], 0, 0
    for b in range(nb):
        L = sub_lens[b] if sub_lens else N
        for h in range(Hkv):
            r, g = ref[b, h, :L], g_scores[b, h, :L]
            nz = r != 0
            rel.append(np.abs(g - r)[nz] / np.abs(r[nz]))
            tau = np.partition(r, L - wl.budget)[L - wl.budget]
            differ = np.setxor1d(g_keep[b, h], keep_ref[b, h])
            band = np.abs(r[differ] - tau) <= 2 * tol * tau
            in_band += int(band.sum())
            out_band += int((~band).sum())
    rel = np.concatenate(rel)
    return {"max_rel_err": float(rel.max()), "p999_rel_err": float(np.quantile(rel, 0.999)),
            "idx_mismatch_in_band": in_band, "idx_mismatch_out_of_band": out_band,
            "note": "GPU vs the fp64 oracle on the cpu_baseline sample, no floor; band = +-2 tol around each head's "
                    "budget-th largest oracle score (tokens inside it may legitimately swap)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2510_07651_amd import binding as obc
    from paper_2510_07651_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(3)
    obc.load_library()
    if args.decode:
        decode_step_bench(args, torch, obc)
        return
    dev = torch.device("cuda:0")
    wl = synth.config(args.workload)
    B, Hq, Hkv, d, N, W = wl.B, wl.Hq, wl.Hkv, wl.d, wl.N, wl.W
    lens = synth.seq_lens_of(wl)
    tokens = sum(lens) if lens else B * N

    # Two independent input sets, alternated, so that no cache can hold a step's K/V from the step before.
    sets = []
    for layer in range(2):
        x = synth.make_inputs(wl, layer=layer)
        sets.append({k: (v.to(dev) if torch.is_tensor(v) else v) for k, v in x.items()})
    var = obc.VARIANT_CODES[args.variant]
    dt = obc.OBC_BF16 if wl.dtype == "bf16" else obc.OBC_F32
    ws = torch.empty(obc.obc_score_workspace_bytes(B, N, W, Hq, Hkv, d, dt, var), dtype=torch.uint8, device=dev)
    nvar = 3 if var == obc.OBC_ALL else 1
    scores = torch.empty((nvar, B, Hkv, N) if nvar == 3 else (B, Hkv, N), dtype=torch.float32, device=dev)
    sel_scores = scores[2] if nvar == 3 else scores
    keep = torch.empty((B, Hkv, wl.budget), dtype=torch.int32, device=dev)
    k_out = torch.empty((B, Hkv, wl.budget, d), dtype=sets[0]["k"].dtype, device=dev)
    v_out = torch.empty_like(k_out)

    def score(i, mask=None):
        s = sets[i & 1]
        obc.obc_score(s["q"], s["k"], s["v"], var, seq_lens=lens, scores=scores, workspace=ws, stage_mask=mask)

    def select(i):
        obc.obc_select(sel_scores, wl.budget, seq_lens=lens, keep_idx=keep)

    def compact(i):
        s = sets[i & 1]
        obc.obc_compact(s["k"], s["v"], keep, k_out=k_out, v_out=v_out)

    def step(i):
        score(i)
        select(i)
        compact(i)

    # The fp64 oracle on the CPU first (seconds of host work during which the GPU idles), so that nothing sits between
    # the GPU-side measurements below and the timed region.
    cpu, oracle_out = None, None
    if not args.no_cpu_baseline:
        import oracle
        import numpy as np
        x = synth.make_inputs(wl, layer=0)
        nb = B if args.cpu_seqs <= 0 else min(args.cpu_seqs, B)
        sub_lens = lens[:nb] if lens else None
        c0 = time.perf_counter()
        s_ref = oracle.score(x["q"][:nb], x["k"][:nb], x["v"][:nb], seq_lens=sub_lens)
        keep_ref = oracle.select(s_ref[2].astype("float32"), wl.budget, sub_lens)
        kb, vb = (x[t][:nb].view(torch.int16).numpy() for t in ("k", "v")) if wl.dtype == "bf16" else \
                 (x[t][:nb].numpy() for t in ("k", "v"))
        oracle.compact(kb, vb, keep_ref)
        c1 = time.perf_counter()
        cpu_tokens = sum(sub_lens) if sub_lens else nb * N
        cpu = {
            "value": round(cpu_tokens / (c1 - c0), 1), "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "%d of %d sequences, all %d KV heads (%d head-tokens): fp64 score (3 variants) + select + "
                      "compact, %.1f s wall on %d threads" % (nb, B, Hkv, cpu_tokens * Hkv, c1 - c0,
                                                             oracle.num_threads()),
        }
        oracle_out = (s_ref, keep_ref, nb, sub_lens)
        del x, kb, vb

    it = min(max(args.steps, 10), 100)
    side = {}

    def side_measurements():
        """Per-stage durations, the box's streaming-read rate, the sink-dominated inputs and the two-stream variant:
        diagnostics beside the headline number, each on its own loop of launches."""
        def stage_loops():
            # Per-stage device durations (events on the launch stream), same alternating inputs; a hundred untimed steps
            # first, so that the stage loops are not the ones that see the clocks ramp up after idle.
            for i in range(100):
                step(i)
            side["stages"] = {
                "sweep1": timed(lambda i: score(i, obc.OBC_STAGE_SWEEP1), it, torch),
                "combine": timed(lambda i: score(i, obc.OBC_STAGE_COMBINE), it, torch),
                "sweep2": timed(lambda i: score(i, obc.OBC_STAGE_SWEEP2), it, torch),
                "obc_select": timed(select, it, torch),
                "obc_compact": timed(compact, it, torch),
            }

        # The box's own streaming-read rate over the same K and V buffers (plain 128-bit loads).
        sink = torch.empty(obc.OBC_PROBE_BLOCKS * 256, dtype=torch.int32, device=dev)

        def stream(i):
            s = sets[i & 1]
            obc.obc_probe_read_bandwidth(s["k"], sink)
            obc.obc_probe_read_bandwidth(s["v"], sink)

        stream(0)
        side["ms_stream"] = timed(stream, it, torch)
        side["ms_sink"], side["ms_pipelined"] = None, None
        if args.plain:
            stage_loops()
            return
        # The same call on inputs where ONE key (an attention sink) holds nearly all of every window row's attention:
        # its cost must not depend on that (side measurement; the metric is on the workload's own inputs).
        import dataclasses
        sink_wl = dataclasses.replace(wl, shared_query=1.0, sink_gain=3.0, sinks=1)
        sx = synth.make_inputs(sink_wl, layer=0)
        sset = {k: (v.to(dev) if torch.is_tensor(v) else v) for k, v in sx.items()}

        def score_sink(i):
            obc.obc_score(sset["q"], sset["k"], sset["v"], var, seq_lens=lens, scores=scores, workspace=ws)

        score_sink(0)
        side["ms_sink"] = timed(score_sink, it, torch)
        del sset, sx
        # The same K steps with consecutive steps (independent inputs, outputs and workspaces) on two streams, so that
        # the narrow select and gather kernels of one step overlap the next step's sweeps.
        pipe = []
        for i in range(2):
            pipe.append({"stream": torch.cuda.Stream(), "ws": torch.empty_like(ws), "scores": torch.empty_like(scores),
                         "keep": torch.empty_like(keep), "k_out": torch.empty_like(k_out), "v_out": torch.empty_like(v_out)})

        def step_on(i):
            s, p = sets[i & 1], pipe[i & 1]
            with torch.cuda.stream(p["stream"]):
                obc.obc_score(s["q"], s["k"], s["v"], var, seq_lens=lens, scores=p["scores"], workspace=p["ws"])
                obc.obc_select(p["scores"][2] if nvar == 3 else p["scores"], wl.budget, seq_lens=lens, keep_idx=p["keep"])
                obc.obc_compact(s["k"], s["v"], p["keep"], k_out=p["k_out"], v_out=p["v_out"])

        for i in range(min(args.warmup, 50)):
            step_on(i)
        torch.cuda.synchronize()
        p0 = time.perf_counter()
        for i in range(args.steps):
            step_on(i)
        torch.cuda.synchronize()
        side["ms_pipelined"] = (time.perf_counter() - p0) * 1e3 / args.steps
        stage_loops()

    step(0)
    torch.cuda.synchronize()
    # The side measurements run BEFORE the timed region by default: they are a few hundred launches, after which the
    # chip's clock management has settled, so the timed region measures sustained throughput also when it is short
    # (--timed-first restores the other order: then a short run right after idle reads some 20 % slower).
    if not args.timed_first:
        side_measurements()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    scored = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        score(i)
        scored[i].record()
        select(i)
        compact(i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = tokens / (ms_per_step * 1e-3)
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))   # device time of each step
    # obc_score's launch-to-completion time inside the timed region itself (events on the launch stream)
    ms_score_timed = sum(marks[i].elapsed_time(scored[i]) for i in range(args.steps)) / args.steps

    if args.timed_first:
        side_measurements()
    ms = {"obc_score": ms_score_timed}
    ms.update(side["stages"])
    ms_stream, ms_sink, ms_pipelined = side["ms_stream"], side["ms_sink"], side["ms_pipelined"]
    esize = 2 if wl.dtype == "bf16" else 4
    head_tokens = tokens * Hkv
    algo_bytes = head_tokens * 2 * d * esize + B * Hq * W * d * esize + nvar * B * Hkv * N * 4
    achieved = algo_bytes / (ms["obc_score"] * 1e-3) / 1e9
    mfma_flops = 4 * 2 * Hq * W * d * tokens
    traffic, traffic_source = None, None
    # HBM bytes of one obc_score call as rocprofv3's counters measured them in a separate profiling run: read from the
    # committed counter summary of this workload (not measured by this run; the file says how it was made)
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % wl.name)
    if os.path.exists(tpath):
        import re
        with open(tpath) as f:
            m = re.search(r"obc_score \(all mfma_\* kernels\):.*?=\s*(\d+) bytes per call", f.read())
        traffic = int(m.group(1)) if m else None
        traffic_source = "profiles/" + os.path.basename(tpath) if m else None
    # Vector-ALU load of the two sweeps beside the memory roofline: the two kernels issue ~22.5 vector instructions per
    # lane and (window row, token) pair, matrix ops included as one each (hardware counter SQ_INSTS_VALU of the two
    # sweeps over the pair count, profiles/sq_counters_c3_*.txt); the chip's published fp32 vector peak, 157.3 TFLOP/s,
    # is 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz fused multiply-adds, i.e. 7.86e13 lane-operations per second.
    pairs = Hq * W * tokens
    lane_ops_per_pair = 22.5
    valu_rate = 256 * 4 * 32 * 2.4e9
    valu_ms = pairs * lane_ops_per_pair / valu_rate * 1e3
    roofline = {
        "bound": "hbm", "kernel": "obc_score = mfma_sweep1 + mfma_combine + mfma_sweep2",
        "achieved": round(achieved, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
        "frac": round(achieved / PEAK_HBM_GBPS, 4), "traffic": traffic, "traffic_source": traffic_source,
        "algorithmic_bytes": algo_bytes,
        "valu": {"pairs": pairs, "lane_ops_per_pair": lane_ops_per_pair, "peak_lane_ops_per_s": valu_rate,
                 "ms_at_peak": round(valu_ms, 4), "frac": round(valu_ms / ms["obc_score"], 4)},
        "kernel_ms": {k: round(v, 4) for k, v in ms.items()},
        # plain streaming read of the same K and V buffers on this machine: the practical ceiling
        "stream_read_GBps": round(2 * sets[0]["k"].numel() * esize / (ms_stream * 1e-3) / 1e9, 1),
        # the four dense contractions of the path (Q K^T twice, P V, O V^T) against the dense bf16 matrix-core peak
        "mfma": {"flops": mfma_flops, "achieved_TFLOPs": round(mfma_flops / (ms["obc_score"] * 1e-3) / 1e12, 1),
                 "peak_TFLOPs": 2500.0, "frac": round(mfma_flops / (ms["obc_score"] * 1e-3) / 2.5e15, 4)},
    }

    parity = None
    if oracle_out is not None:
        # Parity diagnostics on the oracle's sample, outside every timed region.
        import numpy as np
        import oracle
        s_ref, keep_ref, nb, sub_lens = oracle_out
        vi = {"value": 0, "key": 1, "joint": 2, "all": 2}.get(args.variant)
        if vi is not None:
            parity = parity_diagnostics(torch, np, oracle, s_ref[vi], keep_ref if vi == 2 else None, vi, nb, sub_lens, wl,
                                        N, Hkv, nvar, scores, keep, score, select)

    out = {
        "metric": "scored KV tokens/sec (all heads) at N=32K; achieved HBM GB/s vs peak",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "B": B, "Hq": Hq, "Hkv": Hkv, "d": d, "N": N, "W": W, "budget": wl.budget,
                   "variant": args.variant, "path": "score+select+compact"},
        "step_ms": {"median": round(per_step[len(per_step) // 2], 4), "min": round(per_step[0], 4),
                    "max": round(per_step[-1], 4)},
        "head_tokens_per_s": round(head_tokens / (ms_per_step * 1e-3), 1),
        "score_only_tokens_per_s": round(tokens / (ms["obc_score"] * 1e-3), 1),
        "obc_score_ms_one_sink_dominates_every_row": None if ms_sink is None else round(ms_sink, 4),
        "two_streams": None if ms_pipelined is None else {
            "ms_per_step": round(ms_pipelined, 4), "tokens_per_s": round(tokens / (ms_pipelined * 1e-3), 1),
            "note": "consecutive steps alternate between two streams; not the headline value"},
        "roofline": roofline, "cpu_baseline": cpu, "parity": parity,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
