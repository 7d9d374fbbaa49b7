#!/usr/bin/env python3
"""Benchmark of the ESA hot path on one MI355X.

A "step" is one pass of the whole hot path for one chunk of current tokens: compress the
chunk's queries and keys, score every middle token, pick the top-k, gather their keys/values
and attend over [I, M_k, L, C].  The default workload is the metric's: the Llama-3-8B-shaped
layer at 128k context (configuration 3), steady-state last chunk (t0 = 130560, 128384 middle
tokens).  Inputs (Q, K, V, the compressed-key cache of the preceding tokens, weights) are
resident in HBM before the timed region.

Prints ONE JSON line: the contract fields plus `roofline` (dominant call, from HIP events
recorded live on the launch stream) and `cpu_baseline` (the float64 oracle timed on the host
cores on the same step).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

VARIANT_CALLS = ("attend_indexed", "attend_local", "attend_finish", "attend_reencoded")   # timed beside the step
# HBM bytes per launch from the rocprofv3 counter passes summarised under profiles/ (FETCH_SIZE and
# WRITE_SIZE per dispatch, each scaled by what the same counter reads for a plain 256 MiB device copy:
# x2.0 for FETCH_SIZE, x1.0 for WRITE_SIZE), summed over the kernels of the call.  Counters cannot be
# read from inside this script, so the figure is attached only to the workload it was measured on.
MEASURED_TRAFFIC_BYTES = {
    ("C3", 131072, "attend"): 1024.0 * (2.0 * (11645.5 + 8493.5) + (16896.0 + 4096.0)),
    ("C3", 131072, "score"): 1024.0 * (2.0 * (16668.0 + 16718.5 + 279.5) + (3986.0 + 501.5 + 4.0)),
    ("C3", 131072, "select"): 1024.0 * (2.0 * (3.8 + 269.8 + 310.8 + 317.2 + 329.2)
                                        + (24.0 + 7.9 + 121.5 + 8.2 + 11.5)),
    ("C3", 131072, "gather"): 1024.0 * (2.0 * 4137.1 + 8192.0),
}


def algorithmic_work(cfg, t0, n_mid, k_eff, l_c):
    """Per-step algorithmic FLOPs / bytes of each call (Appendix A of the paper; causal part at half)."""
    d_Hq, d_K, d_c, esz = cfg.H * cfg.d, cfg.H_kv * cfg.d, cfg.d_c, 2 if cfg.dtype == "bf16" else 4
    i_end = min(cfg.l_I, t0)
    n_local = t0 - max(t0 - cfg.l_L, i_end)
    keys_eff = i_end + k_eff + n_local + (l_c + 1) / 2.0
    return {
        "compress": {"flops": 2.0 * l_c * (d_Hq + d_K) * d_c,
                     "bytes": (l_c * (d_Hq + d_K) + (d_Hq + d_K) * d_c + 2 * l_c * d_c) * esz},
        "score": {"flops": 2.0 * l_c * n_mid * d_c, "bytes": n_mid * d_c * esz + 4 * n_mid},
        "select": {"flops": 0.0, "bytes": 4.0 * n_mid + 4.0 * k_eff},
        "gather": {"flops": 0.0, "bytes": 4.0 * k_eff * d_K * esz},
        "attend": {"flops": 4.0 * d_Hq * l_c * keys_eff,
                   "bytes": (2 * l_c * d_Hq + 2 * (i_end + k_eff + n_local + l_c) * d_K) * esz},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C3", help="C2, C3 or C5 (prefill), C4 (decode)")
    ap.add_argument("--seq", type=int, default=0, help="override the sequence length (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true",
                    help="time eager launches instead of replaying the step as a captured HIP graph")
    ap.add_argument("--two-branches", action="store_true",
                    help="variant: the selection-independent part (key compression, attention over I, L, C) runs on a "
                         "second stream beside select and gather and esa_attend_finish adds the selected keys; measured "
                         "equal to the one-stream step at configuration 3, slower at configuration 5")
    ap.add_argument("--fused-gather", action="store_true",
                    help="variant: esa_attend_indexed follows the indices itself instead of esa_gather_kv + esa_attend "
                         "(four calls; not the default step)")
    ap.add_argument("--fork-after", choices=("start", "score"), default="score",
                    help="where the second stream starts (the score sweeps want every CU for themselves)")
    ap.add_argument("--batch", type=int, default=1,
                    help="independent sequences per step (the decode configuration is also quoted at 16)")
    ap.add_argument("--prompt", action="store_true",
                    help="secondary metric: prefill the whole prompt chunk by chunk (S / total time) instead of "
                         "timing the last chunk")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain device copy of the key cache (calibrates HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    import paper_2502_14477_amd as esa
    from esa_inputs import get_config, make_layer, segment_bounds, chunk_starts

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = get_config(args.config)
    if args.seq:
        cfg = cfg.scaled(S=args.seq)
    if args.prompt:
        return whole_prompt(args, cfg, esa, torch, np)
    # One stream unless asked otherwise; always one stream under the profiler (one dispatch after the
    # other) and for decode-sized chunks, where nothing of the attention can start early.
    args.single_stream = not args.two_branches or args.eager or cfg.l_C < 16
    t0 = chunk_starts(cfg)[-1]
    l_c = min(cfg.l_C, cfg.S - t0)
    i_end, l_start = segment_bounds(t0, cfg.l_I, cfg.l_L)
    n_mid = l_start - i_end
    k_eff = min(cfg.k, n_mid)

    t_gen = time.time()
    B = args.batch
    layers = [make_layer(cfg, batch=b, q_rows=(t0, t0 + l_c)) for b in range(B)]
    for layer in layers:
        layer.q_row0 = t0
    layer = layers[0]

    def dev(name):
        a = np.stack([getattr(x, name) for x in layers]) if B > 1 else getattr(layer, name)
        if cfg.dtype == "f32":
            return torch.from_numpy(a).cuda()
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)

    def rows(t, r0, r1):
        return t[:, r0:r1] if B > 1 else t[r0:r1]

    Q, K, V = dev("Q"), dev("K"), dev("V")
    # weights are packed once per layer, at load time (batch elements share the layer's weights)
    W_q = esa.esa_pack_weights(torch.from_numpy(layer.W_q.view(np.int16)).cuda().view(torch.bfloat16)
                               if cfg.dtype == "bf16" else torch.from_numpy(layer.W_q).cuda())
    W_k = esa.esa_pack_weights(torch.from_numpy(layer.W_k.view(np.int16)).cuda().view(torch.bfloat16)
                               if cfg.dtype == "bf16" else torch.from_numpy(layer.W_k).cuda())
    # state left by the preceding steps: compressed keys of every earlier token
    kc = torch.zeros(((B,) if B > 1 else ()) + (cfg.S, cfg.d_c), dtype=K.dtype, device="cuda")
    for r0 in range(0, t0, 16384):
        r1 = min(r0 + 16384, t0)
        esa.esa_compress(rows(K, r0, r1), W_k, out=rows(kc, r0, r1))
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    calls = ("compress", "score", "select", "gather", "attend")

    side = torch.cuda.Stream()

    def step():
        # The five calls on one stream.  With --two-branches (Algorithm 1's split of the key set) the key
        # compression (needed by later steps only) and the attention over [I, L, C], which do not depend
        # on the selection, go to a second stream once the score sweeps (which want every CU) are done,
        # and run beside select -> gather; the selected keys and the merge follow on the main stream.
        main = torch.cuda.current_stream()

        def fork():
            side.wait_stream(main)
            with torch.cuda.stream(side):
                esa.esa_compress(rows(K, t0, t0 + l_c), W_k, out=rows(kc, t0, t0 + l_c))
                esa.esa_attend_local(Q, K, V, t0, cfg.l_I, cfg.l_L)

        if args.single_stream:       # queries and keys of the chunk compressed by one call (Eq. 5 has both)
            qc, _ = esa.esa_compress_qk(Q, W_q, rows(K, t0, t0 + l_c), W_k, out_k=rows(kc, t0, t0 + l_c))
        else:
            if args.fork_after == "start":
                fork()
            qc = esa.esa_compress(Q, W_q)
        if n_mid > cfg.k:
            score = esa.esa_score(qc, kc, i_end, l_start)
        else:
            score = torch.zeros(((B,) if B > 1 else ()) + (n_mid,), dtype=torch.float32, device="cuda")
        if not args.single_stream and args.fork_after == "score":
            fork()
        idx = esa.esa_select_topk(score, cfg.k, base=i_end)
        if args.fused_gather:
            if not args.single_stream:
                main.wait_stream(side)
            return esa.esa_attend_indexed(Q, K, V, t0, cfg.l_I, cfg.l_L, idx)
        ks, vs = esa.esa_gather_kv(K, V, idx)
        if not args.single_stream:
            main.wait_stream(side)
            return esa.esa_attend_finish(Q, K, V, t0, cfg.l_I, cfg.l_L, ks, vs)
        return esa.esa_attend(Q, K, V, t0, cfg.l_I, cfg.l_L, ks, vs)

    def timed(fn, n):
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t_start) / n

    def time_step():
        for _ in range(max(args.warmup, 1)):
            step()
        eager = timed(step, args.steps)
        if args.eager:
            return eager, eager, "eager launches"
        # The step is launch-bound on the host (about twenty small kernels), so it is captured once
        # as a HIP graph and replayed; every kernel of the step runs in every replay.
        warm = torch.cuda.Stream()
        warm.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(warm):
            step()
        torch.cuda.current_stream().wait_stream(warm)
        # One graph holds `per_graph` consecutive steps (as a prefill issues its chunks one after the other),
        # so that the start-up gap of a graph launch is not paid by every step.
        per_graph = 5 if args.steps % 5 == 0 else 1
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(per_graph):
                graph_out = step()
        for _ in range(max(args.warmup // per_graph, 1)):
            graph.replay()
        replay = timed(graph.replay, args.steps // per_graph) / per_graph
        ref = step()
        torch.cuda.synchronize()
        assert torch.equal(ref, graph_out), "graph replay and eager step disagree"
        return eager, replay, "HIP graph replay (%d steps per graph)" % per_graph

    try:
        eager_ms, ms_per_step, mode = time_step()
    except Exception as exc:                # a second graph branch is an optimisation, not a requirement
        if args.single_stream:
            raise
        print("bench.py: two-branch step failed (%s); timing the one-stream step" % exc, file=sys.stderr)
        torch.cuda.synchronize()
        args.single_stream = True
        eager_ms, ms_per_step, mode = time_step()

    # Per-call durations from HIP events on the launch stream (torch's current stream).  Each call is
    # issued `reps` times back to back between two events, as one captured graph (as separate launches
    # under --eager), so that the figure is the kernels' own duration and not the host's launch gaps.
    qc_s = esa.esa_compress(Q, W_q)
    score_s = esa.esa_score(qc_s, kc, i_end, l_start) if n_mid > cfg.k else \
        torch.zeros(((B,) if B > 1 else ()) + (n_mid,), dtype=torch.float32, device="cuda")
    idx_s = esa.esa_select_topk(score_s, cfg.k, base=i_end)
    ks_s, vs_s = esa.esa_gather_kv(K, V, idx_s)

    def call_compress():
        esa.esa_compress_qk(Q, W_q, rows(K, t0, t0 + l_c), W_k, out_q=qc_s, out_k=rows(kc, t0, t0 + l_c))

    single = {
        "compress": call_compress,
        "score": (lambda: esa.esa_score(qc_s, kc, i_end, l_start)) if n_mid > cfg.k else (lambda: None),
        "select": lambda: esa.esa_select_topk(score_s, cfg.k, base=i_end),
        "gather": lambda: esa.esa_gather_kv(K, V, idx_s),
        "attend": lambda: esa.esa_attend(Q, K, V, t0, cfg.l_I, cfg.l_L, ks_s, vs_s),
        "attend_indexed": lambda: esa.esa_attend_indexed(Q, K, V, t0, cfg.l_I, cfg.l_L, idx_s),
        "attend_local": lambda: esa.esa_attend_local(Q, K, V, t0, cfg.l_I, cfg.l_L),
        "attend_finish": lambda: esa.esa_attend_finish(Q, K, V, t0, cfg.l_I, cfg.l_L, ks_s, vs_s),
        # Section 3.2 inside the library (the inputs stand in for un-encoded ones: same work)
        "attend_reencoded": lambda: esa.esa_attend_reencoded(Q, K, V, t0, cfg.l_I, cfg.l_L, ks_s, vs_s, 4096.0, 5e5),
    }
    if args.eager:      # under the profiler: only the step's own launches, so that per-kernel averages are the step's
        for c in VARIANT_CALLS:
            del single[c]
    reps, rounds = 10, max(3, min(args.steps, 10))
    call_ms = {}
    for c in single:
        def burst(fn=single[c]):
            for _ in range(reps):
                fn()
        burst()
        torch.cuda.synchronize()
        run = burst
        if not args.eager:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                burst()
            run = g.replay
        run()
        samples = []
        for _ in range(rounds):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            run()
            e1.record()
            torch.cuda.synchronize()
            samples.append(e0.elapsed_time(e1) / reps)
        call_ms[c] = float(np.mean(samples))
        del run

    if args.copy_probe:
        # a plain copy of known size (2 x K bytes moved), the yardstick for the HBM traffic counters
        torch.empty_like(K).copy_(K)
        torch.cuda.synchronize()

    work = algorithmic_work(cfg, t0, n_mid, k_eff, l_c)
    for w in work.values():   # batch elements are independent sequences
        w["flops"] *= B
        w["bytes"] *= B
    per_call_report = {}
    for c in calls:
        us = 1e3 * call_ms[c]
        rep = {"us": round(us, 2)}
        if work[c]["flops"]:
            rep["tflops"] = round(work[c]["flops"] / (us * 1e-6) / 1e12, 2)
        rep["gbs"] = round(work[c]["bytes"] / (us * 1e-6) / 1e9, 1)
        per_call_report[c] = rep
    for c in VARIANT_CALLS:   # variants: fused gather, the two-call form, Section 3.2's re-encoding
        if c in call_ms:
            per_call_report[c] = {"us": round(1e3 * call_ms[c], 2)}
    dominant = max(calls, key=lambda c: call_ms[c])
    if work[dominant]["flops"]:
        achieved = work[dominant]["flops"] / (call_ms[dominant] * 1e-3) / 1e12
        roofline = {"kernel": "esa_" + dominant, "bound": "mfma", "achieved": round(achieved, 2),
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "traffic": None}
    else:
        achieved = work[dominant]["bytes"] / (call_ms[dominant] * 1e-3) / 1e9
        roofline = {"kernel": "esa_" + dominant, "bound": "hbm", "achieved": round(achieved, 1),
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4),
                    "traffic": None}
    traffic = MEASURED_TRAFFIC_BYTES.get((cfg.name, cfg.S, dominant)) if B == 1 else None
    roofline["traffic"] = None if traffic is None else round(traffic)
    roofline["algorithmic"] = round(work[dominant]["flops"] or work[dominant]["bytes"])
    roofline["per_call"] = per_call_report
    step_flops = sum(w["flops"] for w in work.values())
    roofline["step_tflops"] = round(step_flops / (ms_per_step * 1e-3) / 1e12, 2)

    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = cpu_oracle_baseline(layer, cfg, t0, l_c)

    unit = "tokens/s"
    value = B * l_c / (ms_per_step * 1e-3)
    result = {
        "metric": "ESA prefill tokens/s per layer at 128k ctx" if not cfg.decode else "ESA decode step",
        "value": round(value, 1), "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "%s: H=%d H_kv=%d d=%d, S=%d, chunk l_C=%d at t0=%d, l_I=%d l_L=%d k=%d d_c=%d, "
                               "%d middle tokens; one step = compress+score+select+gather+attend for one chunk"
                               % (cfg.name, cfg.H, cfg.H_kv, cfg.d, cfg.S, l_c, t0, cfg.l_I, cfg.l_L, cfg.k,
                                  cfg.d_c, n_mid),
                   "global_batch": B, "seq_len": cfg.S, "parallelism": "single GPU"},
        "roofline": roofline, "cpu_baseline": cpu_baseline,
        "launch_mode": mode + (", one stream" if args.single_stream else ", two branches")
        + (", gather fused into attend" if args.fused_gather else ""), "eager_ms_per_step": round(eager_ms, 4), "setup_s": round(t_gen, 1),
    }
    print(json.dumps(result))


def whole_prompt(args, cfg, esa, torch, np):
    """Secondary metric: every chunk of the prompt in order (the compressed-key cache grows as it
    would in a model), timed as eager launches and as one captured graph of the whole prefill."""
    from esa_inputs import make_layer, segment_bounds, chunk_starts
    layer = make_layer(cfg)

    def dev(a):
        if cfg.dtype == "f32":
            return torch.from_numpy(a).cuda()
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)

    Q, K, V = dev(layer.Q), dev(layer.K), dev(layer.V)
    W_q, W_k = esa.esa_pack_weights(dev(layer.W_q)), esa.esa_pack_weights(dev(layer.W_k))
    kc = torch.zeros((cfg.S, cfg.d_c), dtype=K.dtype, device="cuda")
    starts = chunk_starts(cfg)

    def prefill():
        out = None
        for t0 in starts:
            t1 = min(t0 + cfg.l_C, cfg.S)
            i_end, l_start = segment_bounds(t0, cfg.l_I, cfg.l_L)
            n_mid = l_start - i_end
            if n_mid > cfg.k:
                qc, _ = esa.esa_compress_qk(Q[t0:t1], W_q, K[t0:t1], W_k, out_k=kc[t0:t1])
            else:
                esa.esa_compress(K[t0:t1], W_k, out=kc[t0:t1])
            ks = vs = None
            if n_mid > 0:
                if n_mid > cfg.k:
                    score = esa.esa_score(qc, kc, i_end, l_start)
                else:   # k covers the middle: every middle token is selected, no scores needed
                    score = torch.zeros(n_mid, dtype=torch.float32, device="cuda")
                idx = esa.esa_select_topk(score, cfg.k, base=i_end)
                ks, vs = esa.esa_gather_kv(K, V, idx)
            out = esa.esa_attend(Q[t0:t1], K, V, t0, cfg.l_I, cfg.l_L, ks, vs)
        return out

    def timed(fn, n):
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t_start) / n

    prefill()
    eager_s = timed(prefill, 2)
    warm = torch.cuda.Stream()
    warm.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(warm):
        prefill()
    torch.cuda.current_stream().wait_stream(warm)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        graph_out = prefill()
    graph.replay()
    graph_s = timed(graph.replay, 3)
    ref = prefill()
    torch.cuda.synchronize()
    assert torch.equal(ref, graph_out), "graph replay and eager prefill disagree"
    print(json.dumps({
        "metric": "ESA prefill tokens/s per layer, whole prompt", "value": round(cfg.S / graph_s, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": 3, "warmup": 1, "ms_per_step": round(1e3 * graph_s, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "%s: whole prompt of %d tokens, %d chunks of %d, one layer" % (cfg.name, cfg.S, len(starts), cfg.l_C),
                   "global_batch": 1, "seq_len": cfg.S, "parallelism": "single GPU"},
        "launch_mode": "one HIP graph for the whole prefill", "eager_tokens_per_s": round(cfg.S / eager_s, 1),
        "eager_ms": round(1e3 * eager_s, 3)}))


def cpu_oracle_baseline(layer, cfg, t0, l_c):
    """The float64 oracle, as it stands, on the same step; K' of the preceding tokens is state, not timed."""
    import numpy as np
    from oracle import esa_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    W_q, W_k = orc.widen(layer.W_q, cfg.dtype), orc.widen(layer.W_k, cfg.dtype)
    K = orc.widen(layer.K, cfg.dtype)
    V = orc.widen(layer.V, cfg.dtype)
    q = orc.widen(layer.Q, cfg.dtype)
    kc = np.zeros((cfg.S, cfg.d_c))
    for r0 in range(0, t0, 16384):
        kc[r0:min(r0 + 16384, t0)] = orc.compress(K[r0:min(r0 + 16384, t0)], W_k, None, cfg.dtype)
    times = []
    t_all = time.perf_counter()
    while True:
        ts = time.perf_counter()
        qc = orc.compress(q, W_q, None, cfg.dtype)
        kc[t0:t0 + l_c] = orc.compress(K[t0:t0 + l_c], W_k, None, cfg.dtype)
        orc.esa_step(q, K[:t0 + l_c], V[:t0 + l_c], kc, qc, t0, cfg.l_I, cfg.l_L, cfg.k, 1.0 / np.sqrt(cfg.d))
        times.append(time.perf_counter() - ts)
        if time.perf_counter() - t_all > 12.0 or len(times) >= 5:
            break
    best = min(times)
    return {"value": round(l_c / best, 1), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "the same step (one chunk of %d tokens at t0=%d), float64 numpy, best of %d runs, %.2f s each"
                      % (l_c, t0, len(times), best)}


if __name__ == "__main__":
    main()
