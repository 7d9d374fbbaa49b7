#!/usr/bin/env python3
"""Benchmark of the ESA hot path on one MI355X.

A "step" is one pass of the whole hot path for one chunk of current tokens: compress the
chunk's queries and keys, score every middle token, pick the top-k, gather their keys/values
and attend over [I, M_k, L, C].  The default workload is the metric's first half: the
Llama-3-8B-shaped layer at 128k context (configuration 3), steady-state last chunk
(t0 = 130560, 128384 middle tokens).  The metric's second half, the decode step on a
256k-token cache (configuration 4, batch 1 and 16), is timed in the same run and reported
under `decode`.  Inputs (Q, K, V, the compressed-key cache of the preceding tokens, weights)
are resident in HBM before the timed region.

Prints ONE JSON line: the contract fields plus `roofline` (dominant call, from HIP events
recorded live on the launch stream), `decode`, and `cpu_baseline` (the float64 oracle timed
on the host cores on the same step).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

CALLS = ("compress", "score", "select", "gather", "attend")
# timed beside the five calls: the fused form of score + select + gather that the default step uses, and variants
VARIANT_CALLS = ("score_select_gather", "attend_indexed", "attend_local", "attend_finish", "attend_reencoded")

# HBM bytes per launch from the rocprofv3 counter passes summarised under profiles/ (FETCH_SIZE and
# WRITE_SIZE per dispatch, each scaled by what the same counter reads for a plain 256 MiB device copy:
# x2.0 for FETCH_SIZE, x1.0 for WRITE_SIZE), summed over the kernels of the call.  Counters cannot be
# read from inside this script, so a figure is attached only to the workload it was measured on and only
# while the kernel sources are the ones it was measured on (TRAFFIC_TREE, see csrc_tree_hash).
TRAFFIC_TREE = "656a4f162149bc08"
MEASURED_TRAFFIC_BYTES = {
    ("C3", 131072, "score"): 73494752,
    ("C3", 131072, "attend"): 62817152,
    ("C3", 131072, "compress"): 16025600,
    ("C3", 131072, "gather"): 16861184,
    ("C3", 131072, "select"): 2792000,
    ("C5", 262144, "attend"): 125917184,
    ("C5", 262144, "score"): 156886304,
    ("C5", 262144, "gather"): 67393024,
    ("C5", 262144, "compress"): 21530624,
    ("C5", 262144, "select"): 4890272,
    ("C6", 131072, "score"): 72383168,
    ("C6", 131072, "attend"): 71358080,
    ("C6", 131072, "compress"): 16025600,
    ("C6", 131072, "gather"): 16861184,
    ("C6", 131072, "select"): 2761664,
    ("C4", 262144, "score"): 70009696,
    ("C4", 262144, "attend"): 19967744,
    ("C4", 262144, "gather"): 16861184,
    ("C4", 262144, "select"): 5261696,
    ("C4", 262144, "compress"): 1440768,
}


def csrc_tree_hash():
    """Fingerprint of the kernel sources: the stored traffic figures belong to exactly one such tree."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2502_14477_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


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


class Workload:
    """One configuration's last step, resident on the GPU: B independent sequences."""

    def __init__(self, esa, torch, np, cfg, B):
        from esa_inputs import make_layer, segment_bounds, chunk_starts
        self.cfg, self.B = cfg, B
        self.t0 = chunk_starts(cfg)[-1]
        self.l_c = min(cfg.l_C, cfg.S - self.t0)
        self.i_end, self.l_start = segment_bounds(self.t0, cfg.l_I, cfg.l_L)
        self.n_mid = self.l_start - self.i_end
        self.k_eff = min(cfg.k, self.n_mid)
        t_gen = time.time()
        t0, l_c = self.t0, self.l_c
        layers = [make_layer(cfg, batch=b, q_rows=(t0, t0 + l_c)) for b in range(B)]
        for layer in layers:
            layer.q_row0 = t0
        self.layer = layers[0]

        def dev(name):
            a = np.stack([getattr(x, name) for x in layers]) if B > 1 else getattr(self.layer, name)
            if cfg.dtype == "f32":
                return torch.from_numpy(a).cuda()
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)

        def weights(a):
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16) if cfg.dtype == "bf16" \
                else torch.from_numpy(a).cuda()

        self.Q, self.K, self.V = dev("Q"), dev("K"), dev("V")
        del layers
        # weights are packed once per layer, at load time (batch elements share the layer's weights)
        self.W_q = esa.esa_pack_weights(weights(self.layer.W_q))
        self.W_k = esa.esa_pack_weights(weights(self.layer.W_k))
        # state left by the preceding steps: compressed keys of every earlier token
        self.kc = torch.zeros(((B,) if B > 1 else ()) + (cfg.S, cfg.d_c), dtype=self.K.dtype, device="cuda")
        for r0 in range(0, t0, 16384):
            r1 = min(r0 + 16384, t0)
            esa.esa_compress(self.rows(self.K, r0, r1), self.W_k, out=self.rows(self.kc, r0, r1))
        torch.cuda.synchronize()
        self.setup_s = time.time() - t_gen

    def rows(self, t, r0, r1):
        return t[:, r0:r1] if self.B > 1 else t[r0:r1]

    def cold_copy(self):
        """The same step on its own copy of the caches (distinct memory: nothing of it is in any cache)."""
        import copy
        w = copy.copy(self)
        w.K, w.V, w.kc = self.K.clone(), self.V.clone(), self.kc.clone()
        return w


def step_reads_through_indices(args, l_c):
    """Gather as a call of its own (esa_gather_kv, then esa_attend on the gathered rows) or inside the attention
    kernel (esa_attend_indexed reads the selected cache rows through the index list: one kernel and one write +
    read of the selected rows fewer).  Measured on the step: 122.0 against 126.6 us at configuration 3, 452.8 / 464.0
    at 5, 136.8 / 141.3 at 6, 46.7 / 52.1 for a decode step, 314 / 370 at decode batch 16: the step takes the
    index-driven form unless told otherwise (--gather-call)."""
    if args.fused_gather:
        return True
    return not args.gather_call and not args.two_branches     # the two-branch form finishes on gathered rows


def make_step(esa, torch, w, args, side=None):
    """The five calls for one step of workload w, as a function to call (and to capture)."""
    cfg, t0, l_c, B = w.cfg, w.t0, w.l_c, w.B
    i_end, l_start, n_mid = w.i_end, w.l_start, w.n_mid
    Q, K, V, kc, W_q, W_k = w.Q, w.K, w.V, w.kc, w.W_q, w.W_k
    no_scores = torch.empty(((B,) if B > 1 else ()) + (n_mid,), dtype=torch.float32, device="cuda")
    single_stream = args.single_stream or l_c < 16
    indexed = step_reads_through_indices(args, l_c)

    def step():
        # The five calls on one stream.  With --two-branches (Algorithm 1's split of the key set) the key
        # compression (needed by later steps only) and the attention over [I, L, C], which do not depend
        # on the selection, go to a second stream once the score sweeps (which want every CU) are done,
        # and run beside select -> gather; the selected keys and the merge follow on the main stream.
        main = torch.cuda.current_stream()

        def fork():
            side.wait_stream(main)
            with torch.cuda.stream(side):
                esa.esa_compress(w.rows(K, t0, t0 + l_c), W_k, out=w.rows(kc, t0, t0 + l_c))
                esa.esa_attend_local(Q, K, V, t0, cfg.l_I, cfg.l_L)

        if single_stream:            # queries and keys of the chunk compressed by one call (Eq. 5 has both)
            qc, _ = esa.esa_compress_qk(Q, W_q, w.rows(K, t0, t0 + l_c), W_k, out_k=w.rows(kc, t0, t0 + l_c))
        else:
            if args.fork_after == "start":
                fork()
            qc = esa.esa_compress(Q, W_q)
        if single_stream and not args.separate_calls:
            if indexed:    # the attention kernel reads the selected rows through the index list
                _, idx, _, _ = esa.esa_score_select_gather(qc, kc, i_end, l_start, cfg.k)
                return esa.esa_attend_indexed(Q, K, V, t0, cfg.l_I, cfg.l_L, idx)
            # score, select and gather as one call (the same results with three kernels fewer)
            _, idx, ks, vs = esa.esa_score_select_gather(qc, kc, i_end, l_start, cfg.k, K, V)
            return esa.esa_attend(Q, K, V, t0, cfg.l_I, cfg.l_L, ks, vs)
        # k covers the middle segment in early chunks: every middle token is taken, no scores are read
        score = esa.esa_score(qc, kc, i_end, l_start) if n_mid > cfg.k else no_scores
        if not single_stream and args.fork_after == "score":
            fork()
        idx = esa.esa_select_topk(score, cfg.k, base=i_end)
        if indexed:
            if not single_stream:
                main.wait_stream(side)
            return esa.esa_attend_indexed(Q, K, V, t0, cfg.l_I, cfg.l_L, idx)
        ks, vs = esa.esa_gather_kv(K, V, idx)
        if not single_stream:
            main.wait_stream(side)
            return esa.esa_attend_finish(Q, K, V, t0, cfg.l_I, cfg.l_L, ks, vs)
        return esa.esa_attend(Q, K, V, t0, cfg.l_I, cfg.l_L, ks, vs)

    return step


def wall_ms(torch, fn, n):
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(n):
        fn()
    torch.cuda.synchronize()
    return 1e3 * (time.perf_counter() - t_start) / n


def time_steps(torch, steps_fns, n_steps, warmup, eager_only):
    """Time the step functions in `steps_fns` issued one after the other (one function: the same step
    again and again, its caches warm; several: a rotation over independent copies of the caches, so that
    every step finds its compressed keys and KV rows cold).  Returns (eager ms, replay ms, mode)."""
    n_fn = len(steps_fns)

    def round_of_steps():
        out = None
        for fn in steps_fns:
            out = fn()
        return out

    for _ in range(max(warmup // n_fn, 1)):
        round_of_steps()
    eager = wall_ms(torch, round_of_steps, max(n_steps // n_fn, 1)) / n_fn
    if eager_only:
        return eager, eager, "eager launches", None
    # The step is launch-bound on the host, so it is captured once as a HIP graph and replayed; every
    # kernel of the step runs in every replay.  One graph holds several consecutive steps (as a prefill
    # issues its chunks one after the other), so that the start-up gap of a graph launch is not paid by
    # every step.
    warm = torch.cuda.Stream()
    warm.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(warm):
        round_of_steps()
    torch.cuda.current_stream().wait_stream(warm)
    rounds_per_graph = 1 if n_fn > 1 else (5 if n_steps % 5 == 0 else 1)
    per_graph = rounds_per_graph * n_fn
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(rounds_per_graph):
            graph_out = round_of_steps()
    for _ in range(max(warmup // per_graph, 1)):
        graph.replay()
    replay = wall_ms(torch, graph.replay, max(n_steps // per_graph, 1)) / per_graph
    ref = steps_fns[-1]()
    torch.cuda.synchronize()
    assert torch.equal(ref, graph_out), "graph replay and eager step disagree"
    return eager, replay, "HIP graph replay (%d steps per graph)" % per_graph, graph


def per_call_times(esa, torch, np, w, args, with_variants):
    """Per-call durations from HIP events on the launch stream (torch's current stream).  Each call is
    issued `reps` times back to back between two events, as one captured graph (as separate launches
    under --eager), so that the figure is the kernels' own duration and not the host's launch gaps."""
    cfg, t0, l_c = w.cfg, w.t0, w.l_c
    Q, K, V, kc, W_q, W_k = w.Q, w.K, w.V, w.kc, w.W_q, w.W_k
    i_end, l_start, n_mid, B = w.i_end, w.l_start, w.n_mid, w.B
    qc_s = esa.esa_compress(Q, W_q)
    score_s = esa.esa_score(qc_s, kc, i_end, l_start) if n_mid > cfg.k else \
        torch.empty(((B,) if B > 1 else ()) + (n_mid,), dtype=torch.float32, device="cuda")
    idx_s = esa.esa_select_topk(score_s, cfg.k, base=i_end)
    ks_s, vs_s = esa.esa_gather_kv(K, V, idx_s)

    def call_compress():
        esa.esa_compress_qk(Q, W_q, w.rows(K, t0, t0 + l_c), W_k, out_q=qc_s, out_k=w.rows(kc, t0, t0 + l_c))

    single = {
        "compress": call_compress,
        "score": (lambda: esa.esa_score(qc_s, kc, i_end, l_start)) if n_mid > cfg.k else (lambda: None),
        "select": lambda: esa.esa_select_topk(score_s, cfg.k, base=i_end),
        "gather": lambda: esa.esa_gather_kv(K, V, idx_s),
        "attend": lambda: esa.esa_attend(Q, K, V, t0, cfg.l_I, cfg.l_L, ks_s, vs_s),
    }
    if step_reads_through_indices(args, l_c):      # as the step calls it: no gathered copy
        single["score_select_gather"] = lambda: esa.esa_score_select_gather(qc_s, kc, i_end, l_start, cfg.k)
    else:
        single["score_select_gather"] = lambda: esa.esa_score_select_gather(qc_s, kc, i_end, l_start, cfg.k, K, V)
    single["attend_indexed"] = lambda: esa.esa_attend_indexed(Q, K, V, t0, cfg.l_I, cfg.l_L, idx_s)
    if args.eager:      # under the profiler every attention launch is of the step's kind, so that per-kernel averages are the step's
        if step_reads_through_indices(args, l_c):
            single["attend"] = single["attend_indexed"]
        else:
            del single["attend_indexed"]
    if with_variants:
        single.update({
            "attend_local": lambda: esa.esa_attend_local(Q, K, V, t0, cfg.l_I, cfg.l_L),
            "attend_finish": lambda: esa.esa_attend_finish(Q, K, V, t0, cfg.l_I, cfg.l_L, ks_s, vs_s),
            # Section 3.2 inside the library (the inputs stand in for un-encoded ones: same work)
            "attend_reencoded": lambda: esa.esa_attend_reencoded(Q, K, V, t0, cfg.l_I, cfg.l_L, ks_s, vs_s, 4096.0, 5e5),
        })
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
    return call_ms


def call_report(w, call_ms):
    work = algorithmic_work(w.cfg, w.t0, w.n_mid, w.k_eff, w.l_c)
    for x in work.values():   # batch elements are independent sequences
        x["flops"] *= w.B
        x["bytes"] *= w.B
    rep = {}
    for c in CALLS:
        us = 1e3 * call_ms[c]
        r = {"us": round(us, 2)}
        if us > 0:
            if work[c]["flops"]:
                r["tflops"] = round(work[c]["flops"] / (us * 1e-6) / 1e12, 2)
            r["gbs"] = round(work[c]["bytes"] / (us * 1e-6) / 1e9, 1)
            r["hbm_frac"] = round(r["gbs"] / PEAK_HBM_GBS, 4)
        rep[c] = r
    for c in VARIANT_CALLS:   # variants: fused gather, the two-call form, Section 3.2's re-encoding
        if c in call_ms:
            rep[c] = {"us": round(1e3 * call_ms[c], 2)}
    return work, rep


def workload_text(w):
    cfg = w.cfg
    return ("%s: H=%d H_kv=%d d=%d, S=%d, chunk l_C=%d at t0=%d, l_I=%d l_L=%d k=%d d_c=%d, %d middle tokens; "
            "one step = compress, score, select, gather, attend for one chunk"
            % (cfg.name, cfg.H, cfg.H_kv, cfg.d, cfg.S, w.l_c, w.t0, cfg.l_I, cfg.l_L, cfg.k, cfg.d_c, w.n_mid))


def decode_record(esa, torch, np, args):
    """Configuration 4: one decode step (one new token per sequence) on 256k-token caches, batch 1 and 16."""
    from esa_inputs import get_config
    cfg = get_config("C4")
    out = {"workload": None, "unit": "us/step"}
    for B in (1, 16):
        w = Workload(esa, torch, np, cfg, B)
        out["workload"] = workload_text(w)
        step = make_step(esa, torch, w, args)
        n = max(args.steps, 10)
        eager, replay, mode, graph = time_steps(torch, [step], n, args.warmup, args.eager)
        call_ms = per_call_times(esa, torch, np, w, args, with_variants=False)
        indexed = step_reads_through_indices(args, w.l_c)
        work, rep = call_report(w, call_ms)
        step_bytes = sum(x["bytes"] for c, x in work.items() if not (indexed and c == "gather"))
        rec = {"us_per_step": round(1e3 * replay, 2), "eager_us_per_step": round(1e3 * eager, 2),
               "tokens_per_s": round(B / (replay * 1e-3), 1),
               "step_gbs": round(step_bytes / (replay * 1e-3) / 1e9, 1),
               "step_hbm_frac": round(step_bytes / (replay * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
               "algorithmic_bytes": round(step_bytes), "per_call": rep, "launch_mode": mode,
               "calls": "esa_compress_qk, esa_score_select_gather (no gather), esa_attend_indexed" if indexed else
                        "esa_compress_qk, esa_score_select_gather, esa_attend",
               "setup_s": round(w.setup_s, 1)}
        if B == 1:
            # one sequence's step touches about 100 MB, which the 256 MB memory-side cache keeps between
            # replays: rotate over independent copies of the caches so that every step reads from HBM
            del graph
            copies = [w] + [w.cold_copy() for _ in range(4)]       # 5 x (66 MB K' + 2 x 512 MB KV)
            fns = [make_step(esa, torch, c, args) for c in copies]
            _, cold, _, graph = time_steps(torch, fns, max(n, 20), args.warmup, args.eager)
            rec["cold_us_per_step"] = round(1e3 * cold, 2)
            rec["cold_note"] = "rotation over 5 independent copies of K', K and V (330 MB of K' alone per round)"
            del copies, fns
        out["batch_%d" % B] = rec
        del graph, w, step
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C3", help="C2, C3, C5, C6 (prefill) or C4 (decode)")
    ap.add_argument("--seq", type=int, default=0, help="override the sequence length (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode record (configuration 4, batch 1 and 16)")
    ap.add_argument("--cold", action="store_true",
                    help="also time the step on a rotation over independent copies of the caches (more than 256 MB of "
                         "compressed keys per round), so that nothing is served from the memory-side cache")
    ap.add_argument("--eager", action="store_true",
                    help="time eager launches instead of replaying the step as a captured HIP graph")
    ap.add_argument("--two-branches", action="store_true",
                    help="variant: the selection-independent part (key compression, attention over I, L, C) runs on a "
                         "second stream beside select and gather and esa_attend_finish adds the selected keys; measured "
                         "slower than the one-stream step (144 against 123 us at configuration 3)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="issue esa_score, esa_select_topk and esa_gather_kv as three calls instead of the one fused call "
                         "esa_score_select_gather (same results, three kernels more)")
    ap.add_argument("--fused-gather", action="store_true",
                    help="(the default now; kept so that older command lines still run)")
    ap.add_argument("--gather-call", action="store_true",
                    help="the step gathers the selected rows into a buffer (inside esa_score_select_gather, or by "
                         "esa_gather_kv with --separate-calls) and calls esa_attend on it, instead of the default, the "
                         "index-driven esa_attend_indexed")
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
    from esa_inputs import get_config

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = get_config(args.config)
    if args.seq:
        cfg = cfg.scaled(S=args.seq)
    if args.prompt:
        return whole_prompt(args, cfg, esa, torch, np)
    # One stream unless asked otherwise; always one stream under the profiler (one dispatch after the
    # other) and for decode-sized chunks, where nothing of the attention can start early.
    args.single_stream = not args.two_branches or args.eager or cfg.l_C < 16
    B = args.batch
    w = Workload(esa, torch, np, cfg, B)
    side = torch.cuda.Stream()

    try:
        eager_ms, ms_per_step, mode, graph = time_steps(torch, [make_step(esa, torch, w, args, side)], args.steps, args.warmup,
                                                        args.eager)
    except Exception as exc:                # a second graph branch is an optimisation, not a requirement
        if args.single_stream:
            raise
        print("bench.py: two-branch step failed (%s); timing the one-stream step" % exc, file=sys.stderr)
        torch.cuda.synchronize()
        args.single_stream = True
        eager_ms, ms_per_step, mode, graph = time_steps(torch, [make_step(esa, torch, w, args, side)], args.steps,
                                                        args.warmup, args.eager)
    del graph

    cold_ms = None
    if args.cold:
        per_copy = w.kc.numel() * w.kc.element_size()
        n_copies = max(3, int(320e6 // per_copy) + 1)
        copies = [w] + [w.cold_copy() for _ in range(n_copies - 1)]
        fns = [make_step(esa, torch, c, args, side) for c in copies]
        _, cold_ms, _, graph = time_steps(torch, fns, max(args.steps, 2 * n_copies), args.warmup, args.eager)
        del graph, fns, copies
        torch.cuda.empty_cache()

    # under the profiler (--eager) only the step's own launches are issued, so that per-kernel averages are the step's
    call_ms = per_call_times(esa, torch, np, w, args, with_variants=not args.eager)

    if args.copy_probe:
        # a plain copy of known size (2 x K bytes moved), the yardstick for the HBM traffic counters
        torch.empty_like(w.K).copy_(w.K)
        torch.cuda.synchronize()

    work, per_call_report = call_report(w, call_ms)
    # the dominant kernel: the call whose roofline time (algorithmic work over the chip's peak) is the longest, which
    # is the longest-running call for the prefill configurations; for one-token chunks the longest-running call is
    # the selection, a chain of launch-bound kernels over 1 MB of scores that no roofline describes
    dominant = max(CALLS, key=lambda c: max(work[c]["flops"] / (PEAK_BF16_TFLOPS * 1e12), work[c]["bytes"] / (PEAK_HBM_GBS * 1e9)))
    # the call of that name as the step makes it: the attention reads the selected rows through the index list
    timed_as = "attend_indexed" if dominant == "attend" and step_reads_through_indices(args, w.l_c) else dominant
    if work[dominant]["flops"] / (PEAK_BF16_TFLOPS * 1e12) > work[dominant]["bytes"] / (PEAK_HBM_GBS * 1e9):
        achieved = work[dominant]["flops"] / (call_ms[timed_as] * 1e-3) / 1e12
        roofline = {"kernel": "esa_" + timed_as, "bound": "mfma", "achieved": round(achieved, 2),
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "traffic": None}
        roofline["algorithmic_flops"] = round(work[dominant]["flops"])
    else:
        achieved = work[dominant]["bytes"] / (call_ms[timed_as] * 1e-3) / 1e9
        roofline = {"kernel": "esa_" + timed_as, "bound": "hbm", "achieved": round(achieved, 1),
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4),
                    "traffic": None}
    # `traffic` and `algorithmic_bytes` are both HBM bytes per launch of the dominant call
    traffic = None
    if B == 1 and csrc_tree_hash() == TRAFFIC_TREE:
        traffic = MEASURED_TRAFFIC_BYTES.get((cfg.name, cfg.S, dominant))
    roofline["traffic"] = None if traffic is None else round(traffic)
    roofline["algorithmic_bytes"] = round(work[dominant]["bytes"])
    roofline["traffic_measured_on_tree"] = TRAFFIC_TREE if traffic is not None else None
    roofline["per_call"] = per_call_report
    step_flops = sum(x["flops"] for x in work.values())
    roofline["step_tflops"] = round(step_flops / (ms_per_step * 1e-3) / 1e12, 2)

    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = cpu_oracle_baseline(w.layer, cfg, w.t0, w.l_c)
    workload = workload_text(w)
    n_tok = B * w.l_c
    indexed = step_reads_through_indices(args, w.l_c)

    decode = None
    if not args.no_decode and not cfg.decode and B == 1 and not args.seq:
        del w
        torch.cuda.empty_cache()
        decode = decode_record(esa, torch, np, args)

    value = n_tok / (ms_per_step * 1e-3)
    if cfg.decode:
        metric = "ESA decode tokens/s per layer at %dk ctx" % (cfg.S // 1024)
    else:
        metric = "ESA prefill tokens/s per layer at %dk ctx" % (cfg.S // 1024)
    result = {
        "metric": metric,
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": workload, "global_batch": B, "seq_len": cfg.S, "parallelism": "single GPU"},
        "roofline": roofline, "decode": decode, "cpu_baseline": cpu_baseline,
        "launch_mode": mode + (", one stream" if args.single_stream else ", two branches")
        + (", gather inside the attention kernel (esa_attend_indexed)" if indexed else "")
        + (", five separate calls" if args.separate_calls or not args.single_stream else
           (", score+select as one call" if indexed else
            ", score+select+gather as one call")), "eager_ms_per_step": round(eager_ms, 4),
        "cold_ms_per_step": None if cold_ms is None else round(cold_ms, 4),
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
    # k covers the middle segment in early chunks: every middle token is taken and no scores are read; the
    # buffer is allocated before the capture so that no fill is recorded into the graph
    no_scores = torch.empty(max(cfg.k, 1), dtype=torch.float32, device="cuda")
    no_q = torch.zeros((min(cfg.l_C, cfg.S), cfg.d_c), dtype=K.dtype, device="cuda")     # never read: stands in for Q'
    indexed = step_reads_through_indices(args, cfg.l_C)

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
            if n_mid > 0 and not args.separate_calls:
                # the step of the last-chunk benchmark: score + select as one call, the attention reads the
                # selected rows through the index list (or, with --gather-call, a gathered copy of them)
                if indexed:
                    _, idx, _, _ = esa.esa_score_select_gather(qc if n_mid > cfg.k else no_q, kc, i_end, l_start, cfg.k)
                    out = esa.esa_attend_indexed(Q[t0:t1], K, V, t0, cfg.l_I, cfg.l_L, idx)
                    continue
                _, idx, ks, vs = esa.esa_score_select_gather(qc if n_mid > cfg.k else no_q, kc, i_end, l_start, cfg.k, K, V)
            elif n_mid > 0:
                score = esa.esa_score(qc, kc, i_end, l_start) if n_mid > cfg.k else no_scores[:n_mid]
                idx = esa.esa_select_topk(score, cfg.k, base=i_end)
                ks, vs = esa.esa_gather_kv(K, V, idx)
            out = esa.esa_attend(Q[t0:t1], K, V, t0, cfg.l_I, cfg.l_L, ks, vs)
        return out

    prefill()
    eager_s = wall_ms(torch, prefill, 2) * 1e-3
    warm = torch.cuda.Stream()
    warm.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(warm):
        prefill()
    torch.cuda.current_stream().wait_stream(warm)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        graph_out = prefill()
    graph.replay()
    graph_s = wall_ms(torch, graph.replay, 3) * 1e-3
    ref = prefill()
    torch.cuda.synchronize()
    assert torch.equal(ref, graph_out), "graph replay and eager prefill disagree"
    print(json.dumps({
        "metric": "ESA prefill tokens/s per layer, whole prompt", "value": round(cfg.S / graph_s, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": 3, "warmup": 1, "ms_per_step": round(1e3 * graph_s, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "%s: whole prompt of %d tokens, %d chunks of %d, one layer" % (cfg.name, cfg.S, len(starts), cfg.l_C),
                   "global_batch": 1, "seq_len": cfg.S, "parallelism": "single GPU"},
        "launch_mode": "one HIP graph for the whole prefill"
        + (", five separate calls per chunk" if args.separate_calls else
           ", score+select as one call, gather inside the attention kernel" if indexed else
           ", score+select+gather as one call"), "eager_tokens_per_s": round(cfg.S / eager_s, 1),
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
