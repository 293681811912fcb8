"""Benchmark of the SAAP decode hot path on one MI355X.

One "step" is the decode-time hot path for one token of one layer over a resident, bucket-sorted
KV cache: classify_queries (logits) -> select_buckets_from_logits (the classifier's softmax folded
into the selection kernel) -> sparse_decode_attention (partials + merge in one launch).  The prefill
half (assign_keys, build_bucket_index) runs once during set-up and is timed separately; dense_decode_attention on the same cache is the in-repo baseline.

Cache hygiene: the timed loop cycles through `--query-sets` different queries (hence different
bucket selections), so that consecutive steps do not re-read the same 27 MB from the 256 MB
last-level cache.

Prints ONE JSON line: the step time as `value` (us per token per layer), `roofline` for the sparse
attention launch (algorithmic bytes per launch over its HIP-event time, against the 8 TB/s HBM peak and
against a measured streaming-read ceiling; `traffic` from the committed profiler counters),
`breakdown_us` per call, the dense baseline, the prefill timings and `cpu_baseline` (the CPU oracle on
the host cores).  Options add further objects: `--window`, `--layers`, `--kv8`, `--quality`.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix rate
BYTES_PER_KEY = 512     # one bf16 K row + one bf16 V row, d = 128


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="cfg1_llama8b_128k")
    ap.add_argument("--nprobe", type=int, default=0, help="override the workload's nprobe")
    ap.add_argument("--query-sets", type=int, default=64)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the oracle timing leg (0 = skip)")
    ap.add_argument("--slack", type=int, default=-1, help="free slots behind every bucket (default: 0, or 64 when the step appends)")
    ap.add_argument("--append", choices=["auto", "on", "off"], default="auto",
                    help="the step also stores the token's new key in its bucket (append_keys); "
                         "auto: on for the batched-decode workload, whose definition includes it")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense baseline (keeps profiler summaries to the sparse path)")
    ap.add_argument("--window", default="", help="also time the step with an attention sink + recent-key window, "
                    "e.g. 1+2047 (the paper's default): adds a `window` object to the output")
    ap.add_argument("--kv8", action="store_true",
                    help="also time the attention and the step on an 8-bit (FP8 E4M3) copy of the cache")
    ap.add_argument("--quality", action="store_true",
                    help="also report the attention mass the selection captures (bucket_attention_mass), for the "
                         "random-init classifier, for nearest-centroid routing and for the best possible selection")
    ap.add_argument("--layers", type=int, default=1,
                    help="also time a decode step through this many layers, each with its own synthetic cache, "
                         "centroids, classifier and index (e.g. 32 with --workload cfg4_layer_262k)")
    ap.add_argument("--path", choices=["plan", "list"], default="list",
                    help="list (default): the attention reads the selected lists itself, one team of workgroups per "
                         "list; plan: the selection writes the visit plan and the attention deals all lists' keys to "
                         "the workgroups in equal shares (slower on the benchmark workloads, robust to lists of "
                         "very different sizes)")
    ap.add_argument("--route", choices=["fused", "separate", "attend"], default="separate",
                    help="separate (default): classify_queries, the selection and the attention as three calls; attend: "
                         "select_attend, the selection inside the attention launch (list path); fused: classify_select, "
                         "which at batch 1 runs the selection inside the classifier's output launch (measured no faster: "
                         "13.5 against 13.1 us at the 128k workload)")
    ap.add_argument("--mixed-lengths", action="store_true",
                    help="batched workloads: the sequences hold N, N, N/2, N/2, N/4, N/4, ... keys instead of N each "
                         "(a serving batch of mixed context lengths; the keys beyond a sequence's length are left out "
                         "of its index), which makes the lists of the batch very unequal")
    ap.add_argument("--prefill-block", type=int, default=0, metavar="TQ",
                    help="also time prefill_sparse_attention on the last TQ tokens of the context (1+2047 always attended, "
                         "one list per token and KV head from the classifier); S * TQ * Hkv <= 4096")
    ap.add_argument("--no-fixed-cost", action="store_true",
                    help="skip the fixed-cost launches (same kernel, next to no bytes), so that a profiler's per-kernel "
                         "average covers real launches only")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain device copies of 256 MiB (reference for the HBM byte counters)")
    return ap.parse_args()


def timed(fn, iters, torch):
    """Average milliseconds of fn(i) over iters eager calls, bracketed by events on the current stream."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(iters):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


class GraphLoop:
    """`count` consecutive calls fn(i), i = 0..count-1, captured once as a HIP graph (the calls are
    launch-bound otherwise: a decode step is a handful of kernels of a few microseconds each).
    The captured work is exactly the eager work; nothing is skipped."""

    def __init__(self, fn, count, torch):
        self.torch, self.count = torch, count
        fn(0)                                   # allocate workspaces before the capture
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            for i in range(count):
                fn(i)
        torch.cuda.synchronize()

    def run(self, replays=1):
        for _ in range(replays):
            self.graph.replay()

    def timed_ms_per_call(self, replays):
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        self.run(1)
        torch.cuda.synchronize()
        e0.record()
        self.run(replays)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (replays * self.count)

    def replay_ms_per_call(self, replays):
        """Per-replay mean call time (ms), one event pair per replay: the spread over replays."""
        torch = self.torch
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
        self.run(1)
        torch.cuda.synchronize()
        ev[0].record()
        for r in range(replays):
            self.graph.replay()
            ev[r + 1].record()
        torch.cuda.synchronize()
        return [ev[r].elapsed_time(ev[r + 1]) / self.count for r in range(replays)]


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2502_08246_amd as saap
    from synth import gen

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    saap.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = gen.CONFIGS[args.workload]
    if args.nprobe:
        cfg = cfg.replace(nprobe=args.nprobe)
    scale = 1.0 / math.sqrt(cfg.d)
    T = args.query_sets
    with_append = args.append == "on" or (args.append == "auto" and cfg.name == "cfg3_batch8_128k")
    if args.slack < 0:
        args.slack = 64 if with_append else 0

    # ---------------------------------------------------------------- inputs (synthetic, seeded)
    cache = gen.make_cache(cfg, args.seed, dev)
    cent = gen.make_centroids(cfg, args.seed, dev, cache)
    xq, q = gen.make_queries(cfg, args.seed, dev, n_steps=T)
    W1, b1, W2, b2 = gen.make_classifier(cfg, args.seed, dev)
    torch.cuda.synchronize()

    # ---------------------------------------------------------------- prefill half, timed once warm
    ids = saap.assign_keys(cache["x_keys"], cent)
    torch.cuda.synchronize()
    ws = saap.workspace(0, dev)
    rescored = int(ws[65536 + 16380:65536 + 16384].view(torch.int32).item())   # diagnostic word of assign_keys
    seq_lengths = [cfg.N] * cfg.S
    if args.mixed_lengths:
        # an id outside [0,B) keeps a key out of the index: sequence s keeps its first N >> (s // 2) keys
        seq_lengths = [max(cfg.N >> (s // 2), 1) for s in range(cfg.S)]
        ids = ids.clone()
        for s_i, n_s in enumerate(seq_lengths):
            ids[s_i, :, n_s:] = -1
    index = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, args.slack)
    torch.cuda.synchronize()
    ms_assign = timed(lambda i: saap.assign_keys(cache["x_keys"], cent, out=ids), 3, torch)
    ms_build = timed(lambda i: saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, args.slack), 3, torch)
    # what the matrix pipes sustain on a bare loop of assign_keys' instruction: on the keys' own values (random
    # bf16), on small integers and on zeros; the published peak is reached on none of them
    mfma_probe = {}
    probe_sink = torch.zeros(4, dtype=torch.float32, device=dev)
    probe_ops = {"keys": cache["x_keys"].reshape(-1)[: 1 << 20],
                 "small_integers": torch.randint(-2, 3, (1 << 20,), device=dev).to(torch.bfloat16),
                 "zeros": torch.zeros(1 << 20, dtype=torch.bfloat16, device=dev)}
    for name, ops_t in probe_ops.items():
        flop_box = [saap.mfma_rate_probe(ops_t, 4096, probe_sink)]      # untimed first launch
        ms_p = timed(lambda i: flop_box.append(saap.mfma_rate_probe(ops_t, 4096, probe_sink)), 3, torch)
        mfma_probe[name] = round(flop_box[-1] / (ms_p * 1e-3) / 1e12, 1)
    off, ln, idx, Ks, Vs = index
    n_keys_total = cfg.Hkv * sum(seq_lengths)
    assign_flop = 2.0 * cfg.S * cfg.Hkv * cfg.N * cfg.B * cfg.d          # assign_keys ran on every key
    window = None
    if args.window:
        # the same cache indexed with a resident run (sink + recent keys); the step then also pushes
        # the token's own key: classify + select + windowed attention + window_push
        n_sink, n_recent = (int(v) for v in args.window.split("+"))
        w_slack = 64
        w_state = saap.build_windowed_index(ids, cache["K"], cache["V"], cfg.B, w_slack, n_sink, n_recent)
        window = (n_sink, n_recent, w_state)
    x_keys = cache.pop("x_keys")
    del x_keys

    # ---------------------------------------------------------------- decode buffers
    scores = torch.empty(cfg.S, cfg.Hq, cfg.B, dtype=torch.float32, device=dev)
    sel = torch.empty(cfg.S, cfg.Hkv, cfg.nprobe, dtype=torch.int32, device=dev)
    out = torch.empty(cfg.S, cfg.Hq, cfg.d, dtype=torch.float32, device=dev)
    lse = torch.empty(cfg.S, cfg.Hq, dtype=torch.float32, device=dev)
    sel_sets = torch.empty(T, cfg.S, cfg.Hkv, cfg.nprobe, dtype=torch.int32, device=dev)

    # the classifier's softmax is folded into the selection kernel (one launch less per step)
    def classify(i):
        saap.classify_queries(xq[i % T], W1, b1, W2, b2, cfg.Hkv, output_kind=saap.LOGITS, out=scores)

    planned = args.path == "plan"
    plan = torch.empty(saap.visit_plan_ints(cfg.S, cfg.Hq, cfg.Hkv, cfg.nprobe), dtype=torch.int32, device=dev)
    plan_sets = torch.empty(T, plan.numel(), dtype=torch.int32, device=dev)

    def select(i):
        if planned:
            saap.select_buckets_planned(scores, off, ln, cfg.Hkv, cfg.nprobe, input_kind=saap.LOGITS, out=sel, plan=plan)
        else:
            saap.select_buckets_from_logits(scores, cfg.Hkv, cfg.nprobe, out=sel)

    def attend(i):
        if planned:
            saap.planned_decode_attention(q[i % T], Ks, Vs, plan, cfg.nprobe, scale, out=out, lse=lse)
        else:
            saap.sparse_decode_attention(q[i % T], Ks, Vs, off, ln, sel, scale, out=out, lse=lse)

    if with_append:
        # the T tokens whose keys get appended, drawn like the cache; replays append the same T keys
        # again, the copies pile up in the slack (64 slots per bucket hold the whole run)
        new = gen.make_cache(cfg.replace(N=T), args.seed, dev)
        a_x, a_k, a_v = (new[k].permute(2, 0, 1, 3).contiguous() for k in ("x_keys", "K", "V"))   # [T,S,Hkv,d]
        a_pos = (cfg.N + torch.arange(T, dtype=torch.int32, device=dev)).repeat_interleave(cfg.S).reshape(T, cfg.S).contiguous()
        a_flag = torch.zeros(4, dtype=torch.int32, device=dev)
        a_ids = torch.empty(cfg.S, cfg.Hkv, dtype=torch.int32, device=dev)

        # the index as built: the 8-bit run fills the slack from the start again, and the host timing leg
        # reads keys by position, so it must not see the positions appended beyond the N it holds
        ln_built, idx_built = ln.clone(), idx.clone()

    def append(i):
        saap.append_keys(a_x[i % T], a_k[i % T], a_v[i % T], a_pos[i % T], cent, None, off, ln, idx, Ks, Vs,
                         overflow_flag=a_flag, new_ids=a_ids)

    def route(i):
        saap.classify_select(xq[i % T], W1, b1, W2, b2, cfg.Hkv, cfg.nprobe, off=off, ln=ln, logits=scores, out=sel,
                             plan=plan if planned else None)

    scores_sets = torch.empty(T, cfg.S, cfg.Hq, cfg.B, dtype=torch.float32, device=dev)

    def select_attend_set(i):
        saap.select_attend(scores_sets[i % T], q[i % T], Ks, Vs, off, ln, cfg.nprobe, scale, selected=sel, out=out, lse=lse)

    def step(i):
        if args.route == "attend":
            classify(i)
            saap.select_attend(scores, q[i % T], Ks, Vs, off, ln, cfg.nprobe, scale, selected=sel, out=out, lse=lse)
        else:
            if args.route == "fused":
                route(i)
            else:
                classify(i)
                select(i)
            attend(i)
        if with_append:
            append(i)

    # selections of every query set (for the byte accounting and the per-kernel loops)
    for t in range(T):
        classify(t)
        scores_sets[t].copy_(scores)
        saap.select_buckets_planned(scores, off, ln, cfg.Hkv, cfg.nprobe, input_kind=saap.LOGITS, out=sel_sets[t],
                                    plan=plan_sets[t])
    torch.cuda.synchronize()
    keys_per_set = torch.gather(ln.unsqueeze(0).expand(T, -1, -1, -1).to(torch.int64), 3, sel_sets.to(torch.int64)).sum(dim=(1, 2, 3))
    keys_touched = float(keys_per_set.to(torch.float64).mean().item())   # per step (all sequences, all KV heads)
    bytes_step = keys_touched * BYTES_PER_KEY

    # ---------------------------------------------------------------- the timed region
    # K steps = K // T replays of a T-step graph plus one replay of a (K % T)-step graph.
    g_full = GraphLoop(step, T, torch)
    rem = args.steps % T
    g_rem = GraphLoop(step, rem, torch) if rem else None
    warm = args.warmup
    while warm > 0:
        g_full.run(1)
        warm -= T
    if g_rem:
        g_rem.run(1)            # every graph of the timed region has been replayed once before the clock starts
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g_full.run(args.steps // T)
    if g_rem:
        g_rem.run(1)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    us_token_layer = wall_ms * 1e3 / cfg.S
    # the same step with the selection inside the attention launch (select_attend), for the record beside `value`
    alt_route = None
    if args.route == "separate" and not planned:
        def step_attend(i):
            classify(i)
            saap.select_attend(scores, q[i % T], Ks, Vs, off, ln, cfg.nprobe, scale, selected=sel, out=out, lse=lse)
            if with_append:
                append(i)

        ms_alt = GraphLoop(step_attend, T, torch).timed_ms_per_call(max(1, args.steps // T))
        alt_route = {"step": "classify_queries (logits) + select_attend" + (" + append_keys" if with_append else ""),
                     "us_per_token_layer": round(ms_alt * 1e3 / cfg.S, 3), "how": "bench.py --route attend"}

    # ---------------------------------------------------------------- per-call timings (events, same stream)
    def attend_set(i):
        if planned:
            saap.planned_decode_attention(q[i % T], Ks, Vs, plan_sets[i % T], cfg.nprobe, scale, out=out, lse=lse)
        else:
            saap.sparse_decode_attention(q[i % T], Ks, Vs, off, ln, sel_sets[i % T], scale, out=out, lse=lse)

    def dense(i):
        saap.dense_decode_attention(q[i % T], Ks, Vs, scale, off=off, ln=ln, out=out, lse=lse)

    reps = max(2, args.steps // T)
    g_attn = GraphLoop(attend_set, T, torch)
    ms_attn = g_attn.timed_ms_per_call(reps)
    spread = np.percentile(np.array(g_attn.replay_ms_per_call(max(reps, 20))) * 1e3, [10, 50, 90])
    ms_classify = GraphLoop(classify, T, torch).timed_ms_per_call(reps)
    ms_select = GraphLoop(select, T, torch).timed_ms_per_call(reps)
    ms_route = GraphLoop(route, T, torch).timed_ms_per_call(reps)
    ms_select_attend = GraphLoop(select_attend_set, T, torch).timed_ms_per_call(reps)
    ms_append = GraphLoop(append, T, torch).timed_ms_per_call(2) if with_append else None
    ms_dense = None if args.no_dense else GraphLoop(dense, 8, torch).timed_ms_per_call(3)
    # Fixed cost of the attention launch: the same call on the same lists with every bucket one key long, i.e.
    # the same grid, prologue, partial results, arrival counters and merge with next to no bytes to stream.
    ln_one = torch.ones_like(ln)
    if planned:
        plan_one = torch.stack([saap.build_visit_plan(sel_sets[t], off, ln_one, cfg.Hq) for t in range(T)])

    def attend_fixed(i):
        if planned:
            saap.planned_decode_attention(q[i % T], Ks, Vs, plan_one[i % T], cfg.nprobe, scale, out=out, lse=lse)
        else:
            saap.sparse_decode_attention(q[i % T], Ks, Vs, off, ln_one, sel_sets[i % T], scale, out=out, lse=lse)

    ms_fixed = None if args.no_fixed_cost else GraphLoop(attend_fixed, T, torch).timed_ms_per_call(reps)
    achieved = bytes_step / (ms_attn * 1e-3) / 1e9
    # streaming-read ceiling of this device: non-temporal 16-byte loads over the whole sorted cache
    sink = torch.zeros(4096, dtype=torch.int32, device=dev)
    kv_bytes = Ks.numel() * Ks.element_size() + Vs.numel() * Vs.element_size()

    def probe(i):
        saap.stream_read_probe(Ks, sink)
        saap.stream_read_probe(Vs, sink)

    ms_probe = GraphLoop(probe, 4, torch).timed_ms_per_call(3)
    ceiling = kv_bytes / (ms_probe * 1e-3) / 1e9

    window_result = None
    if window:
        n_sink, n_recent, (w_off, w_ln, w_idx, w_Ks, w_Vs, w_res) = window
        new = gen.make_cache(cfg.replace(N=T), args.seed, dev)          # T tokens to push, drawn like the cache
        xn, kn, vn = (new[k].permute(2, 0, 1, 3).contiguous() for k in ("x_keys", "K", "V"))   # [T,S,Hkv,d]
        pos = (cfg.N + torch.arange(T, dtype=torch.int32, device=dev)).repeat_interleave(cfg.S).reshape(T, cfg.S).contiguous()
        w_flag = torch.zeros(4, dtype=torch.int32, device=dev)
        w_new = torch.empty(cfg.S, cfg.Hkv, dtype=torch.int32, device=dev)

        def w_attend(i):
            saap.windowed_decode_attention(q[i % T], w_Ks, w_Vs, w_off, w_ln, sel_sets[i % T], cfg.B, scale, out=out, lse=lse)

        def w_push(i):
            # replays push the same T positions again: the ring slots are rewritten and the displaced
            # copies pile up in the slack, which is sized for the whole run
            saap.window_push(xn[i % T], kn[i % T], vn[i % T], pos[i % T], cent, None, w_off, w_ln, w_idx, w_Ks, w_Vs,
                             w_res, n_sink, n_recent, overflow_flag=w_flag, new_ids=w_new)

        def w_step(i):
            classify(i)
            select(i)
            saap.windowed_decode_attention(q[i % T], w_Ks, w_Vs, w_off, w_ln, sel, cfg.B, scale, out=out, lse=lse)
            w_push(i)

        def w_step_attend(i):
            classify(i)
            saap.select_attend(scores, q[i % T], w_Ks, w_Vs, w_off, w_ln, cfg.nprobe, scale, selected=sel, out=out, lse=lse,
                               resident_run=cfg.B)
            w_push(i)

        w_keys = torch.gather(w_ln[:, :, :cfg.B].unsqueeze(0).expand(T, -1, -1, -1).to(torch.int64), 3,
                              sel_sets.to(torch.int64)).sum(dim=(1, 2, 3)).to(torch.float64).mean().item()
        w_keys += float(w_ln[:, :, cfg.B].sum().item())
        w_reps = max(2, min(reps, 4))
        ms_w_attn = GraphLoop(w_attend, T, torch).timed_ms_per_call(w_reps)
        ms_w_push = GraphLoop(w_push, T, torch).timed_ms_per_call(w_reps)
        ms_w_step = GraphLoop(w_step, T, torch).timed_ms_per_call(w_reps)
        ms_w_step_attend = GraphLoop(w_step_attend, T, torch).timed_ms_per_call(w_reps)
        torch.cuda.synchronize()
        window_result = {
            "n_sink": n_sink, "n_recent": n_recent, "slack": 64,
            "step_us_per_token_layer": round(ms_w_step * 1e3 / cfg.S, 3),
            "step": "classify_queries + select_buckets + windowed_decode_attention + window_push",
            "step_with_select_attend_us_per_token_layer": round(ms_w_step_attend * 1e3 / cfg.S, 3),
            "windowed_decode_attention_us": round(ms_w_attn * 1e3, 3),
            "window_push_us": round(ms_w_push * 1e3, 3),
            "bytes_per_launch": round(w_keys * BYTES_PER_KEY),
            "achieved_GBps": round(w_keys * BYTES_PER_KEY / (ms_w_attn * 1e-3) / 1e9, 1),
            "overflow_flag": int(w_flag[0].item()),
        }

    quality_result = None
    if args.quality:
        # Share of each query's softmax attention that lies in the visited buckets, mean over heads and
        # query sets: for the lists of the random-init classifier (the timed step), for the symmetric
        # "K-means" routing (queries scored against the key centroids, one-layer model) and for the
        # nprobe buckets that hold the most attention (the ceiling for any router at this nprobe).
        G = cfg.Hq // cfg.Hkv
        mass = torch.empty(cfg.S, cfg.Hq, cfg.B, dtype=torch.float32, device=dev)
        km_scores = torch.empty(cfg.S, cfg.Hq, cfg.B, dtype=torch.float32, device=dev)
        km_sel = torch.empty(cfg.S, cfg.Hkv, cfg.nprobe, dtype=torch.int32, device=dev)
        TQ = min(T, 16)
        acc = {"classifier_random_init": 0.0, "kmeans_routing": 0.0, "best_possible": 0.0}
        ms_mass = timed(lambda i: saap.bucket_attention_mass(q[i % T], Ks, off, ln, scale, out=mass), 4, torch)
        for t in range(TQ):
            saap.bucket_attention_mass(q[t], Ks, off, ln, scale, out=mass)
            saap.classify_queries(xq[t], None, None, cent, None, cfg.Hkv, out=km_scores)
            saap.select_buckets(km_scores, cfg.Hkv, cfg.nprobe, out=km_sel)
            group_mass = mass.view(cfg.S, cfg.Hkv, G, cfg.B)
            for key, lists in (("classifier_random_init", sel_sets[t]), ("kmeans_routing", km_sel)):
                idx_q = lists.to(torch.int64).unsqueeze(2).expand(-1, -1, G, -1)
                acc[key] += float(torch.gather(group_mass, 3, idx_q).sum(-1).mean().item())
            # best lists under GQA: the nprobe buckets with the largest mass summed over the group
            best = torch.topk(group_mass.sum(2), cfg.nprobe, dim=-1).indices.unsqueeze(2).expand(-1, -1, G, -1)
            acc["best_possible"] += float(torch.gather(group_mass, 3, best).sum(-1).mean().item())
        quality_result = {k: round(v / TQ, 4) for k, v in acc.items()}
        quality_result.update({"query_sets": TQ, "metric": "mean share of softmax attention mass inside the visited buckets",
                               "bucket_attention_mass_us": round(ms_mass * 1e3, 2)})

    prefill_result = None
    if args.prefill_block:
        # a block of prompt tokens at the end of the context, every token with its own lists (reading of the
        # Conclusion's "prefill-time sparse attention": the decode-time rule per token, causal)
        Tq, p_sink, p_recent = args.prefill_block, 1, 2047
        if cfg.S * Tq * cfg.Hkv > 4096 or Tq >= cfg.N - p_sink - p_recent or args.mixed_lengths or with_append:
            print("bench.py --prefill-block: S * TQ * Hkv must be <= 4096, TQ well below N, equal lengths, a step without append", file=sys.stderr)
            sys.exit(2)
        xq_t, q_t = gen.make_queries(cfg, args.seed + 1, dev, n_steps=Tq)
        xq_b = torch.stack(list(xq_t), 1).contiguous()            # [S,Tq,Hq,d]
        q_b = torch.stack(list(q_t), 1).contiguous()
        lg_b = saap.classify_queries(xq_b.view(cfg.S * Tq, cfg.Hq, cfg.d), W1, b1, W2, b2, cfg.Hkv, output_kind=saap.LOGITS)
        sel_b = saap.select_buckets_from_logits(lg_b, cfg.Hkv, cfg.nprobe)
        sel_b = sel_b.view(cfg.S, Tq, cfg.Hkv, cfg.nprobe).permute(0, 2, 1, 3).contiguous()      # [S,Hkv,Tq,nprobe]
        pos0 = torch.full((cfg.S,), cfg.N - Tq, dtype=torch.int32, device=dev)
        p_out = torch.empty(cfg.S, Tq, cfg.Hq, cfg.d, dtype=torch.float32, device=dev)
        p_lse = torch.empty(cfg.S, Tq, cfg.Hq, dtype=torch.float32, device=dev)
        p_off, p_ln, p_idx, p_Ks, p_Vs = index

        def prefill_block(i):
            saap.prefill_sparse_attention(q_b, cache["K"], cache["V"], p_Ks, p_Vs, p_off, p_ln, p_idx, sel_b, pos0, p_sink,
                                          p_recent, scale, out=p_out, lse=p_lse)

        ms_block = GraphLoop(prefill_block, 4, torch).timed_ms_per_call(5)
        # keys each (token, KV head) attends: sink + recent + the listed buckets' members between them
        visited = 0
        first_hi = cfg.N - Tq + 1 - p_recent                       # token 0 attends bucket members at positions < first_hi
        for s_i in range(cfg.S):
            for h_i in range(cfg.Hkv):
                row = ids[s_i, h_i].to(torch.int64)
                counts = torch.bincount(row[p_sink:first_hi], minlength=cfg.B)
                steps_in = torch.nn.functional.one_hot(row[first_hi:first_hi + Tq - 1], cfg.B).cumsum(0)
                per_tok = torch.cat([counts[None], counts[None] + steps_in], 0)            # [Tq,B]
                visited += int(torch.gather(per_tok, 1, sel_b[s_i, h_i].to(torch.int64)).sum().item())
        visited += cfg.S * cfg.Hkv * Tq * (p_sink + p_recent)
        prefill_result = {
            "block_tokens": Tq, "n_sink": p_sink, "n_recent": p_recent, "nprobe": cfg.nprobe,
            "prefill_sparse_attention_us_per_block": round(ms_block * 1e3, 2),
            "us_per_token": round(ms_block * 1e3 / (cfg.S * Tq), 3),
            "keys_attended_per_token_and_kv_head": round(visited / (cfg.S * cfg.Hkv * Tq), 1),
            "bytes_per_block": visited * BYTES_PER_KEY,
            "achieved_GBps": round(visited * BYTES_PER_KEY / (ms_block * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(visited * BYTES_PER_KEY / (ms_block * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "note": "every token reads its own keys (512 B per attended key); dense causal attention of the same block "
                    "would read the whole context once per block",
        }

    kv8_result = None
    if args.kv8:
        # the same index over an 8-bit copy of the sorted cache (256 bytes per visited key)
        K8, V8, k_sc, v_sc = saap.quantize_kv(Ks, Vs)
        torch.cuda.synchronize()
        ms_quant = timed(lambda i: saap.quantize_kv(Ks, Vs), 2, torch)

        def attend8_set(i):
            saap.sparse_decode_attention_fp8(q[i % T], K8, V8, k_sc, v_sc, off, ln, sel_sets[i % T], scale, out=out, lse=lse)

        ln8, idx8 = (ln_built.clone(), idx_built.clone()) if with_append else (ln, idx)
        if with_append:
            a_flag8 = torch.zeros(4, dtype=torch.int32, device=dev)

        def step8(i):
            classify(i)
            select(i)
            saap.sparse_decode_attention_fp8(q[i % T], K8, V8, k_sc, v_sc, off, ln8, sel, scale, out=out, lse=lse)
            if with_append:
                saap.append_keys_fp8(a_x[i % T], a_k[i % T], a_v[i % T], a_pos[i % T], cent, None, off, ln8, idx8, K8, V8,
                                     k_sc, v_sc, overflow_flag=a_flag8, new_ids=a_ids)

        def dense8(i):
            saap.dense_decode_attention_fp8(q[i % T], K8, V8, k_sc, v_sc, scale, off=off, ln=ln, out=out, lse=lse)

        ms_attn8 = GraphLoop(attend8_set, T, torch).timed_ms_per_call(reps)
        ms_step8 = GraphLoop(step8, T, torch).timed_ms_per_call(reps)
        ms_dense8 = None if args.no_dense else GraphLoop(dense8, 8, torch).timed_ms_per_call(3)
        kv8_result = {
            "format": "OCP FP8 E4M3, one power-of-two scale per (sequence, KV head) and tensor",
            "step_us_per_token_layer": round(ms_step8 * 1e3 / cfg.S, 3),
            "step": "classify_queries (logits) + select_buckets_from_logits + sparse_decode_attention_fp8"
                    + (" + append_keys_fp8" if with_append else ""),
            "append_overflow_flag": int(a_flag8[0].item()) if with_append else None,
            "sparse_decode_attention_fp8_us": round(ms_attn8 * 1e3, 3),
            "bytes_per_launch": round(keys_touched * BYTES_PER_KEY / 2),
            "achieved_GBps": round(keys_touched * BYTES_PER_KEY / 2 / (ms_attn8 * 1e-3) / 1e9, 1),
            "speedup_vs_16bit_attention": round(ms_attn / ms_attn8, 2),
            "dense_decode_attention_fp8_us": None if ms_dense8 is None else round(ms_dense8 * 1e3, 3),
            "quantize_kv_ms": round(ms_quant, 3),
        }
        del K8, V8

    layers_result = None
    if args.layers > 1:
        # A decode step through L layers: every layer has its own cache (seed + layer), centroids,
        # classifier and index, so nothing a layer reads was left in the caches by the layer before.
        TL = min(T, 8)
        layers = [dict(W=(W1, b1, W2, b2), off=off, ln=ln, Ks=Ks, Vs=Vs, xq=xq[:TL], q=q[:TL])]
        t_build0 = time.perf_counter()
        for l in range(1, args.layers):
            c_l = gen.make_cache(cfg, args.seed + l, dev)
            cent_l = gen.make_centroids(cfg, args.seed + l, dev, c_l)
            ids_l = saap.assign_keys(c_l["x_keys"], cent_l)
            o_l, n_l, _, K_l, V_l = saap.build_bucket_index(ids_l, c_l["K"], c_l["V"], cfg.B, 0)
            xq_l, q_l = gen.make_queries(cfg, args.seed + l, dev, n_steps=TL)
            layers.append(dict(W=gen.make_classifier(cfg, args.seed + l, dev), off=o_l, ln=n_l, Ks=K_l, Vs=V_l,
                               xq=xq_l, q=q_l))
            del c_l, ids_l, cent_l
            torch.cuda.synchronize()
            print(f"layer {l} indexed", file=sys.stderr, flush=True)
        build_s = time.perf_counter() - t_build0

        def model_step(i):
            for L in layers:
                saap.classify_queries(L["xq"][i % TL], *L["W"], cfg.Hkv, output_kind=saap.LOGITS, out=scores)
                saap.select_buckets_from_logits(scores, cfg.Hkv, cfg.nprobe, out=sel)
                saap.sparse_decode_attention(L["q"][i % TL], L["Ks"], L["Vs"], L["off"], L["ln"], sel, scale, out=out, lse=lse)

        def model_dense(i):
            for L in layers:
                saap.dense_decode_attention(L["q"][i % TL], L["Ks"], L["Vs"], scale, off=L["off"], ln=L["ln"], out=out, lse=lse)

        ms_model = GraphLoop(model_step, TL, torch).timed_ms_per_call(max(2, min(reps, 8)))
        ms_model_dense = None if args.no_dense else GraphLoop(model_dense, 2, torch).timed_ms_per_call(2)
        layers_result = {
            "layers": args.layers,
            "step": "per layer: classify_queries (logits) + select_buckets_from_logits + sparse_decode_attention",
            "us_per_token": round(ms_model * 1e3 / cfg.S, 2),
            "us_per_token_layer": round(ms_model * 1e3 / cfg.S / args.layers, 3),
            "dense_attention_us_per_layer": None if ms_model_dense is None else round(ms_model_dense * 1e3 / args.layers, 3),
            "sorted_cache_GiB": round(sum(L["Ks"].numel() * 2 * L["Ks"].element_size() for L in layers) / 2**30, 2),
            "prefill_s_all_layers": round(build_s, 1),
        }

    # HBM bytes per launch of the dominant kernel, from the committed rocprofv3 counter summary of
    # this workload (a separate profiling run; see profiles/): null if there is none.
    traffic = None
    tag = cfg.name + (f"_nprobe{cfg.nprobe}" if args.nprobe else "")
    prof = os.path.join(ROOT, "profiles", f"sparse_attention_{tag}_hbm_traffic.md")
    traffic_source = f"no committed counter summary for this workload (profiles/{os.path.basename(prof)} absent)"
    if os.path.exists(prof):
        for line in open(prof):
            if line.startswith("attn_kernel traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
                traffic_source = (f"profiles/{os.path.basename(prof)}: rocprofv3 FETCH_SIZE + WRITE_SIZE of a separate run "
                                  "of this command, scaled by a plain copy of known size")

    # the paper's own timing (another machine; context only), from the cited fixture
    paper_ctx = {"hardware": "H100 80GB, one head, 171k context (Section 6.2, timing table)"}
    for line in open(os.path.join(ROOT, "tests", "golden", "timing_table.txt")):
        if not line.startswith("#") and line.strip():
            name, _, us = line.split()
            paper_ctx[{"flashattention_v2": "flashattention_v2_us", "saap_nprobe32": "saap_us"}[name]] = float(us)

    result = {
        "metric": "sparse decode attention us/token/layer @128k-500k ctx; HBM GB/s vs roofline",
        "value": round(us_token_layer, 3),
        "unit": "us/token/layer",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {
            "workload": cfg.name, "S": cfg.S, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "d": cfg.d, "N": cfg.N, "B": cfg.B,
            "nprobe": cfg.nprobe, "classifier": f"{cfg.d}->{cfg.hidden}->{cfg.B}", "query_sets": T,
            "step": ("classify_queries (logits) + select_attend" if args.route == "attend" else
                     ("classify_select" if args.route == "fused" else
                      "classify_queries (logits) + " + ("select_buckets_planned" if planned else "select_buckets_from_logits"))
                     + (" + planned_decode_attention" if planned else " + sparse_decode_attention"))
                    + (" + append_keys" if with_append else ""),
            "slack": args.slack, "launch": "hip graph", "path": args.path, "route": args.route,
            "sequence_lengths": seq_lengths if args.mixed_lengths else None,
        },
        "roofline": {
            "kernel": ("attn_plan_kernel<bf16,G=4> (planned_decode_attention, partials + merge)" if planned else
                       "attn_kernel<bf16,G=4,list> (sparse_decode_attention, partials + merge)"),
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_source": traffic_source,
            "bytes_per_launch": round(bytes_step),
            "avg_launch_us": round(ms_attn * 1e3, 3),
            "fixed_cost_us": None if ms_fixed is None else round(ms_fixed * 1e3, 3),
            "fixed_cost_how": "the same launch on the same lists with every bucket one key long",
            "stream_us_at_read_ceiling": round(bytes_step / (ceiling * 1e9) * 1e6, 3),
            "fixed_plus_stream_us": None if ms_fixed is None else round(ms_fixed * 1e3 + bytes_step / (ceiling * 1e9) * 1e6, 3),
            "launch_us_p10_p50_p90": [round(float(v), 3) for v in spread],
            "stream_read_ceiling_GBps": round(ceiling, 1),
            "frac_of_stream_read_ceiling": round(achieved / ceiling, 4),
        },
        "breakdown_us": {
            "classify_queries_logits": round(ms_classify * 1e3, 3),
            "select_buckets_from_logits": round(ms_select * 1e3, 3),
            "classify_select": round(ms_route * 1e3, 3),
            "sparse_decode_attention": round(ms_attn * 1e3, 3),
            "select_attend": round(ms_select_attend * 1e3, 3),
            "dense_decode_attention": None if ms_dense is None else round(ms_dense * 1e3, 3),
            "append_keys": None if ms_append is None else round(ms_append * 1e3, 3),
        },
        "dense": None if ms_dense is None else {
            "us": round(ms_dense * 1e3, 3),
            "GBps": round(n_keys_total * BYTES_PER_KEY / (ms_dense * 1e-3) / 1e9, 1),
            "speedup_sparse_vs_dense": round(ms_dense / ms_attn, 2),
        },
        "selectivity": round(keys_touched / n_keys_total, 5),
        "prefill": {
            "assign_keys_ms": round(ms_assign, 3),
            "assign_keys_TFLOPs": round(assign_flop / (ms_assign * 1e-3) / 1e12, 1),
            "assign_keys_frac_of_bf16_mfma_peak": round(assign_flop / (ms_assign * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "assign_keys_rescored": rescored,
            "mfma_32x32x16_bf16_bare_loop_TFLOPs_by_operand_values": mfma_probe,
            "build_bucket_index_ms": round(ms_build, 3),
            "build_bucket_index_GBps": round(2.0 * n_keys_total * BYTES_PER_KEY / (ms_build * 1e-3) / 1e9, 1),
        },
        "paper_context": paper_ctx,
    }
    if window_result:
        result["window"] = window_result
    if layers_result:
        result["model_step"] = layers_result
    if kv8_result:
        result["kv8"] = kv8_result
    if prefill_result:
        result["prefill_sparse_attention"] = prefill_result
    if alt_route:
        result["select_attend_route"] = alt_route
    if quality_result:
        result["routing_quality"] = quality_result
    if with_append:
        result["append_overflow_flag"] = int(a_flag[0].item())

    if args.calibrate_copy:
        # a plain copy of known size: the profiler's FETCH_SIZE / WRITE_SIZE for it give the
        # scale between counter units and bytes
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["calibrate_copy_bytes"] = int(src.numel())

    # ---------------------------------------------------------------- oracle timing leg (host cores)
    if args.cpu_seconds > 0:
        from oracle import ref
        h = gen.to_host_f32
        threads = min(16, os.cpu_count() or 1)
        ref.set_threads(threads)
        threads = ref.get_threads()                       # what OpenMP will really use
        cpu_model = "unknown"
        try:
            for line in open("/proc/cpuinfo"):
                if line.lower().startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        hK, hV = h(cache["K"]), h(cache["V"])
        h_off = off.cpu().numpy()
        h_ln, h_idx = ((ln_built if with_append else ln).cpu().numpy(), (idx_built if with_append else idx).cpu().numpy())
        hW1, hb1, hW2, hb2 = h(W1), h(b1), h(W2), h(b2)
        hxq, hq = h(xq), h(q)
        done, t_cpu0 = 0, time.perf_counter()
        while True:
            sc = ref.classify_queries(hxq[done % T], hW1, hb1, hW2, hb2, cfg.Hkv)
            se = ref.select_buckets(sc, cfg.Hkv, cfg.nprobe)
            ref.sparse_decode_attention(hq[done % T], hK, hV, h_off, h_ln, h_idx, se, scale)
            done += 1
            el = time.perf_counter() - t_cpu0
            if el > args.cpu_seconds or done >= 10 * T:
                break
        # context figures, one call each: the same sparse step on one thread, and the dense oracle
        ref.set_threads(1)
        t1 = time.perf_counter()
        sc = ref.classify_queries(hxq[0], hW1, hb1, hW2, hb2, cfg.Hkv)
        se = ref.select_buckets(sc, cfg.Hkv, cfg.nprobe)
        ref.sparse_decode_attention(hq[0], hK, hV, h_off, h_ln, h_idx, se, scale)
        single_us = (time.perf_counter() - t1) * 1e6 / cfg.S
        ref.set_threads(threads)
        t1 = time.perf_counter()
        ref.dense_decode_attention(np.ascontiguousarray(hq[0][:1]), np.ascontiguousarray(hK[:1]), np.ascontiguousarray(hV[:1]), scale)
        dense_cpu_us = (time.perf_counter() - t1) * 1e6
        result["cpu_baseline"] = {
            "value": round(el / done * 1e6 / cfg.S, 1),
            "unit": "us/token/layer",
            "cores": threads,
            "host_cpu_count": os.cpu_count(),
            "cpu_model": cpu_model,
            "kind": "oracle",
            "sample": f"{done} decode steps (classify + select + sparse attention) of the same workload, "
                      f"{threads} OpenMP threads over (sequence, head) in attention; classifier and selection single-threaded",
            "single_thread_us": round(single_us, 1),
            "dense_oracle_us": round(dense_cpu_us, 1),
            "dense_oracle_sample": f"one dense call on sequence 0 (all {cfg.Hkv} KV heads, N={cfg.N}), {threads} threads",
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
