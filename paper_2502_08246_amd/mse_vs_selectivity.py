"""Approximation error of the sparse attention against selectivity, on a synthetic workload, with
the library's own calls (arXiv 2502.08246, Appendix B "Experiments": MSE between the approximate
and the exact attention output against the fraction of keys visited, random selection as the
baseline; Appendix E.4: the same for several numbers of partitions at fixed nprobe / nlist).

    python -m paper_2502_08246_amd.mse_vs_selectivity --workload cfg1_llama8b_128k --nlist 256,1024,4096

For every number of buckets: spherical k-means on the head's own key features (lloyd_iterations),
assign_keys, build_bucket_index; for every decode query the exact output (dense_decode_attention)
and the per-bucket attention mass (bucket_attention_mass).  A router is a score tensor [S,Hq,B]
handed to select_buckets (summed over the GQA group, Section 5):
    random          uniform random scores: a random subset of the buckets
    kmeans          the query scored against the key centroids (the symmetric baseline of Section 6.1)
    query_model     f_q trained with train_query_model for --train-steps steps (left out at 0)
    best_possible   the true attention mass of each bucket: the lists no router can beat on captured mass
For every visited fraction the report holds, per router, the selectivity (share of the keys in the
visited buckets, mean over heads) and the mean squared error of sparse_decode_attention against
the exact output (also relative to the mean square of the exact output).  At fraction 1 every
router visits every key and the error is that of the summation order alone.
torch is used for memory, random scores and the averages.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def evaluate_lists(q, exact, Ks, Vs, off, ln, selected, scale, n_keys):
    """One query set q [S,Hq,d] and lists `selected` [S,Hkv,nprobe] -> (mse, selectivity): mean squared
    difference between sparse_decode_attention over the lists and `exact` [S,Hq,d], and the share of
    the n_keys keys of a head that the lists visit, mean over (sequence, KV head)."""
    import paper_2502_08246_amd as saap

    out, _ = saap.sparse_decode_attention(q, Ks, Vs, off, ln, selected, scale)
    mse = float(((out.double() - exact.double()) ** 2).mean().item())
    visited = ln.gather(2, selected.to(ln.device, dtype=ln.dtype).long()).sum(-1).double()
    return mse, float((visited / n_keys).mean().item())


def curves(cfg, nlists, fractions, n_queries=16, lloyd_iters=5, train_steps=0, seed=0):
    """Runs the sweep on workload `cfg` (one sequence) and returns the report as a dict."""
    import torch

    import paper_2502_08246_amd as saap
    from synth import gen

    if not torch.cuda.is_available():
        raise RuntimeError("mse_vs_selectivity needs a GPU")
    saap.load_library()
    dev = "cuda:0"
    if cfg.S != 1:
        cfg = cfg.replace(S=1)
    scale = 1.0 / math.sqrt(cfg.d)
    cache = gen.make_cache(cfg, seed, dev)
    x, K, V = cache["x_keys"], cache["K"], cache["V"]
    xq, q = gen.make_queries(cfg, seed, dev, n_steps=n_queries)
    exact = [saap.dense_decode_attention(q[t], K, V, scale)[0] for t in range(n_queries)]
    mean_square = float(torch.stack(exact).double().pow(2).mean().item())
    g = torch.Generator(device=dev).manual_seed(seed + 7)

    report = {"workload": cfg.name, "N": cfg.N, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "queries": n_queries,
              "exact_output_mean_square": mean_square, "lloyd_iterations": lloyd_iters, "data": "synthetic",
              "curves": []}
    for B in nlists:
        cfg_b = cfg.replace(B=B, nprobe=min(max(round(cfg.nprobe * B / cfg.B), 1), B))
        stride = max(cfg.N // B, 1)
        init = x[0, :, ::stride][:, :B].contiguous()                     # B key features per head, evenly spaced
        cent = saap.lloyd_iterations(x, init, lloyd_iters)
        ids = saap.assign_keys(x, cent)
        off, ln, _, Ks, Vs = saap.build_bucket_index(ids, K, V, B, 0)
        routers = ["random", "kmeans", "best_possible"]
        weights = None
        if train_steps > 0:
            from .train_query_model import train
            weights = train(cfg_b, steps=train_steps, seed=seed, centroids=cent, return_weights=True)["weights"]
            routers.insert(2, "query_model")
        scores = {r: torch.empty(1, cfg.Hq, B, dtype=torch.float32, device=dev) for r in routers}
        nprobes = sorted({min(max(int(round(f * B)), 1), B) for f in fractions})
        acc = {(r, n): [0.0, 0.0] for r in routers for n in nprobes}
        for t in range(n_queries):
            scores["random"].copy_(torch.rand(1, cfg.Hq, B, generator=g, device=dev))
            saap.classify_queries(xq[t], None, None, cent, None, cfg.Hkv, out=scores["kmeans"])
            saap.bucket_attention_mass(q[t], Ks, off, ln, scale, out=scores["best_possible"])
            if weights is not None:
                saap.classify_queries(xq[t], *weights, cfg.Hkv, out=scores["query_model"])
            for r in routers:
                for n in nprobes:
                    sel = saap.select_buckets(scores[r], cfg.Hkv, n)
                    mse, share = evaluate_lists(q[t], exact[t], Ks, Vs, off, ln, sel, scale, cfg.N)
                    acc[(r, n)][0] += mse
                    acc[(r, n)][1] += share
        torch.cuda.synchronize()
        for n in nprobes:
            row = {"nlist": B, "nprobe": n, "nprobe_over_nlist": round(n / B, 5)}
            for r in routers:
                mse, share = (v / n_queries for v in acc[(r, n)])
                row[r] = {"selectivity": round(share, 5), "mse": mse, "relative_mse": mse / mean_square}
            report["curves"].append(row)
        del Ks, Vs
    return report


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="cfg1_llama8b_128k")
    ap.add_argument("--nlist", default="", help="comma-separated bucket counts (default: the workload's B)")
    ap.add_argument("--fractions", default="0.005,0.01,0.02,0.05,0.1,0.2,0.5,1.0", help="nprobe / nlist values")
    ap.add_argument("--queries", type=int, default=16, help="decode queries per head")
    ap.add_argument("--lloyd-iters", type=int, default=5)
    ap.add_argument("--train-steps", type=int, default=0, help="train f_q this many steps per nlist and add its curve")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    from synth import gen

    cfg = gen.CONFIGS[args.workload]
    nlists = [int(v) for v in args.nlist.split(",") if v] or [cfg.B]
    fractions = [float(v) for v in args.fractions.split(",") if v]
    try:
        report = curves(cfg, nlists, fractions, args.queries, args.lloyd_iters, args.train_steps, args.seed)
    except RuntimeError as e:
        print(e, file=sys.stderr)
        sys.exit(2)
    print(json.dumps(report))


if __name__ == "__main__":
    main()
