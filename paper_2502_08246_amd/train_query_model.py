"""Trains the query model f_q on a synthetic workload with the library's own calls and reports the
attention mass its lists capture (arXiv 2502.08246, Section 4 "Query assignment function", Eq. 1).

    python -m paper_2502_08246_amd.train_query_model --workload cfg1_llama8b_128k --steps 400

Steps, all on the GPU: keys are assigned and indexed (assign_keys, build_bucket_index); for every
training query the target row of A * H_k comes from bucket_attention_mass_batch; training steps are
query_model_loss_grads + adam_update on fp32 weights, one weight set per KV head (its G query
heads share it, as in the decode step).  Evaluation on held-out queries: classify_queries +
select_buckets with the trained weights, then the share of each query's attention mass inside
the selected buckets, next to the random-init model, nearest-centroid routing and the best
possible lists.  torch is used for memory, reshapes and the final averages only.
Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def parse():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="cfg1_llama8b_128k")
    ap.add_argument("--train-queries", type=int, default=2048, help="decode queries per head in the training set")
    ap.add_argument("--eval-queries", type=int, default=64, help="held-out decode queries per head")
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--batch", type=int, default=1024, help="rows per weight set and step")
    ap.add_argument("--lr", type=float, default=1e-3, help="Adam learning rate (the paper: 1e-5 for 40k iterations)")
    ap.add_argument("--batch-norm", action="store_true",
                    help="train the model with batch normalisation of the hidden layer (Section 6.1) and fold it for inference")
    ap.add_argument("--seed", type=int, default=0)
    return ap.parse_args()


def train(cfg, train_queries=2048, eval_queries=64, steps=400, batch=1024, lr=1e-3, seed=0, centroids=None,
          return_weights=False, batch_norm=False):
    """Runs the whole procedure on workload `cfg` (one sequence) and returns the report as a dict.
    centroids [Hkv,B,d]: the partition to train for (default: the workload's own centroids);
    return_weights: the report also holds "weights" = (W1, b1, W2, b2) as classify_queries takes them;
    batch_norm: the hidden layer is normalised over the batch during training (scale 1 and shift 0 at the
    start, eps 1e-5, momentum 0.1) and the running statistics are folded into W1, b1 for the evaluation."""
    import types

    import torch

    import paper_2502_08246_amd as saap
    from synth import gen

    args = types.SimpleNamespace(train_queries=train_queries, eval_queries=eval_queries, steps=steps, batch=batch, lr=lr,
                                 seed=seed)
    if not torch.cuda.is_available():
        raise RuntimeError("train_query_model needs a GPU")
    saap.load_library()
    dev = "cuda:0"
    if cfg.S != 1:
        cfg = cfg.replace(S=1)
    G, Hw, B, d = cfg.Hq // cfg.Hkv, cfg.Hkv, cfg.B, cfg.d
    scale = 1.0 / math.sqrt(d)

    cache = gen.make_cache(cfg, args.seed, dev)
    cent = centroids if centroids is not None else gen.make_centroids(cfg, args.seed, dev, cache)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, 0)
    del cache, Vs
    T_all = args.train_queries + args.eval_queries
    xq, q = gen.make_queries(cfg, args.seed, dev, n_steps=T_all)

    # targets: the bucket attention mass of every query; the queries of a KV head form one batch
    # (rows ordered (step, head of the group)), scored on the matrix cores in pieces of 4096 rows
    q_rows = q[:, 0].reshape(T_all, Hw, G, d).permute(1, 0, 2, 3).reshape(1, Hw, T_all * G, d).contiguous()
    mass_rows = torch.empty(1, Hw, T_all * G, B, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for r0 in range(0, T_all * G, 4096):
        r1 = min(r0 + 4096, T_all * G)
        piece, _ = saap.bucket_attention_mass_batch(q_rows[:, :, r0:r1].contiguous(), Ks, off, ln, scale)
        mass_rows[:, :, r0:r1] = piece
    torch.cuda.synchronize()
    target_s = time.perf_counter() - t0
    # [T, Hq, B] view of the same numbers for the evaluation
    mass = mass_rows[0].reshape(Hw, T_all, G, B).permute(1, 0, 2, 3).reshape(T_all, cfg.Hq, B).contiguous()

    def per_weight_set(a, lo, hi):
        # [T,(S,)Hq,X] -> [Hw, (hi-lo)*G, X]: the rows of the G heads that share weight set h
        a = a[lo:hi].reshape(hi - lo, Hw, G, a.shape[-1])
        return a.permute(1, 0, 2, 3).reshape(Hw, (hi - lo) * G, a.shape[-1]).contiguous()

    n_tr = args.train_queries
    x_tr, t_tr = per_weight_set(xq[:, 0], 0, n_tr), per_weight_set(mass, 0, n_tr)
    rows = x_tr.shape[1]
    R = min(args.batch, rows)
    g = torch.Generator(device=dev).manual_seed(args.seed + 1)

    W1b, b1b, W2b, b2b = gen.make_classifier(cfg, args.seed, dev)          # the random-init model of the benchmark
    P = tuple(t.float().contiguous() for t in (W1b, b1b, W2b, b2b))
    M = tuple(torch.zeros_like(p) for p in P)
    V = tuple(torch.zeros_like(p) for p in P)
    grads = tuple(torch.empty_like(p) for p in P)
    loss = torch.empty(Hw, dtype=torch.float32, device=dev)
    if batch_norm:
        bn_gamma, bn_beta = torch.ones_like(P[1]), torch.zeros_like(P[1])
        run_mean, run_var = torch.zeros_like(P[1]), torch.ones_like(P[1])
        bn_grads = (torch.empty_like(bn_gamma), torch.empty_like(bn_beta))
        bn_M = tuple(torch.zeros_like(t) for t in bn_grads)
        bn_V = tuple(torch.zeros_like(t) for t in bn_grads)

    def evaluate(weights):
        """Mean captured attention mass on the held-out queries for lists made from `weights`
        (None: nearest-centroid routing), and for the best possible lists."""
        probs = torch.empty(1, cfg.Hq, B, dtype=torch.float32, device=dev)
        sel = torch.empty(1, Hw, cfg.nprobe, dtype=torch.int32, device=dev)
        got = best = 0.0
        for t in range(n_tr, T_all):
            if weights is None:
                saap.classify_queries(xq[t], None, None, cent, None, Hw, out=probs)
            else:
                saap.classify_queries(xq[t], *weights, Hw, out=probs)
            saap.select_buckets(probs, Hw, cfg.nprobe, out=sel)
            gm = mass[t].view(1, Hw, G, B)
            lists = sel.to(torch.int64).unsqueeze(2).expand(-1, -1, G, -1)
            got += float(torch.gather(gm, 3, lists).sum(-1).mean().item())
            top = torch.topk(gm.sum(2), cfg.nprobe, dim=-1).indices.unsqueeze(2).expand(-1, -1, G, -1)
            best += float(torch.gather(gm, 3, top).sum(-1).mean().item())
        n = T_all - n_tr
        return got / n, best / n

    def as_inference_weights(params):
        if batch_norm:
            W1f, b1f = saap.fold_batch_norm(params[0], params[1], bn_gamma, bn_beta, run_mean, run_var, out_dtype=xq.dtype)
            return (W1f, b1f, params[2].to(xq.dtype).contiguous(), params[3].contiguous())
        return tuple(p.to(xq.dtype).contiguous() if i in (0, 2) else p.contiguous() for i, p in enumerate(params))

    cap_init, cap_best = evaluate((W1b, b1b, W2b, b2b))
    cap_kmeans, _ = evaluate(None)

    losses = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for step in range(1, args.steps + 1):
        pick = torch.randint(0, rows, (R,), generator=g, device=dev)
        xb, tb = x_tr[:, pick].contiguous(), t_tr[:, pick].contiguous()
        if batch_norm:
            saap.query_model_bn_loss_grads(xb, tb, P, bn_gamma, bn_beta, run_mean, run_var, grads=grads,
                                           grad_gamma=bn_grads[0], grad_beta=bn_grads[1], loss=loss)
            for p, gr, m, v in zip((bn_gamma, bn_beta), bn_grads, bn_M, bn_V):
                saap.adam_update(p, gr, m, v, step, args.lr)
        else:
            saap.query_model_loss_grads(xb, tb, P, grads=grads, loss=loss)
        for p, gr, m, v in zip(P, grads, M, V):
            saap.adam_update(p, gr, m, v, step, args.lr)
        if step == 1 or step % max(args.steps // 8, 1) == 0 or step == args.steps:
            losses.append((step, round(float(loss.mean().item()), 4)))
    torch.cuda.synchronize()
    train_s = time.perf_counter() - t0
    cap_trained, _ = evaluate(as_inference_weights(P))

    report = {
        "workload": cfg.name, "B": B, "nprobe": cfg.nprobe, "classifier": f"{d}->{cfg.hidden}->{B}", "weight_sets": Hw,
        "batch_norm": bool(batch_norm),
        "train_queries_per_head": n_tr, "eval_queries_per_head": T_all - n_tr, "steps": args.steps, "batch_rows": R,
        "lr": args.lr, "loss": losses, "ms_per_step": round(train_s / max(args.steps, 1) * 1e3, 3),
        "targets_s": round(target_s, 2),
        "captured_attention_mass": {"random_init": round(cap_init, 4), "trained": round(cap_trained, 4),
                                    "kmeans_routing": round(cap_kmeans, 4), "best_possible": round(cap_best, 4)},
        "selectivity": round(cfg.nprobe / B, 4), "data": "synthetic",
    }
    if return_weights:
        report["weights"] = as_inference_weights(P)
    return report


def main():
    args = parse()
    from synth import gen

    try:
        report = train(gen.CONFIGS[args.workload], args.train_queries, args.eval_queries, args.steps, args.batch, args.lr,
                       args.seed, batch_norm=args.batch_norm)
    except RuntimeError as e:
        print(e, file=sys.stderr)
        sys.exit(2)
    print(json.dumps(report))


if __name__ == "__main__":
    main()
