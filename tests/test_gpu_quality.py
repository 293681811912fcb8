"""The MSE-against-selectivity harness (Appendix B "Experiments", Appendix E.4): its two numbers against the
oracle on the same lists, and the properties the curves must have at any size."""
import math

import numpy as np
import pytest
import torch

from oracle import ref
from synth import gen

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
SCALE = 1.0 / math.sqrt(128.0)


@pytest.fixture(scope="module")
def saap():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the -m gpu tests need a real device")
    import paper_2502_08246_amd as lib
    lib.load_library()
    ref.set_threads(16)
    return lib


def h(t):
    return gen.to_host_f32(t)


@pytest.mark.parametrize("nprobe", [1, 5, 16])
def test_evaluate_lists_against_the_oracle(saap, nprobe):
    from paper_2502_08246_amd.mse_vs_selectivity import evaluate_lists
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=2, Hq=8, Hkv=2, N=3000, B=16, nprobe=nprobe, hidden=64)
    cache = gen.make_cache(cfg, 83, DEV)
    cent = gen.make_centroids(cfg, 83, DEV, cache, n_train=2048)
    _, q = gen.make_queries(cfg, 83, DEV)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, 0)
    scores = torch.rand(cfg.S, cfg.Hq, cfg.B, generator=torch.Generator(device=DEV).manual_seed(1), device=DEV)
    sel = saap.select_buckets(scores, cfg.Hkv, nprobe)
    exact, _ = saap.dense_decode_attention(q[0], cache["K"], cache["V"], SCALE)
    mse, share = evaluate_lists(q[0], exact, Ks, Vs, off, ln, sel, SCALE, cfg.N)
    torch.cuda.synchronize()
    # the oracle's side from the inputs: ids, index, lists, both attentions in double precision
    hK, hV = h(cache["K"]), h(cache["V"])
    r_ids = ref.assign_keys(h(cache["x_keys"]), h(cent))
    r_off, r_ln, r_idx, _, _ = ref.build_bucket_index(r_ids, hK, hV, cfg.B, 0)
    r_sel = ref.select_buckets(scores.cpu().numpy(), cfg.Hkv, nprobe)
    assert np.array_equal(np.sort(sel.cpu().numpy(), -1), np.sort(r_sel, -1))
    r_sparse, _ = ref.sparse_decode_attention(h(q[0]), hK, hV, r_off, r_ln, r_idx, r_sel, SCALE)
    r_dense, _ = ref.dense_decode_attention(h(q[0]), hK, hV, SCALE)
    r_mse = float(((r_sparse - r_dense) ** 2).mean())
    # each output is within 2e-3 + 1e-2 |ref| of the oracle's; the error of their squared difference follows
    tol = 2 * math.sqrt(max(r_mse, 1e-12)) * 3e-3 + 1e-5
    assert abs(mse - r_mse) <= tol, (mse, r_mse)
    if nprobe == cfg.B:
        assert mse < 1e-9 and r_mse < 1e-20
    want_share = ref.selectivity(r_ln.reshape(-1, cfg.B), r_sel.reshape(-1, nprobe), cfg.N)
    assert abs(share - want_share) < 1e-12


def test_curves_have_the_properties_that_hold_at_any_size(saap):
    from paper_2502_08246_amd.mse_vs_selectivity import curves
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=1, Hq=8, Hkv=2, N=6000, B=32, nprobe=4, hidden=64)
    rep = curves(cfg, [16, 64], [0.05, 0.25, 1.0], n_queries=6, lloyd_iters=3, train_steps=12, seed=3)
    rows = rep["curves"]
    assert [(r["nlist"], r["nprobe"]) for r in rows] == [(16, 1), (16, 4), (16, 16), (64, 3), (64, 16), (64, 64)]
    routers = ("random", "kmeans", "query_model", "best_possible")
    for r in rows:
        for name in routers:
            assert 0.0 < r[name]["selectivity"] <= 1.0 and r[name]["mse"] >= 0.0
        if r["nprobe"] == r["nlist"]:                       # every key visited: only the summation order differs
            for name in routers:
                assert r[name]["selectivity"] == 1.0 and r[name]["relative_mse"] < 1e-9
    for B in (16, 64):
        sub = [r for r in rows if r["nlist"] == B]
        for name in routers:                                # nested lists: more buckets, more keys
            shares = [r[name]["selectivity"] for r in sub]
            assert shares == sorted(shares)
        # the buckets that hold the attention mass approximate better than a random subset
        assert sub[1]["best_possible"]["mse"] < sub[1]["random"]["mse"]
