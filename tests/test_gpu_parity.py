"""GPU parity tests: every C entry point, called through the binding on cuda:0, against the CPU
oracle on the same seeded inputs.  Integer results (bucket ids, CSR arrays, selected buckets) must
match bit for bit; attention outputs within the stated tolerance
    |gpu - ref| <= 2e-3 + 1e-2 |ref|   (bf16 inputs, fp32 accumulation)
    |gpu - ref| <= 1e-5 + 1e-5 |ref|   (fp32 inputs).
Sizes are chosen so that the oracle finishes in seconds while the kernels still see several
workgroups, several tiles and ragged tails."""
import math

import numpy as np
import pytest
import torch

from oracle import ref
from synth import gen

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL = {"bf16": (2e-3, 1e-2), "f32": (1e-5, 1e-5)}
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


def assert_close(got, want, dtype, what=""):
    atol, rtol = TOL[dtype]
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    fin = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), fin), f"{what}: finiteness differs"
    assert np.array_equal(got[~fin], want[~fin]), f"{what}: non-finite values differ"
    err = np.abs(got[fin] - want[fin])
    lim = atol + rtol * np.abs(want[fin])
    bad = err > lim
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"


def small(name, **kw):
    return gen.CONFIGS[name].replace(**kw)


def make_inputs(cfg, seed=0):
    cache = gen.make_cache(cfg, seed, DEV)
    cent = gen.make_centroids(cfg, seed, DEV, cache, n_train=min(8192, max(4 * cfg.B, 2048)))
    xq, q = gen.make_queries(cfg, seed, DEV)
    W = gen.make_classifier(cfg, seed, DEV)
    return cache, cent, xq, q, W


# ------------------------------------------------------------------------------ dense attention
@pytest.mark.parametrize("dtype,S,Hq,Hkv,N", [
    ("bf16", 1, 4, 1, 5000), ("bf16", 2, 8, 2, 3001), ("f32", 1, 1, 1, 4096), ("f32", 2, 4, 2, 1237),
    ("bf16", 1, 2, 1, 70), ("bf16", 1, 8, 1, 900), ("bf16", 1, 1, 1, 1),
])
def test_dense_attention(saap, dtype, S, Hq, Hkv, N):
    cfg = small("cfg1_llama8b_128k", S=S, Hq=Hq, Hkv=Hkv, N=N, B=16, dtype=dtype)
    cache = gen.make_cache(cfg, 3, DEV)
    _, q = gen.make_queries(cfg, 3, DEV)
    out, lse = saap.dense_decode_attention(q[0], cache["K"], cache["V"], SCALE)
    torch.cuda.synchronize()
    ro, rl = ref.dense_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), SCALE)
    assert_close(out.cpu().numpy(), ro, dtype, "dense out")
    assert_close(lse.cpu().numpy(), rl, dtype, "dense lse")


# ------------------------------------------------------------------------------ index build
@pytest.mark.parametrize("dtype,S,Hkv,N,B,slack", [
    ("bf16", 1, 2, 10000, 64, 0), ("bf16", 2, 2, 4097, 100, 3), ("f32", 1, 1, 4096, 64, 0), ("bf16", 1, 1, 300, 1024, 1),
])
def test_build_bucket_index(saap, dtype, S, Hkv, N, B, slack):
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    dt = gen.torch_dtype(dtype)
    # skewed ids with some empty buckets
    w = torch.rand(B, generator=g, device=DEV) ** 4
    w[::7] = 0
    w[0] = 1.0
    ids = torch.multinomial(w, S * Hkv * N, replacement=True, generator=g).to(torch.int32).view(S, Hkv, N)
    K = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(dt)
    V = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(dt)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, K, V, B, slack)
    torch.cuda.synchronize()
    ro, rl, ri, rK, rV = ref.build_bucket_index(ids.cpu().numpy(), h(K), h(V), B, slack)
    assert np.array_equal(off.cpu().numpy(), ro)
    assert np.array_equal(ln.cpu().numpy(), rl)
    assert np.array_equal(idx.cpu().numpy(), ri)          # stable order, slack slots -1
    member = ri >= 0
    assert np.array_equal(h(Ks)[member], rK[member])
    assert np.array_equal(h(Vs)[member], rV[member])


# ------------------------------------------------------------------------------ selection
@pytest.mark.parametrize("S,Hq,Hkv,B,nprobe,mode", [
    (1, 32, 8, 1024, 51, 0), (2, 8, 2, 4096, 410, 0), (1, 1, 1, 64, 8, 0), (1, 8, 2, 100, 100, 0),
    (2, 8, 2, 300, 17, 1), (1, 4, 1, 8192, 1, 0), (1, 4, 4, 48, 5, 0),
])
def test_select_buckets(saap, S, Hq, Hkv, B, nprobe, mode):
    g = torch.Generator(device=DEV)
    g.manual_seed(B + nprobe)
    scores = torch.softmax(3 * torch.randn(S, Hq, B, generator=g, device=DEV), dim=-1)
    scores[:, :, B // 2] = scores[:, :, 1]            # planted ties
    scores[:, :, B - 1] = scores[:, :, 0]
    # coarse values: many exact ties after the group sum
    scores[0, :, : B // 4] = torch.round(scores[0, :, : B // 4] * 64) / 64
    sel = saap.select_buckets(scores, Hkv, nprobe, mode)
    torch.cuda.synchronize()
    want = ref.select_buckets(scores.cpu().numpy(), Hkv, nprobe, mode)
    assert np.array_equal(sel.cpu().numpy(), want)


@pytest.mark.parametrize("B,nprobe", [(1024, 51), (4096, 410), (64, 8), (512, 64), (2048, 65)])
def test_select_buckets_with_ties_at_the_threshold(saap, B, nprobe):
    """Equal scores straddling the nprobe-th place: the lowest ids must be taken."""
    S, Hq, Hkv = 2, 8, 2
    scores = torch.full((S, Hq, B), 1.0 / B, device=DEV)                  # all equal
    scores[1, :, 10::3] = 2.0 / B                                          # sequence 1: two plateaus
    scores[1, 4:, 7] = 0.5                                                 # head group 1: one clear winner
    sel = saap.select_buckets(scores, Hkv, nprobe)
    torch.cuda.synchronize()
    want = ref.select_buckets(scores.cpu().numpy(), Hkv, nprobe)
    assert np.array_equal(sel.cpu().numpy(), want)
    assert sel[0, 0].tolist() == list(range(nprobe))


@pytest.mark.parametrize("S,Hq,Hkv,B,nprobe,mode", [
    (1, 32, 8, 1024, 51, 0), (1, 32, 8, 4096, 410, 0), (2, 8, 2, 2048, 102, 0), (1, 4, 1, 64, 8, 0), (2, 4, 4, 96, 5, 0),
    (1, 8, 1, 1000, 37, 0), (1, 8, 4, 1024, 51, 1), (1, 16, 8, 8192, 300, 0), (3, 2, 1, 16, 3, 0),
])
def test_select_buckets_from_logits(saap, S, Hq, Hkv, B, nprobe, mode):
    """The fused softmax + selection: its probabilities against the definition in float64, its selection
    bit for bit against the oracle's selection made on those same fp32 probabilities."""
    g = torch.Generator(device=DEV)
    g.manual_seed(3 * B + nprobe)
    logits = 4 * torch.randn(S, Hq, B, generator=g, device=DEV)
    logits[:, :, B // 2] = logits[:, :, 1]            # planted ties
    logits[0, :, : B // 4] = torch.round(logits[0, :, : B // 4] * 2) / 2
    probs = torch.empty_like(logits)
    sel = saap.select_buckets_from_logits(logits, Hkv, nprobe, mode, probs=probs)
    sel_only = saap.select_buckets_from_logits(logits, Hkv, nprobe, mode)
    torch.cuda.synchronize()
    z = logits.cpu().numpy().astype(np.float64)
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    np.testing.assert_allclose(probs.cpu().numpy(), e / e.sum(axis=-1, keepdims=True), rtol=1e-5, atol=1e-12)
    want = ref.select_buckets(probs.cpu().numpy(), Hkv, nprobe, mode)
    assert np.array_equal(sel.cpu().numpy(), want)
    assert torch.equal(sel, sel_only)                  # the optional output changes nothing
    # and the two-call route (softmax kernel of classify_queries, then select_buckets) agrees wherever
    # the group sums are not within rounding of each other at the threshold
    two = saap.select_buckets(torch.softmax(logits, dim=-1), Hkv, nprobe, mode)
    torch.cuda.synchronize()
    a, b = sel.cpu().numpy(), two.cpu().numpy()
    differ = sum(len(set(x.tolist()) ^ set(y.tolist())) for x, y in zip(a.reshape(-1, nprobe), b.reshape(-1, nprobe)))
    assert differ <= 2 * a.shape[0] * a.shape[1], differ      # at most one swap at the threshold per list


# ------------------------------------------------------------------------------ sparse attention
def _oracle_index(cfg, cache, cent, slack):
    ids = ref.assign_keys(h(cache["x_keys"]), h(cent))
    return ids, ref.build_bucket_index(ids, h(cache["K"]), h(cache["V"]), cfg.B, slack)


@pytest.mark.parametrize("dtype,S,Hq,Hkv,N,B,nprobe,slack,alpha", [
    ("bf16", 1, 4, 1, 6000, 64, 8, 0, None),
    ("bf16", 2, 8, 2, 5003, 128, 13, 2, 0.3),
    ("f32", 1, 1, 1, 4096, 64, 8, 0, None),
    ("f32", 1, 4, 2, 2500, 32, 5, 1, 0.3),
    ("bf16", 1, 8, 1, 3000, 32, 32, 0, None),       # G = 8, all buckets
    ("bf16", 1, 2, 1, 3000, 32, 1, 0, 0.3),         # G = 2, one bucket
])
def test_sparse_attention(saap, dtype, S, Hq, Hkv, N, B, nprobe, slack, alpha):
    cfg = small("cfg1_llama8b_128k", S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=nprobe, dtype=dtype, alpha=alpha, hidden=64)
    cache, cent, xq, q, W = make_inputs(cfg, 7)
    ids, (off, ln, idx, rK, rV) = _oracle_index(cfg, cache, cent, slack)
    scores = ref.classify_queries(h(xq[0]), h(W[0]), None, h(W[2]), None, Hkv)
    sel = ref.select_buckets(scores, Hkv, nprobe)
    # GPU side: its own index build from the oracle's ids, then attention with the oracle's selection
    d_ids = torch.from_numpy(ids).to(DEV)
    g_off, g_ln, g_idx, Ks, Vs = saap.build_bucket_index(d_ids, cache["K"], cache["V"], B, slack)
    d_sel = torch.from_numpy(sel).to(DEV)
    out, lse = saap.sparse_decode_attention(q[0], Ks, Vs, g_off, g_ln, d_sel, SCALE)
    torch.cuda.synchronize()
    ro, rl = ref.sparse_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), off, ln, idx, sel, SCALE)
    assert_close(out.cpu().numpy(), ro, dtype, "sparse out")
    assert_close(lse.cpu().numpy(), rl, dtype, "sparse lse")
    # bf16 output option
    out16, _ = saap.sparse_decode_attention(q[0], Ks, Vs, g_off, g_ln, d_sel, SCALE, out_dtype=torch.bfloat16)
    assert_close(out16.float().cpu().numpy(), ro, "bf16", "sparse out (bf16 store)")


def test_sparse_all_buckets_equals_dense_and_empty_selection(saap):
    cfg = small("cfg1_llama8b_128k", S=1, Hq=8, Hkv=2, N=7001, B=96, nprobe=96, hidden=64)
    cache, cent, xq, q, W = make_inputs(cfg, 11)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, 2)
    g = torch.Generator(device="cpu")
    g.manual_seed(1)
    sel = torch.stack([torch.randperm(cfg.B, generator=g) for _ in range(2)]).view(1, 2, cfg.B).to(torch.int32).to(DEV)
    o_sparse, l_sparse = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, sel, SCALE)
    o_dense, l_dense = saap.dense_decode_attention(q[0], cache["K"], cache["V"], SCALE)
    o_gaps, l_gaps = saap.dense_decode_attention(q[0], Ks, Vs, SCALE, off=off, ln=ln)
    torch.cuda.synchronize()
    ro, rl = ref.dense_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), SCALE)
    for o, l, what in ((o_sparse, l_sparse, "nprobe=B"), (o_dense, l_dense, "dense"), (o_gaps, l_gaps, "dense over sorted")):
        assert_close(o.cpu().numpy(), ro, "bf16", what)
        assert_close(l.cpu().numpy(), rl, "bf16", what + " lse")
    # nothing selected: zeros and -inf
    empty = torch.empty(1, 2, 0, dtype=torch.int32, device=DEV)
    o, l = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, empty, SCALE)
    # only empty buckets selected
    ln2 = ln.clone()
    ln2[:, :, 5] = 0
    o2, l2 = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln2, torch.full((1, 2, 1), 5, dtype=torch.int32, device=DEV), SCALE)
    torch.cuda.synchronize()
    for oo, ll in ((o, l), (o2, l2)):
        assert (oo == 0).all() and torch.isneginf(ll).all()


def test_sparse_independent_mode(saap):
    cfg = small("cfg1_llama8b_128k", S=2, Hq=8, Hkv=2, N=4000, B=64, nprobe=6, hidden=64)
    cache, cent, xq, q, W = make_inputs(cfg, 13)
    ids, (off, ln, idx, rK, rV) = _oracle_index(cfg, cache, cent, 0)
    scores = ref.classify_queries(h(xq[0]), h(W[0]), None, h(W[2]), None, cfg.Hkv)
    sel = ref.select_buckets(scores, cfg.Hkv, cfg.nprobe, mode=1)
    g_off, g_ln, g_idx, Ks, Vs = saap.build_bucket_index(torch.from_numpy(ids).to(DEV), cache["K"], cache["V"], cfg.B, 0)
    out, lse = saap.sparse_decode_attention(q[0], Ks, Vs, g_off, g_ln, torch.from_numpy(sel).to(DEV), SCALE,
                                            mode=saap.INDEPENDENT)
    torch.cuda.synchronize()
    ro, rl = ref.sparse_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), off, ln, idx, sel, SCALE, mode=1)
    assert_close(out.cpu().numpy(), ro, "bf16", "independent out")
    assert_close(lse.cpu().numpy(), rl, "bf16", "independent lse")


@pytest.mark.parametrize("dtype,S,Hq,Hkv,N,B,nprobe,kind", [
    ("bf16", 1, 32, 8, 30000, 256, 13, "random"), ("bf16", 2, 4, 2, 5000, 64, 6, "same"), ("f32", 1, 8, 1, 3000, 48, 5, "disjoint"),
    ("bf16", 1, 8, 2, 6000, 128, 128, "all"), ("bf16", 1, 4, 1, 2500, 48, 0, "random"), ("bf16", 3, 4, 2, 700, 8192, 20, "random"),
])
def test_independent_lists_share_one_pass_over_the_union(saap, dtype, S, Hq, Hkv, N, B, nprobe, kind):
    """Independent routing with several heads per KV head: lists that overlap, coincide, are disjoint or hold
    every bucket; each head must see exactly the keys of its own list (oracle: per-head restricted softmax)."""
    cfg = small("cfg1_llama8b_128k", S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=max(nprobe, 1), dtype=dtype, hidden=64)
    cache = gen.make_cache(cfg, 71, DEV)
    cent = gen.make_centroids(cfg, 71, DEV, cache, n_train=max(2048, B))
    _, q = gen.make_queries(cfg, 71, DEV)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, 0)
    rng = np.random.default_rng(B + nprobe)
    G = Hq // Hkv
    sel = np.zeros((S, Hq, nprobe), dtype=np.int32)
    for s in range(S):
        for hq in range(Hq):
            if kind == "random":
                sel[s, hq] = rng.permutation(B)[:nprobe]
            elif kind == "same":
                sel[s, hq] = (np.arange(nprobe) * 7 + 3 * (hq // G)) % B
            elif kind == "disjoint":
                sel[s, hq] = (hq % G) * nprobe + np.arange(nprobe)
            else:
                sel[s, hq] = rng.permutation(B)
    out, lse = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, torch.from_numpy(sel).to(DEV), SCALE, mode=saap.INDEPENDENT)
    torch.cuda.synchronize()
    ro, rl = ref.sparse_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), off.cpu().numpy(), ln.cpu().numpy(),
                                         idx.cpu().numpy(), sel, SCALE, mode=1)
    assert_close(out.cpu().numpy(), ro, dtype, "independent out")
    assert_close(lse.cpu().numpy(), rl, dtype, "independent lse")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_with_extreme_scores(saap, dtype):
    """Softmax far from the benign range: scores in the thousands with one dominant key (the output is that
    key's value), a running maximum that keeps rising along the cache, identical keys (the output is the
    mean of the values), and huge negative scores; sparse and dense kernels against the oracle."""
    S, Hq, Hkv, N, B = 1, 4, 1, 3000, 12
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator(device="cpu").manual_seed(17)
    K = torch.randn(S, Hkv, N, 128, generator=g)
    V = torch.randn(S, Hkv, N, 128, generator=g)
    q = torch.randn(S, Hq, 128, generator=g)
    qn = q / q.norm(dim=-1, keepdim=True)
    # head 0: keys grow along the cache in the direction of the query (every batch raises the maximum)
    K[0, 0] += torch.linspace(0, 60, N).unsqueeze(1) * qn[0, 0]
    # head 1: one key dominates by a wide margin
    K[0, 0, 1234] = 400.0 * qn[0, 1]
    # head 2's query is opposite to most keys' drift (huge negative scores), head 3's is zero (uniform weights)
    q[0, 2] = -30.0 * qn[0, 0]
    q[0, 3] = 0.0
    q[0, 0] = 25.0 * qn[0, 0]
    q[0, 1] = 30.0 * qn[0, 1]
    K, V, q = (t.to(dt).to(DEV).contiguous() for t in (K, V, q))
    ids = (torch.arange(N, dtype=torch.int32) % B).reshape(1, 1, N).to(DEV).contiguous()
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, K, V, B, 1)
    sel = torch.arange(B, dtype=torch.int32, device=DEV).reshape(1, 1, B)
    scale = 1.0                                             # no 1/sqrt(d): keeps the scores large
    out, lse = saap.sparse_decode_attention(q, Ks, Vs, off, ln, sel, scale)
    o_d, l_d = saap.dense_decode_attention(q, K, V, scale)
    torch.cuda.synchronize()
    ro, rl = ref.dense_decode_attention(h(q), h(K), h(V), np.float32(scale))
    assert np.abs(rl).max() > 1000                          # the case is what it claims to be
    # fp32: a score s is known to about |s| * 2^-23 * sqrt(d) in single precision, here about 2e-3 for
    # |s| ~ 1.5e3; the weights exp(s - max) inherit that as a relative error, so the fp32 tolerance of
    # benign scores (1e-5) does not apply: 2e-4 absolute + relative is what this case can hold
    def check(got, want, what):
        if dtype == "bf16":
            return assert_close(got, want, dtype, what)
        err = np.abs(np.asarray(got, np.float64) - want)
        assert (err <= 2e-4 + 2e-4 * np.abs(want)).all(), f"{what}: max err {err.max():.3e}"

    for got_o, got_l, what in ((out, lse, "sparse"), (o_d, l_d, "dense")):
        check(got_o.cpu().numpy(), ro, f"{what} out")
        check(got_l.cpu().numpy(), rl, f"{what} lse")
    np.testing.assert_allclose(out[0, 1].cpu().numpy(), h(V)[0, 0, 1234], rtol=1e-2, atol=2e-3)     # the dominant key
    np.testing.assert_allclose(out[0, 3].cpu().numpy(), h(V)[0, 0].mean(0), rtol=1e-2, atol=2e-3)  # uniform weights


def test_attention_is_deterministic_and_workspace_stays_clean(saap):
    cfg = small("cfg1_llama8b_128k", S=1, Hq=8, Hkv=2, N=20000, B=128, nprobe=16, hidden=64)
    cache, cent, xq, q, W = make_inputs(cfg, 17)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, 0)
    scores = saap.classify_queries(xq[0], W[0], W[1], W[2], W[3], cfg.Hkv)
    sel = saap.select_buckets(scores, cfg.Hkv, cfg.nprobe)
    outs = []
    for _ in range(5):
        o, l = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, sel, SCALE)
        outs.append((o.clone(), l.clone()))
    torch.cuda.synchronize()
    for o, l in outs[1:]:
        assert torch.equal(o, outs[0][0]) and torch.equal(l, outs[0][1])
    ws = saap.workspace(0, DEV)
    assert int(ws[:65536].to(torch.int64).sum().item()) == 0     # arrival counters are back to zero


def test_limits_max_buckets_and_group_of_eight(saap):
    """The largest supported bucket count (8192) with every bucket visited, one bucket per few keys,
    many empty buckets, G = 8 and G = 1, and more units than compute units."""
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    for (S, Hq, Hkv, N, B, nprobe) in [(1, 8, 1, 20000, 8192, 8192), (1, 2, 2, 9000, 8192, 5000), (40, 8, 8, 600, 16, 3)]:
        dt = torch.bfloat16
        K = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(dt)
        V = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(dt)
        q = torch.randn(S, Hq, 128, generator=g, device=DEV).to(dt)
        ids = torch.randint(0, B, (S, Hkv, N), generator=g, device=DEV, dtype=torch.int32)
        ids[ids % 3 == 1] = 0                                   # a third of the buckets stay empty, bucket 0 is huge
        off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, K, V, B, 0)
        scores = torch.rand(S, Hq, B, generator=g, device=DEV)
        sel = saap.select_buckets(scores, Hkv, nprobe)
        out, lse = saap.sparse_decode_attention(q, Ks, Vs, off, ln, sel, SCALE)
        torch.cuda.synchronize()
        r_off, r_ln, r_idx, _, _ = ref.build_bucket_index(ids.cpu().numpy(), h(K), h(V), B, 0)
        assert np.array_equal(off.cpu().numpy(), r_off) and np.array_equal(idx.cpu().numpy(), r_idx)
        r_sel = ref.select_buckets(scores.cpu().numpy(), Hkv, nprobe)
        assert np.array_equal(sel.cpu().numpy(), r_sel)
        ro, rl = ref.sparse_decode_attention(h(q), h(K), h(V), r_off, r_ln, r_idx, r_sel, SCALE)
        assert_close(out.cpu().numpy(), ro, "bf16", f"limits {S},{Hq},{Hkv},{B},{nprobe}")
        assert_close(lse.cpu().numpy(), rl, "bf16", "limits lse")


# ------------------------------------------------------------------------------ classifier
@pytest.mark.parametrize("dtype,S,Hq,Hkv,hidden,B,Hw_kind,bias", [
    ("bf16", 1, 32, 8, 512, 1024, "kv", False), ("bf16", 8, 8, 2, 256, 160, "kv", True),
    ("f32", 1, 1, 1, 256, 64, "kv", False), ("f32", 3, 4, 2, 64, 48, "q", True), ("bf16", 2, 8, 2, 96, 64, "one", True),
    ("bf16", 5, 4, 1, 64, 4096, "q", False),
    ("bf16", 1, 32, 8, 1024, 1024, "kv", True),      # the paper's model size (Section 6.1: hidden layer of 1024)
    ("bf16", 2, 8, 2, 1536, 208, "kv", False),       # the largest hidden layer the kernels take
    ("bf16", 1, 32, 8, 512, 4096, "kv", True),       # many buckets, few rows: 128 buckets per workgroup
    ("bf16", 2, 16, 8, 256, 4000, "kv", False),      # the same with a ragged last slab
])
def test_classify_queries(saap, dtype, S, Hq, Hkv, hidden, B, Hw_kind, bias):
    cfg = small("cfg1_llama8b_128k", S=S, Hq=Hq, Hkv=Hkv, N=16, B=B, hidden=hidden, dtype=dtype)
    Hw = {"one": 1, "kv": Hkv, "q": Hq}[Hw_kind]
    xq, _ = gen.make_queries(cfg, 19, DEV)
    W1, b1, W2, b2 = gen.make_classifier(cfg, 19, DEV, Hw=Hw)
    if bias:
        g = torch.Generator(device=DEV)
        g.manual_seed(2)
        b1 = torch.randn(b1.shape, generator=g, device=DEV)
        b2 = torch.randn(b2.shape, generator=g, device=DEV)
    else:
        b1 = b2 = None
    p = saap.classify_queries(xq[0], W1, b1, W2, b2, Hkv)
    z = saap.classify_queries(xq[0], W1, b1, W2, b2, Hkv, output_kind=saap.LOGITS)
    torch.cuda.synchronize()
    hb = lambda t: None if t is None else h(t)
    rp = ref.classify_queries(h(xq[0]), h(W1), hb(b1), h(W2), hb(b2), Hkv)
    rz = ref.classify_queries(h(xq[0]), h(W1), hb(b1), h(W2), hb(b2), Hkv, output_kind=1)
    # fp32 accumulation of exact products over d and hidden terms: logits to ~1e-5 absolute,
    # probabilities to the same relative amount
    np.testing.assert_allclose(z.cpu().numpy(), rz, rtol=2e-5, atol=5e-5)
    np.testing.assert_allclose(p.cpu().numpy(), rp, rtol=1e-4, atol=1e-9)


@pytest.mark.parametrize("dtype,S,Hq,Hkv,B,Hw_kind,bias", [
    ("bf16", 1, 32, 8, 1024, "kv", False), ("bf16", 3, 8, 2, 176, "kv", True), ("f32", 2, 4, 2, 64, "q", True),
    ("bf16", 2, 4, 1, 4096, "one", False),
])
def test_classify_queries_one_layer(saap, dtype, S, Hq, Hkv, B, Hw_kind, bias):
    """hidden = 0: z = W2 x + b2, the centroid routing of the paper's K-means baseline when W2 holds centroids."""
    cfg = small("cfg1_llama8b_128k", S=S, Hq=Hq, Hkv=Hkv, N=16, B=B, hidden=32, dtype=dtype)
    Hw = {"one": 1, "kv": Hkv, "q": Hq}[Hw_kind]
    xq, _ = gen.make_queries(cfg, 23, DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(4)
    W = (torch.randn(Hw, B, cfg.d, generator=g, device=DEV) / math.sqrt(cfg.d)).to(xq.dtype)
    b2 = torch.randn(Hw, B, generator=g, device=DEV) if bias else None
    z = saap.classify_queries(xq[0], None, None, W, b2, Hkv, output_kind=saap.LOGITS)
    p = saap.classify_queries(xq[0], None, None, W, b2, Hkv)
    torch.cuda.synchronize()
    hb = None if b2 is None else h(b2)
    rz = ref.classify_queries(h(xq[0]), None, None, h(W), hb, Hkv, output_kind=1)
    rp = ref.classify_queries(h(xq[0]), None, None, h(W), hb, Hkv)
    np.testing.assert_allclose(z.cpu().numpy(), rz, rtol=2e-5, atol=5e-5)
    np.testing.assert_allclose(p.cpu().numpy(), rp, rtol=1e-4, atol=1e-9)


# ------------------------------------------------------------------------------ assignment
def _plant_ties(x, cent):
    """Duplicate centroids (exact ties) and keys placed exactly between two centroids (near ties)."""
    cent = cent.clone()
    cent[:, 5] = cent[:, 2]
    cent[:, -1] = cent[:, 2]
    x = x.clone()
    x[:, :, :64] = (3.0 * cent[:, 2]).unsqueeze(0).unsqueeze(2).to(x.dtype)
    mid = (cent[:, 7].float() + cent[:, 9].float()).to(x.dtype)
    x[:, :, 64:128] = mid.unsqueeze(0).unsqueeze(2)
    return x, cent


@pytest.mark.parametrize("dtype,S,Hkv,N,B,bias", [
    ("bf16", 1, 2, 4000, 64, False), ("bf16", 2, 2, 1031, 1024, False), ("bf16", 1, 1, 5000, 100, True),
    ("f32", 1, 1, 4096, 64, False), ("f32", 1, 2, 500, 37, True), ("bf16", 1, 1, 700, 4096, False),
    ("bf16", 1, 2, 300, 4100, True),            # more buckets than the re-scoring pass keeps scores for
])
def test_assign_keys(saap, dtype, S, Hkv, N, B, bias):
    cfg = small("cfg1_llama8b_128k", S=S, Hq=Hkv, Hkv=Hkv, N=N, B=B, dtype=dtype)
    cache = gen.make_cache(cfg, 23, DEV)
    cent = gen.make_centroids(cfg, 23, DEV, n_train=max(2 * B, 2048))
    x, cent = _plant_ties(cache["x_keys"], cent)
    b = None
    if bias:
        b = (-0.5 * cent.float().pow(2).sum(-1)).contiguous()
    ids = saap.assign_keys(x, cent, b)
    torch.cuda.synchronize()
    want = ref.assign_keys(h(x), h(cent), None if b is None else h(b))
    got = ids.cpu().numpy()
    assert np.array_equal(got, want), f"{(got != want).sum()} of {got.size} ids differ"
    assert (got[:, :, :64] == 2).all()                      # the lowest of the tied duplicates


def test_assign_keys_degenerate_rows(saap):
    """Zero keys score the same against every centroid (all of them are candidates of the re-scoring
    pass), and keys equal to a centroid shared by two ids: the lowest id wins in both cases."""
    cfg = small("cfg1_llama8b_128k", S=1, Hq=2, Hkv=2, N=600, B=200, dtype="bf16")
    cache = gen.make_cache(cfg, 61, DEV)
    cent = gen.make_centroids(cfg, 61, DEV, n_train=2048)
    x = cache["x_keys"].clone()
    x[:, :, 100:300] = 0
    cent[:, 150] = cent[:, 17]
    x[:, :, 300:320] = cent[:, 17].unsqueeze(0).unsqueeze(2)
    ids = saap.assign_keys(x, cent)
    torch.cuda.synchronize()
    want = ref.assign_keys(h(x), h(cent), None)
    got = ids.cpu().numpy()
    assert np.array_equal(got, want)
    assert (got[:, :, 100:300] == 0).all()


@pytest.mark.parametrize("S,Hkv,N,B,bias", [(1, 2, 6000, 1024, False), (2, 1, 3000, 1536, True), (1, 1, 4000, 96, False)])
def test_assign_keys_every_key_between_two_centroids(saap, S, Hkv, N, B, bias):
    """Every key is the sum of two centroids, so its best two scores are close and all keys go through the
    re-scoring pass: several groups of 32 keys per workgroup, more tiles per wave than it keeps scores for
    (B = 1536), fewer tiles than waves (B = 96)."""
    g = torch.Generator(device="cpu").manual_seed(97)
    cent = torch.randn(Hkv, B, 128, generator=g).to(torch.bfloat16).to(DEV)
    i0 = torch.randint(0, B, (S, Hkv, N), generator=g).to(DEV)
    i1 = torch.randint(0, B, (S, Hkv, N), generator=g).to(DEV)
    c = cent.float()
    x = torch.stack([torch.stack([c[hh][i0[s, hh]] + c[hh][i1[s, hh]] for hh in range(Hkv)]) for s in range(S)])
    x = x.to(torch.bfloat16).contiguous()
    b = (-0.5 * c.pow(2).sum(-1)).contiguous() if bias else None
    ids = saap.assign_keys(x, cent, b)
    torch.cuda.synchronize()
    want = ref.assign_keys(h(x), h(cent), None if b is None else h(b))
    got = ids.cpu().numpy()
    assert np.array_equal(got, want), f"{(got != want).sum()} of {got.size} ids differ"


# ------------------------------------------------------------------------------ append
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_append_keys(saap, dtype):
    cfg = small("cfg1_llama8b_128k", S=2, Hq=8, Hkv=2, N=2000, B=32, nprobe=32, dtype=dtype, hidden=64)
    cache, cent, xq, q, W = make_inputs(cfg, 29)
    slack, steps = 2, 6
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, slack)
    torch.cuda.synchronize()
    r_off, r_ln, r_idx, rKs, rVs = ref.build_bucket_index(ids.cpu().numpy(), h(cache["K"]), h(cache["V"]), cfg.B, slack)
    new = gen.make_cache(cfg.replace(N=steps), 31, DEV)
    # make every step hit the same bucket for sequence 0 / head 0 so that its slack runs out
    new["x_keys"][0, 0, :] = (4.0 * cent[0, 3].float()).to(new["x_keys"].dtype)
    Kall = torch.cat([cache["K"], new["K"]], dim=2)
    Vall = torch.cat([cache["V"], new["V"]], dim=2)
    flags = []
    for t in range(steps):
        pos = torch.full((cfg.S,), cfg.N + t, dtype=torch.int32, device=DEV)
        xn, kn, vn = (new[k][:, :, t].contiguous() for k in ("x_keys", "K", "V"))
        nid, flag = saap.append_keys(xn, kn, vn, pos, cent, None, off, ln, idx, Ks, Vs)
        torch.cuda.synchronize()
        rid, rflag = ref.append_keys(h(xn), h(kn), h(vn), pos.cpu().numpy(), h(cent), None, r_off, r_ln, r_idx, rKs, rVs)
        assert np.array_equal(nid.cpu().numpy(), rid)
        flags.append(rflag)
        assert (flag[0].item() != 0) == (rflag != 0)        # a fresh flag per call
        assert np.array_equal(ln.cpu().numpy(), r_ln)
        assert np.array_equal(idx.cpu().numpy(), r_idx)
    assert flags[-1] == 1 and flags[0] == 0                 # overflow happened, and only after the slack ran out
    member = r_idx != -1
    assert np.array_equal(h(Ks)[member], rKs[member])
    # attention over the grown cache, all buckets
    sel = torch.arange(cfg.B, dtype=torch.int32, device=DEV).repeat(cfg.S, cfg.Hkv, 1)
    out, lse = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, sel, SCALE)
    torch.cuda.synchronize()
    ro, rl = ref.sparse_decode_attention(h(q[0]), h(Kall), h(Vall), r_off, r_ln, r_idx, sel.cpu().numpy(), SCALE)
    assert_close(out.cpu().numpy(), ro, dtype, "attention after append")
    assert_close(lse.cpu().numpy(), rl, dtype, "lse after append")


# ------------------------------------------------------------------------------ whole path, config 0
def test_config0_end_to_end(saap):
    """BASELINE config 0: fp32, one head, N=4096, B=64, classifier 128->256->64, 16 queries, nprobe 8 and 64."""
    cfg = gen.CONFIGS["cfg0_tiny_f32"]
    cache, cent, xq, q, (W1, b1, W2, b2) = make_inputs(cfg, 0)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, 0)
    torch.cuda.synchronize()
    r_ids = ref.assign_keys(h(cache["x_keys"]), h(cent))
    assert np.array_equal(ids.cpu().numpy(), r_ids)
    r_off, r_ln, r_idx, _, _ = ref.build_bucket_index(r_ids, h(cache["K"]), h(cache["V"]), cfg.B, 0)
    assert np.array_equal(off.cpu().numpy(), r_off) and np.array_equal(ln.cpu().numpy(), r_ln)
    assert np.array_equal(idx.cpu().numpy(), r_idx)
    hK, hV = h(cache["K"]), h(cache["V"])
    for t in range(cfg.n_queries):
        scores = saap.classify_queries(xq[t], W1, b1, W2, b2, cfg.Hkv)
        sel = saap.select_buckets(scores, cfg.Hkv, cfg.nprobe)
        out, lse = saap.sparse_decode_attention(q[t], Ks, Vs, off, ln, sel, SCALE)
        sel_all = saap.select_buckets(scores, cfg.Hkv, cfg.B)
        out_all, lse_all = saap.sparse_decode_attention(q[t], Ks, Vs, off, ln, sel_all, SCALE)
        out_d, lse_d = saap.dense_decode_attention(q[t], cache["K"], cache["V"], SCALE)
        torch.cuda.synchronize()
        r_scores = ref.classify_queries(h(xq[t]), h(W1), h(b1), h(W2), h(b2), cfg.Hkv)
        np.testing.assert_allclose(scores.cpu().numpy(), r_scores, rtol=1e-4, atol=1e-9)
        # selection is bit-exact on the same score buffer (here: the GPU's)
        r_sel = ref.select_buckets(scores.cpu().numpy(), cfg.Hkv, cfg.nprobe)
        assert np.array_equal(sel.cpu().numpy(), r_sel)
        ro, rl = ref.sparse_decode_attention(h(q[t]), hK, hV, r_off, r_ln, r_idx, r_sel, SCALE)
        assert_close(out.cpu().numpy(), ro, "f32", f"cfg0 query {t}")
        assert_close(lse.cpu().numpy(), rl, "f32", f"cfg0 lse {t}")
        rd, rdl = ref.dense_decode_attention(h(q[t]), hK, hV, SCALE)
        assert_close(out_all.cpu().numpy(), rd, "f32", "cfg0 nprobe=64 vs dense")
        assert_close(out_d.cpu().numpy(), rd, "f32", "cfg0 dense")
        assert_close(lse_all.cpu().numpy(), rdl, "f32", "cfg0 nprobe=64 lse")


# ------------------------------------------------------------------------------ the second launch shape
@pytest.mark.parametrize("dtype,S,Hq,Hkv,N,B", [
    ("bf16", 8, 32, 8, 3001, 16),      # 64 units, G = 4
    ("f32", 16, 16, 4, 1999, 8),       # 64 units, G = 4, wide rows
    ("bf16", 8, 64, 8, 2500, 16),      # G = 8
    ("bf16", 1, 64, 64, 1100, 8),      # G = 1
])
def test_many_units_take_the_two_workgroups_per_compute_unit_shape(saap, dtype, S, Hq, Hkv, N, B):
    """Many (sequence, head) units with enough keys: for dense attention (16-bit and 8-bit) the launch plan
    takes 256-thread workgroups, two per compute unit.  Dense attention, sparse attention over every bucket
    (= dense) and over half of them, and the 8-bit cache, each against the oracle; ragged N, so the last
    chunk of a unit is partial."""
    cfg = small("cfg1_llama8b_128k", S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=B, dtype=dtype, hidden=64)
    cache, cent, xq, q, W = make_inputs(cfg, 97)
    hK, hV = h(cache["K"]), h(cache["V"])
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, 0)
    out_d, lse_d = saap.dense_decode_attention(q[0], cache["K"], cache["V"], SCALE)
    all_b = torch.arange(B, dtype=torch.int32, device=DEV).repeat(S, Hkv, 1)
    out_a, lse_a = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, all_b, SCALE)
    half = torch.stack([torch.randperm(B, device=DEV)[:B // 2] for _ in range(S * Hkv)]).reshape(S, Hkv, B // 2).to(torch.int32)
    out_h, lse_h = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, half, SCALE)
    torch.cuda.synchronize()
    do, dl = ref.dense_decode_attention(h(q[0]), hK, hV, SCALE)
    assert_close(out_d.cpu().numpy(), do, dtype, "dense out")
    assert_close(lse_d.cpu().numpy(), dl, dtype, "dense lse")
    assert_close(out_a.cpu().numpy(), do, dtype, "all buckets out")
    assert_close(lse_a.cpu().numpy(), dl, dtype, "all buckets lse")
    r_ids = ids.cpu().numpy()
    r_off, r_ln, r_idx, _, _ = ref.build_bucket_index(r_ids, hK, hV, B, 0)
    ro, rl = ref.sparse_decode_attention(h(q[0]), hK, hV, r_off, r_ln, r_idx, half.cpu().numpy(), SCALE)
    assert_close(out_h.cpu().numpy(), ro, dtype, "half of the buckets out")
    assert_close(lse_h.cpu().numpy(), rl, dtype, "half of the buckets lse")
    if dtype == "bf16":
        K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
        out8, lse8 = saap.dense_decode_attention_fp8(q[0], K8, V8, ks, vs, SCALE, off=off, ln=ln)
        torch.cuda.synchronize()
        Kd = ref.dequantize_fp8(K8.cpu().numpy(), ks.cpu().numpy())
        Vd = ref.dequantize_fp8(V8.cpu().numpy(), vs.cpu().numpy())
        all_np = all_b.cpu().numpy()
        sorted_pos = np.arange(Kd.shape[2], dtype=np.int32)
        # the decoded sorted cache attended through an identity index: every bucket, in its stored order
        ident = np.broadcast_to(sorted_pos, r_idx.shape).copy()
        ro8, rl8 = ref.sparse_decode_attention(h(q[0]), Kd, Vd, r_off, r_ln, ident, all_np, SCALE)
        assert_close(out8.cpu().numpy(), ro8, dtype, "8-bit dense out")
        assert_close(lse8.cpu().numpy(), rl8, dtype, "8-bit dense lse")


@pytest.mark.parametrize("hidden,B", [(64, 100), (48, 64), (0, 100), (1600, 64)])
def test_classifier_shapes_outside_its_limits_are_refused_on_the_device_too(saap, hidden, B):
    """hidden must be a multiple of 32 (at most 1536) and B a multiple of 16: anything else returns
    SAAP_UNSUPPORTED before a kernel is enqueued, so the output buffer keeps what it held."""
    S, Hq, Hkv = 2, 8, 2
    g = torch.Generator(device=DEV).manual_seed(3)
    xq = torch.randn(S, Hq, 128, generator=g, device=DEV).to(torch.bfloat16)
    W1 = None if hidden == 0 else torch.randn(Hkv, hidden, 128, generator=g, device=DEV).to(torch.bfloat16)
    W2 = torch.randn(Hkv, B, hidden if hidden else 128, generator=g, device=DEV).to(torch.bfloat16)
    out = torch.full((S, Hq, B), -7.0, dtype=torch.float32, device=DEV)
    with pytest.raises(saap.SaapError) as e:
        saap.classify_queries(xq, W1, None, W2, None, Hkv, out=out)
    torch.cuda.synchronize()
    assert e.value.status == -2
    assert (out == -7.0).all()


@pytest.mark.gpu
def test_mfma_rate_probe_runs_and_counts_flop(saap):
    # measurement aid: the launch completes, reports its operation count, and rejects bad arguments
    ops = torch.randn(1 << 16, device="cuda").to(torch.bfloat16)
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    flop = saap.mfma_rate_probe(ops, 16, sink, wgs_per_cu=1)
    torch.cuda.synchronize()
    cus = saap.load_library().saap_device_compute_units()
    assert flop == cus * 4 * 16 * 8 * 2.0 * 32 * 32 * 16
    with pytest.raises(saap.SaapError):
        saap.mfma_rate_probe(ops, 0, sink)
