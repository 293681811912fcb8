"""Pins for the CPU oracle (oracle/saap_ref.c): every oracle function is checked against
something other than itself -- numpy/scipy library routines on small inputs, closed forms,
invariants, and the one table of the paper that is a closed form (balanced selectivity).
No GPU is involved.  Each test is chosen so that a plausible mistake in the oracle (wrong
sign, dropped scale, transposed operand, off-by-one in the index, unstable order) fails it.
"""
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bf16_round(a):
    """Round float32 -> bf16 (RNE) -> float32 with integer arithmetic."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


# ----------------------------------------------------------------------------- assign_keys
def test_assign_matches_numpy_argmax(rng):
    S, Hkv, N, B, d = 2, 3, 257, 13, 128
    x = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    c = rng.standard_normal((Hkv, B, d)).astype(np.float32)
    bias = rng.standard_normal((Hkv, B)).astype(np.float32)
    for b in (None, bias):
        ids = ref.assign_keys(x, c, b)
        t = np.einsum("shnd,hbd->shnb", x.astype(np.float64), c.astype(np.float64))
        if b is not None:
            t = t + b.astype(np.float64)[None, :, None, :]
        assert np.array_equal(ids, t.argmax(-1).astype(np.int32))


def test_assign_planted_and_euclidean(rng):
    Hkv, B, d, N = 2, 32, 128, 400
    c = rng.standard_normal((Hkv, B, d)).astype(np.float32)
    c /= np.linalg.norm(c, axis=-1, keepdims=True)
    truth = rng.integers(0, B, size=(1, Hkv, N))
    x = np.stack([3.0 * c[h, truth[0, h]] for h in range(Hkv)])[None] + 0.01 * rng.standard_normal((1, Hkv, N, d))
    x = x.astype(np.float32)
    assert np.array_equal(ref.assign_keys(x, c), truth.astype(np.int32))
    # bias = -|c|^2/2 turns the rule into the Euclidean nearest centroid
    c2 = (c * rng.uniform(0.5, 2.0, size=(Hkv, B, 1))).astype(np.float32)
    bias = (-0.5 * (c2.astype(np.float64) ** 2).sum(-1)).astype(np.float32)
    ids = ref.assign_keys(x, c2, bias)
    dist = ((x.astype(np.float64)[:, :, :, None, :] - c2.astype(np.float64)[None, :, None, :, :]) ** 2).sum(-1)
    near = dist.argmin(-1)
    # the float32 rounding of the bias can only matter at near-ties; none are planted here
    assert np.array_equal(ids, near.astype(np.int32))


def test_assign_ties_and_permutation(rng):
    B, d, N = 16, 128, 200
    c = rng.standard_normal((1, B, d)).astype(np.float32)
    c[0, 9] = c[0, 4]          # exact duplicates: the lower id must win
    c[0, 12] = c[0, 4]
    x = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    x[0, 0, :50] = 5.0 * c[0, 4] + 0.01 * x[0, 0, :50]
    ids = ref.assign_keys(x, c)
    assert (ids[0, 0, :50] == 4).all()
    assert not np.isin(ids, (9, 12)).any()
    perm = rng.permutation(B)
    cu = rng.standard_normal((1, B, d)).astype(np.float32)
    a = ref.assign_keys(x, cu)
    b = ref.assign_keys(x, cu[:, perm])
    assert np.array_equal(perm[b], a)


# ------------------------------------------------------------------- build_bucket_index
@pytest.mark.parametrize("slack", [0, 3])
def test_build_index_matches_argsort_and_invariants(rng, slack):
    S, Hkv, N, B, d = 2, 2, 1000, 37, 128
    ids = rng.integers(0, B, size=(S, Hkv, N)).astype(np.int32)
    ids[0, 0][ids[0, 0] == 5] = 6      # an empty bucket
    K = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    V = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    off, ln, idx, Ks, Vs = ref.build_bucket_index(ids, K, V, B, slack)
    Ncap = N + B * slack
    assert idx.shape == (S, Hkv, Ncap)
    for s in range(S):
        for h in range(Hkv):
            cnt = np.bincount(ids[s, h], minlength=B)
            assert np.array_equal(ln[s, h], cnt)
            assert off[s, h, 0] == 0
            assert np.array_equal(np.diff(off[s, h]), cnt + slack)
            order = np.argsort(ids[s, h], kind="stable")
            members = np.concatenate([idx[s, h, off[s, h, b]:off[s, h, b] + ln[s, h, b]] for b in range(B)])
            assert np.array_equal(members, order)           # stable: ascending position inside a bucket
            assert np.array_equal(np.sort(members), np.arange(N))
            for b in range(B):
                run = slice(off[s, h, b], off[s, h, b] + ln[s, h, b])
                assert (ids[s, h, idx[s, h, run]] == b).all()
                assert np.array_equal(Ks[s, h, run], K[s, h, idx[s, h, run]])
                assert np.array_equal(Vs[s, h, run], V[s, h, idx[s, h, run]])
                assert (idx[s, h, off[s, h, b] + ln[s, h, b]:off[s, h, b + 1]] == -1).all()
    if slack == 0:
        assert (off[:, :, B] == N).all()


def test_append_uses_free_slot_and_reports_overflow(rng):
    S, Hkv, N, B, d, slack = 2, 2, 64, 4, 128, 1
    c = rng.standard_normal((Hkv, B, d)).astype(np.float32)
    x = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    K = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    V = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    ids = ref.assign_keys(x, c)
    off, ln, idx, Ks, Vs = ref.build_bucket_index(ids, K, V, B, slack)
    ln0 = ln.copy()
    xn = np.stack([np.stack([4.0 * c[h, (s + h) % B] for h in range(Hkv)]) for s in range(S)]).astype(np.float32)
    kn = rng.standard_normal((S, Hkv, d)).astype(np.float32)
    vn = rng.standard_normal((S, Hkv, d)).astype(np.float32)
    pos = np.array([N, N], dtype=np.int32)
    new_ids, flag = ref.append_keys(xn, kn, vn, pos, c, None, off, ln, idx, Ks, Vs)
    assert flag == 0
    for s in range(S):
        for h in range(Hkv):
            b = (s + h) % B
            assert new_ids[s, h] == b
            assert ln[s, h, b] == ln0[s, h, b] + 1
            j = off[s, h, b] + ln0[s, h, b]
            assert idx[s, h, j] == N and np.array_equal(Ks[s, h, j], kn[s, h]) and np.array_equal(Vs[s, h, j], vn[s, h])
    ln1 = ln.copy()
    new_ids, flag = ref.append_keys(xn, kn, vn, pos, c, None, off, ln, idx, Ks, Vs)   # slack exhausted
    assert flag == 1 and np.array_equal(ln, ln1)


# --------------------------------------------------------------------- classify_queries
@pytest.mark.parametrize("Hw_kind", ["one", "kv", "q"])
def test_classifier_matches_library_matmul_softmax(rng, Hw_kind):
    S, Hq, Hkv, d, hid, B = 3, 8, 2, 128, 96, 48
    Hw = {"one": 1, "kv": Hkv, "q": Hq}[Hw_kind]
    xq = rng.standard_normal((S, Hq, d)).astype(np.float32)
    W1 = (rng.standard_normal((Hw, hid, d)) / np.sqrt(d)).astype(np.float32)
    W2 = (rng.standard_normal((Hw, B, hid)) / np.sqrt(hid)).astype(np.float32)
    b1 = rng.standard_normal((Hw, hid)).astype(np.float32)
    b2 = rng.standard_normal((Hw, B)).astype(np.float32)
    p = ref.classify_queries(xq, W1, b1, W2, b2, Hkv)
    z = ref.classify_queries(xq, W1, b1, W2, b2, Hkv, output_kind=1)
    G = Hq // Hkv
    for hq in range(Hq):
        w = {"one": 0, "kv": hq // G, "q": hq}[Hw_kind]
        h = np.maximum(xq[:, hq].astype(np.float64) @ W1[w].astype(np.float64).T + b1[w], 0.0)
        zz = h @ W2[w].astype(np.float64).T + b2[w]
        np.testing.assert_allclose(z[:, hq], zz, rtol=1e-6, atol=1e-6)
        np.testing.assert_allclose(p[:, hq], softmax(zz, axis=-1), rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-6)


def test_classifier_zero_output_layer_is_uniform(rng):
    S, Hq, Hkv, d, hid, B = 1, 4, 1, 128, 64, 32
    xq = rng.standard_normal((S, Hq, d)).astype(np.float32)
    W1 = rng.standard_normal((1, hid, d)).astype(np.float32)
    p = ref.classify_queries(xq, W1, None, np.zeros((1, B, hid), np.float32), None, Hkv)
    np.testing.assert_allclose(p, 1.0 / B, rtol=1e-7)
    # a bias alone decides the distribution when W2 = 0
    b2 = rng.standard_normal((1, B)).astype(np.float32)
    p = ref.classify_queries(xq, W1, None, np.zeros((1, B, hid), np.float32), b2, Hkv)
    np.testing.assert_allclose(p[0, 2], softmax(b2[0].astype(np.float64)), rtol=1e-6)


# ----------------------------------------------------------------------- select_buckets
@pytest.mark.parametrize("mode", [0, 1])
def test_select_matches_stable_argsort(rng, mode):
    S, Hq, Hkv, B, nprobe = 3, 8, 2, 200, 17
    G = Hq // Hkv
    scores = softmax(rng.standard_normal((S, Hq, B)) * 3, axis=-1).astype(np.float32)
    scores[0, :, 50] = scores[0, :, 20]            # planted ties
    scores[1, :, 7] = scores[1, :, 150]
    sel = ref.select_buckets(scores, Hkv, nprobe, mode)
    if mode == 0:
        g = scores.reshape(S, Hkv, G, B)
        acc = g[:, :, 0]
        for i in range(1, G):
            acc = (acc + g[:, :, i]).astype(np.float32)
    else:
        acc = scores
    want = np.argsort(-acc.astype(np.float64), axis=-1, kind="stable")[..., :nprobe]
    assert np.array_equal(sel, want.astype(np.int32))


def test_select_ties_pick_lower_id_and_full_probe():
    B = 12
    scores = np.zeros((1, 4, B), np.float32)
    scores[0, :, 3] = 0.25
    scores[0, :, 8] = 0.25
    scores[0, :, 5] = 0.125
    sel = ref.select_buckets(scores, 1, 4, 0)
    assert sel.tolist() == [[[3, 8, 5, 0]]]
    sel = ref.select_buckets(scores, 1, B, 0)
    assert sorted(sel[0, 0].tolist()) == list(range(B))
    assert ref.select_buckets(scores, 1, 0, 0).shape == (1, 1, 0)


def test_select_group_sum_is_single_precision():
    # (a + b) + c differs between float32 and float64 accumulation for these values;
    # the ranking is defined on the float32 sum in head order.
    B = 2
    s = np.zeros((1, 4, B), np.float32)
    s[0, :, 0] = [1.0, 2.0 ** -24, 2.0 ** -24, 0.0]       # float32: stays 1.0 ; float64: 1 + 2^-23
    s[0, :, 1] = [1.0, 0.0, 0.0, 0.0]
    sel = ref.select_buckets(s, 1, 1, 0)
    assert sel[0, 0, 0] == 0     # exact float32 tie -> lower id (float64 would also give 0)
    s[0, :, 1] = [1.0, 2.0 ** -24, 2.0 ** -24, 2.0 ** -24]   # float32: 1.0 ; float64: larger than bucket 0
    sel = ref.select_buckets(s, 1, 1, 0)
    assert sel[0, 0, 0] == 0     # still a float32 tie; a float64 sum would have picked bucket 1


# ---------------------------------------------------------------------------- attention
def _tiny_case(rng, S=2, Hq=4, Hkv=2, N=300, B=9, d=128, slack=0):
    K = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    V = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    q = rng.standard_normal((S, Hq, d)).astype(np.float32)
    ids = rng.integers(0, B, size=(S, Hkv, N)).astype(np.int32)
    off, ln, idx, Ks, Vs = ref.build_bucket_index(ids, K, V, B, slack)
    return K, V, q, ids, off, ln, idx


def test_dense_attention_matches_library_softmax(rng):
    K, V, q, *_ = _tiny_case(rng)
    scale = 1.0 / np.sqrt(128.0)
    out, lse = ref.dense_decode_attention(q, K, V, scale)
    S, Hq, d = q.shape
    G = Hq // K.shape[1]
    for s in range(S):
        for hq in range(Hq):
            a = (K[s, hq // G].astype(np.float64) @ q[s, hq].astype(np.float64)) * np.float32(scale)
            w = softmax(a)
            np.testing.assert_allclose(out[s, hq], w @ V[s, hq // G].astype(np.float64), rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(lse[s, hq], logsumexp(a), rtol=1e-12)


@pytest.mark.parametrize("mode,slack", [(0, 0), (0, 2), (1, 0)])
def test_sparse_attention_matches_brute_force(rng, mode, slack):
    K, V, q, ids, off, ln, idx = _tiny_case(rng, slack=slack)
    S, Hq, d = q.shape
    Hkv, B = K.shape[1], ln.shape[2]
    G = Hq // Hkv
    nprobe = 4
    lists = Hq if mode == 1 else Hkv
    sel = np.stack([np.stack([rng.permutation(B)[:nprobe] for _ in range(lists)]) for _ in range(S)]).astype(np.int32)
    scale = 0.1
    out, lse = ref.sparse_decode_attention(q, K, V, off, ln, idx, sel, scale, mode)
    for s in range(S):
        for hq in range(Hq):
            h = hq // G
            chosen = sel[s, hq if mode == 1 else h]
            mask = np.isin(ids[s, h], chosen)          # membership straight from the ids, not from the index
            a = (K[s, h][mask].astype(np.float64) @ q[s, hq].astype(np.float64)) * np.float32(scale)
            np.testing.assert_allclose(out[s, hq], softmax(a) @ V[s, h][mask].astype(np.float64), rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(lse[s, hq], logsumexp(a), rtol=1e-12)


def test_sparse_with_all_buckets_equals_dense(rng):
    K, V, q, ids, off, ln, idx = _tiny_case(rng, slack=1)
    S, Hq, d = q.shape
    Hkv, B = K.shape[1], ln.shape[2]
    sel = np.tile(rng.permutation(B).astype(np.int32), (S, Hkv, 1))
    scale = 1.0 / np.sqrt(128.0)
    o1, l1 = ref.sparse_decode_attention(q, K, V, off, ln, idx, sel, scale)
    o2, l2 = ref.dense_decode_attention(q, K, V, scale)
    np.testing.assert_allclose(o1, o2, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(l1, l2, rtol=1e-12)


def test_attention_closed_forms(rng):
    S, Hq, Hkv, N, B, d = 1, 2, 1, 120, 6, 128
    q = rng.standard_normal((S, Hq, d)).astype(np.float32)
    ids = rng.integers(0, B, size=(S, Hkv, N)).astype(np.int32)
    sel = np.array([[[1, 4]]], dtype=np.int32)
    member = np.isin(ids[0, 0], [1, 4])
    # equal keys -> uniform weights -> mean of the visited values; lse = a + log(count)
    K = np.tile(rng.standard_normal((1, 1, 1, d)).astype(np.float32), (1, 1, N, 1))
    V = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    off, ln, idx, _, _ = ref.build_bucket_index(ids, K, V, B)
    out, lse = ref.sparse_decode_attention(q, K, V, off, ln, idx, sel, 0.05)
    for hq in range(Hq):
        np.testing.assert_allclose(out[0, hq], V[0, 0][member].astype(np.float64).mean(0), rtol=1e-9, atol=1e-12)
        a = np.float64(np.float32(0.05)) * (K[0, 0, 0].astype(np.float64) @ q[0, hq].astype(np.float64))
        np.testing.assert_allclose(lse[0, hq], a + np.log(member.sum()), rtol=1e-12)
    # equal values -> that value, whatever the keys
    K = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    V = np.tile(rng.standard_normal((1, 1, 1, d)).astype(np.float32), (1, 1, N, 1))
    out, _ = ref.sparse_decode_attention(q, K, V, off, ln, idx, sel, 0.3)
    np.testing.assert_allclose(out[0, 0], V[0, 0, 0].astype(np.float64), rtol=1e-12)
    # one visited key -> its value; lse = its score
    ids1 = np.zeros((S, Hkv, N), np.int32)
    ids1[0, 0, 77] = 3
    V = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    off, ln, idx, _, _ = ref.build_bucket_index(ids1, K, V, B)
    out, lse = ref.sparse_decode_attention(q, K, V, off, ln, idx, np.array([[[3]]], np.int32), 0.3)
    np.testing.assert_allclose(out[0, 1], V[0, 0, 77].astype(np.float64), rtol=1e-12)
    np.testing.assert_allclose(lse[0, 1], np.float64(np.float32(0.3)) * (K[0, 0, 77].astype(np.float64) @ q[0, 1].astype(np.float64)), rtol=1e-12)
    # nothing visited -> zeros and -inf
    out, lse = ref.sparse_decode_attention(q, K, V, off, ln, idx, np.array([[[5]]], np.int32), 0.3)
    assert (out == 0).all() and np.isneginf(lse).all()


def test_attention_split_and_merge_is_associative(rng):
    """Appendix F, Algorithm 2 (merge): attention over a union of disjoint parts equals the
    log-sum-exp weighted combination of the parts' results."""
    K, V, q, ids, off, ln, idx = _tiny_case(rng, S=1, Hq=2, Hkv=1, N=500, B=8)
    scale = 0.2
    whole, lse = ref.sparse_decode_attention(q, K, V, off, ln, idx, np.arange(8, dtype=np.int32).reshape(1, 1, 8), scale)
    parts = [np.array([[[0, 5, 6]]], np.int32), np.array([[[1]]], np.int32), np.array([[[2, 3, 4, 7]]], np.int32)]
    res = [ref.sparse_decode_attention(q, K, V, off, ln, idx, p, scale) for p in parts]
    lses = np.stack([r[1] for r in res])             # [parts,S,Hq]
    w = np.exp(lses - logsumexp(lses, axis=0))
    merged = sum(w[i][..., None] * res[i][0] for i in range(len(parts)))
    np.testing.assert_allclose(merged, whole, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(logsumexp(lses, axis=0), lse, rtol=1e-12)


def test_attention_scale_times_query(rng):
    """Only the product scale * q enters the scores: doubling q and halving the scale changes nothing."""
    K, V, q, ids, off, ln, idx = _tiny_case(rng, S=1, Hq=2, Hkv=1, N=200, B=4)
    sel = np.array([[[0, 2]]], np.int32)
    o1, l1 = ref.sparse_decode_attention(q, K, V, off, ln, idx, sel, 0.25)
    o2, l2 = ref.sparse_decode_attention(2.0 * q, K, V, off, ln, idx, sel, 0.125)
    np.testing.assert_allclose(o1, o2, rtol=1e-12)
    np.testing.assert_allclose(l1, l2, rtol=1e-12)


# -------------------------------------------------------------------------- selectivity
def test_balanced_selectivity_matches_paper_table():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "selectivity_balanced.txt")) if l.strip() and not l.startswith("#")]
    C, per = 1024, 128
    ln = np.full((8, C), per, np.int32)
    for nprobe, pct in rows:
        nprobe, pct = int(nprobe), float(pct)
        sel = np.stack([np.random.default_rng(h).permutation(C)[:nprobe] for h in range(8)]).astype(np.int32)
        got = 100.0 * ref.selectivity(ln, sel, C * per)
        assert abs(got - 100.0 * nprobe / C) < 1e-12
        assert abs(got - pct) <= 0.05 + 1e-9, (nprobe, got, pct)     # the paper prints one decimal


def test_selectivity_counts_realised_sizes(rng):
    ln = rng.integers(0, 50, size=(3, 20)).astype(np.int32)
    sel = np.stack([rng.permutation(20)[:5] for _ in range(3)]).astype(np.int32)
    want = np.mean([ln[l, sel[l]].sum() / 1000.0 for l in range(3)])
    assert abs(ref.selectivity(ln, sel, 1000) - want) < 1e-15


def test_bf16_inputs_are_exact_in_oracle(rng):
    """bf16 data widened to float32 is what the oracle consumes: products of two such numbers are
    exact in float64, so the in-order sum of the assignment is reproducible by any exact method."""
    x = _bf16_round(rng.standard_normal((1, 1, 64, 128)).astype(np.float32))
    c = _bf16_round(rng.standard_normal((1, 8, 128)).astype(np.float32))
    ids = ref.assign_keys(x, c)
    from fractions import Fraction
    for n in range(0, 64, 9):
        best, bid = None, -1
        for b in range(8):
            t = sum(Fraction(float(x[0, 0, n, j])) * Fraction(float(c[0, b, j])) for j in range(128))
            if best is None or t > best:
                best, bid = t, b
        assert ids[0, 0, n] == bid


def test_one_layer_classifier_is_the_centroid_routing_of_the_kmeans_baseline():
    """hidden = 0: logits are the inner products with the rows of W2 (library matmul), and their
    arg-max agrees with assign_keys on the same vectors: a query routed like a key (Section 6.1)."""
    rng = np.random.default_rng(11)
    S, Hq, Hkv, B, d = 2, 4, 2, 16, 128
    xq = rng.standard_normal((S, Hq, d)).astype(np.float32)
    cent = rng.standard_normal((Hkv, B, d)).astype(np.float32)
    bias = rng.standard_normal((Hkv, B)).astype(np.float32)
    z = ref.classify_queries(xq, None, None, cent, bias, Hkv, output_kind=1)
    want = np.stack([[xq[s, hq].astype(np.float64) @ cent[hq // 2].astype(np.float64).T + bias[hq // 2]
                      for hq in range(Hq)] for s in range(S)])
    np.testing.assert_allclose(z, want, rtol=1e-6, atol=1e-6)
    ids = ref.assign_keys(xq.reshape(S, Hkv, 2, d), cent, bias)          # the same vectors seen as keys
    np.testing.assert_array_equal(z.argmax(-1).reshape(S, Hkv, 2), ids)
    p = ref.classify_queries(xq, None, None, cent, bias, Hkv)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-6)


def test_centroid_update_is_the_normalised_member_mean():
    """Against numpy: mean of the members, unit norm; an empty bucket keeps its centroid; one more
    Lloyd step never lowers the spherical k-means objective (sum of <x, c_assigned>) for unit-norm x."""
    rng = np.random.default_rng(12)
    S, Hkv, N, B, d = 2, 2, 400, 8, 128
    x = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=-1, keepdims=True)
    cent = rng.standard_normal((Hkv, B, d)).astype(np.float32)
    cent /= np.linalg.norm(cent, axis=-1, keepdims=True)
    ids = ref.assign_keys(x, cent)
    ids[ids == 3] = 2                                   # bucket 3 loses its members
    new = ref.update_centroids(x, ids, cent)
    for h in range(Hkv):
        for b in range(B):
            members = np.concatenate([x[s, h][ids[s, h] == b] for s in range(S)]).astype(np.float64)
            if b == 3:
                np.testing.assert_array_equal(new[h, b], cent[h, b].astype(np.float64))
                continue
            m = members.mean(0)
            np.testing.assert_allclose(new[h, b], m / np.linalg.norm(m), rtol=1e-12, atol=1e-14)
    plain = ref.update_centroids(x, ids, cent, normalize=False)
    np.testing.assert_allclose(plain[0, 0], np.concatenate([x[s, 0][ids[s, 0] == 0] for s in range(S)]).astype(np.float64).mean(0),
                               rtol=1e-12, atol=1e-14)
    # monotone objective over two full iterations
    def objective(c):
        a = ref.assign_keys(x, c.astype(np.float32))
        return sum(float((x[s, h].astype(np.float64) * c[h][a[s, h]]).sum()) for s in range(S) for h in range(Hkv)), a
    o0, a0 = objective(cent.astype(np.float64))
    c1 = ref.update_centroids(x, a0, cent)
    o1, a1 = objective(c1)
    c2 = ref.update_centroids(x, a1, c1.astype(np.float32))
    o2, _ = objective(c2)
    assert o1 >= o0 - 1e-6 and o2 >= o1 - 1e-3          # c1 is rounded to float32 for the second assignment
