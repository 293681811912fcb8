"""Pins of the oracle's bucket attention mass (the target A * H_k of Eq. 1, Section 4): numpy brute
force, rows that sum to one, and the identity that links it to the two attention oracles:
the mass of a set of buckets equals exp(lse over those buckets - lse over all keys)."""
import math

import numpy as np

from oracle import ref


def _inputs(seed, S=2, Hkv=2, G=2, N=300, d=128, B=7):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    V = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    q = rng.standard_normal((S, Hkv * G, d)).astype(np.float32)
    ids = rng.integers(0, B, (S, Hkv, N)).astype(np.int32)
    return q, K, V, ids


def test_mass_against_numpy_softmax():
    q, K, V, ids = _inputs(1)
    S, Hq, d = q.shape
    Hkv, N, B = K.shape[1], K.shape[2], 7
    scale = np.float32(1.0 / math.sqrt(d))
    mass = ref.bucket_attention_mass(q, K, ids, scale, B)
    for s in range(S):
        for hq in range(Hq):
            h = hq // (Hq // Hkv)
            a = float(scale) * (K[s, h].astype(np.float64) @ q[s, hq].astype(np.float64))
            p = np.exp(a - a.max())
            p /= p.sum()
            want = np.bincount(ids[s, h], weights=p, minlength=B)
            np.testing.assert_allclose(mass[s, hq], want, rtol=1e-10, atol=1e-15)
    np.testing.assert_allclose(mass.sum(-1), 1.0, rtol=1e-12)


def test_mass_of_a_selection_links_sparse_and_dense_lse():
    q, K, V, ids = _inputs(2)
    S, Hq, d = q.shape
    Hkv, B = K.shape[1], 7
    scale = np.float32(1.0 / math.sqrt(d))
    mass = ref.bucket_attention_mass(q, K, ids, scale, B)
    off, ln, idx, Ks, Vs = ref.build_bucket_index(ids, K, V, B, 0)
    sel = np.array([[[1, 4, 6], [0, 2, 3]], [[5, 1, 0], [6, 2, 4]]], dtype=np.int32)
    _, lse_sel = ref.sparse_decode_attention(q, K, V, off, ln, idx, sel, scale)
    _, lse_all = ref.dense_decode_attention(q, K, V, scale)
    G = Hq // Hkv
    for s in range(S):
        for hq in range(Hq):
            got = mass[s, hq][sel[s, hq // G]].sum()
            np.testing.assert_allclose(got, math.exp(lse_sel[s, hq] - lse_all[s, hq]), rtol=1e-9)


def test_one_bucket_and_one_dominant_key():
    q, K, V, ids = _inputs(3, S=1, Hkv=1, G=1, N=50, B=3)
    scale = np.float32(1.0)
    assert np.allclose(ref.bucket_attention_mass(q, K, np.zeros_like(ids), scale, 1), 1.0)
    K[0, 0, 17] = 50.0 * q[0, 0] / np.linalg.norm(q[0, 0])        # one key takes all the attention
    mass = ref.bucket_attention_mass(q, K, ids, scale, 3)
    assert mass[0, 0, ids[0, 0, 17]] > 1 - 1e-9
