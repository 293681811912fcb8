"""Pins of the oracle's prefill-time sparse attention (the reading of the paper's Conclusion written in
oracle/saap_ref.c: the decode-time rule of Sections 3-5 applied to every token of a block of the prompt)
against numpy / scipy brute force, against causal softmax attention, and against the decode-time
function it must reduce to for a single token.  No GPU."""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import ref


def make(seed, S=2, Hq=4, Hkv=2, Nt=90, Tq=12, B=6, d=128):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((S, Tq, Hq, d)).astype(np.float32)
    K = rng.standard_normal((S, Hkv, Nt, d)).astype(np.float32)
    V = rng.standard_normal((S, Hkv, Nt, d)).astype(np.float32)
    ids = rng.integers(0, B, size=(S, Hkv, Nt)).astype(np.int32)
    return rng, q, K, V, ids


def brute(q, K, V, ids, sel, pos0, n_sink, n_recent, scale):
    S, Tq, Hq, d = q.shape
    Hkv, Nt = K.shape[1], K.shape[2]
    G = Hq // Hkv
    out = np.zeros((S, Tq, Hq, d))
    lse = np.zeros((S, Tq, Hq))
    pos = np.arange(Nt)
    for s in range(S):
        for t in range(Tq):
            L = pos0[s] + t + 1
            for hq in range(Hq):
                h = hq // G
                mask = (pos < L) & ((pos < n_sink) | (pos >= L - n_recent) | np.isin(ids[s, h], sel[s, h, t]))
                if not mask.any():                      # nothing visible: zero output, log-sum-exp of nothing
                    lse[s, t, hq] = -np.inf
                    continue
                a = (K[s, h][mask].astype(np.float64) @ q[s, t, hq].astype(np.float64)) * scale
                out[s, t, hq] = softmax(a) @ V[s, h][mask].astype(np.float64)
                lse[s, t, hq] = logsumexp(a)
    return out, lse


@pytest.mark.parametrize("n_sink,n_recent,nprobe,pos0", [(1, 7, 2, (30, 70)), (0, 0, 3, (0, 5)), (3, 16, 0, (78, 0)), (2, 1, 6, (10, 11))])
def test_matches_brute_force(n_sink, n_recent, nprobe, pos0):
    rng, q, K, V, ids = make(3)
    B, scale = 6, float(np.float32(0.11))     # the oracle takes the scale as a float
    S, Tq, Hq, _ = q.shape
    sel = np.stack([rng.permutation(B)[:nprobe] for _ in range(S * 2 * Tq)]).reshape(S, 2, Tq, nprobe).astype(np.int32)
    pos0 = np.array(pos0, dtype=np.int32)
    out, lse = ref.prefill_sparse_attention(q, K, V, ids, sel, pos0, n_sink, n_recent, scale, B)
    bo, bl = brute(q, K, V, ids, sel, pos0, n_sink, n_recent, scale)
    np.testing.assert_allclose(out, bo, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(lse, bl, rtol=1e-12)


def test_every_bucket_listed_is_causal_attention():
    """With all buckets in every list (or a window as long as the prompt) the restriction disappears: the result is
    plain causal softmax attention, computed here with a lower-triangular mask on the full score matrix."""
    rng, q, K, V, ids = make(5, S=1, Hq=2, Hkv=1, Nt=40, Tq=40)
    B, scale = 6, 0.09375
    every = np.tile(np.arange(B, dtype=np.int32), (1, 1, 40, 1))
    pos0 = np.zeros(1, dtype=np.int32)
    a = np.einsum("thd,nd->htn", q[0].astype(np.float64), K[0, 0].astype(np.float64)) * scale
    a = np.where(np.tril(np.ones((40, 40), dtype=bool))[None], a, -np.inf)
    want = np.einsum("htn,nd->thd", softmax(a, axis=-1), V[0, 0].astype(np.float64))
    for sel, n_sink, n_recent in ((every, 0, 0), (every[..., :0], 0, 40), (every[..., :2], 1, 64)):
        out, lse = ref.prefill_sparse_attention(q, K, V, ids, sel, pos0, n_sink, n_recent, scale, B)
        np.testing.assert_allclose(out[0], want, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(lse[0], logsumexp(a, axis=-1).T, rtol=1e-12)
    # the first token sees its own key only
    np.testing.assert_allclose(out[0, 0], np.broadcast_to(V[0, 0, 0], (2, 128)), rtol=1e-12)


def test_one_token_is_the_decode_time_attention_over_the_keys_so_far():
    """A block of one token at the last position: the keys so far are the whole cache, and the function must agree
    with the decode-time attention with sink and recent keys (pinned on its own)."""
    rng, q, K, V, ids = make(7, S=2, Hq=4, Hkv=2, Nt=120, Tq=1)
    B, scale = 6, 0.125
    sel = np.stack([rng.permutation(B)[:2] for _ in range(4)]).reshape(2, 2, 1, 2).astype(np.int32)
    pos0 = np.array([119, 119], dtype=np.int32)
    out, lse = ref.prefill_sparse_attention(q, K, V, ids, sel, pos0, 2, 9, scale, B)
    wo, wl = ref.windowed_decode_attention(q[:, 0], K, V, ids, sel[:, :, 0], 2, 9, scale, B)
    np.testing.assert_allclose(out[:, 0], wo, rtol=1e-13)
    np.testing.assert_allclose(lse[:, 0], wl, rtol=1e-13)
    # a token in the middle: the same with the cache cut after its own key
    pos0 = np.array([50, 77], dtype=np.int32)
    out, lse = ref.prefill_sparse_attention(q, K, V, ids, sel, pos0, 2, 9, scale, B)
    for s in range(2):
        L = pos0[s] + 1
        wo, wl = ref.windowed_decode_attention(q[s:s + 1, 0], K[s:s + 1, :, :L], V[s:s + 1, :, :L], ids[s:s + 1, :, :L],
                                               sel[s:s + 1, :, 0], 2, 9, scale, B)
        np.testing.assert_allclose(out[s, 0], wo[0], rtol=1e-13)
        np.testing.assert_allclose(lse[s, 0], wl[0], rtol=1e-13)
