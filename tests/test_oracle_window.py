"""Pins of the oracle's resident-block functions (attention sink + recent keys, Section 3
"Per-head attention span" and Appendix F of arXiv 2502.08246) against numpy brute force and
against what the mathematics fixes.  No GPU."""
import numpy as np
import pytest

from oracle import ref


def softmax_attention(q, K, V, scale):
    """Textbook fp64 softmax attention of one query over the rows of K, V."""
    a = (K.astype(np.float64) @ q.astype(np.float64)) * scale
    if a.size == 0:
        return np.zeros(V.shape[1]), -np.inf
    m = a.max()
    w = np.exp(a - m)
    return (w[:, None] * V.astype(np.float64)).sum(0) / w.sum(), m + np.log(w.sum())


def make(seed, S=2, Hq=4, Hkv=2, N=300, B=8, d=128, extra=40):
    rng = np.random.default_rng(seed)
    Nt = N + extra
    x = rng.standard_normal((S, Hkv, Nt, d)).astype(np.float32)
    K = rng.standard_normal((S, Hkv, Nt, d)).astype(np.float32)
    V = rng.standard_normal((S, Hkv, Nt, d)).astype(np.float32)
    cent = rng.standard_normal((Hkv, B, d)).astype(np.float32)
    q = rng.standard_normal((S, Hq, d)).astype(np.float32)
    ids = np.argmax(np.einsum("shnd,hbd->shnb", x.astype(np.float64), cent.astype(np.float64)), axis=-1).astype(np.int32)
    return x, K, V, cent, q, ids


def brute_windowed(q, K, V, ids, sel, n_sink, n_recent, scale):
    S, Hq, d = q.shape
    Hkv, Nt = K.shape[1], K.shape[2]
    G = Hq // Hkv
    out = np.zeros((S, Hq, d))
    lse = np.zeros((S, Hq))
    pos = np.arange(Nt)
    for s in range(S):
        for hq in range(Hq):
            h = hq // G
            mask = (pos < n_sink) | (pos >= Nt - n_recent) | np.isin(ids[s, h], sel[s, h])
            out[s, hq], lse[s, hq] = softmax_attention(q[s, hq], K[s, h][mask], V[s, h][mask], scale)
    return out, lse


@pytest.mark.parametrize("n_sink,n_recent,nprobe", [(1, 15, 3), (4, 32, 0), (0, 16, 2), (2, 0, 3), (0, 0, 4), (1, 31, 8)])
def test_windowed_attention_matches_brute_force(n_sink, n_recent, nprobe):
    x, K, V, cent, q, ids = make(1)
    B = cent.shape[1]
    rng = np.random.default_rng(5)
    sel = np.stack([np.stack([rng.permutation(B)[:nprobe] for _ in range(K.shape[1])]) for _ in range(K.shape[0])]).astype(np.int32)
    scale = float(np.float32(1.0 / np.sqrt(128.0)))   # the oracle takes the scale as a float
    out, lse = ref.windowed_decode_attention(q, K, V, ids, sel, n_sink, n_recent, scale, B)
    bo, bl = brute_windowed(q, K, V, ids, sel, n_sink, n_recent, scale)
    np.testing.assert_allclose(out, bo, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, bl, rtol=1e-12, atol=1e-12)


def test_all_buckets_plus_window_is_dense_and_no_bucket_is_the_window_alone():
    x, K, V, cent, q, ids = make(2)
    S, Hkv, Nt, d = K.shape
    B = cent.shape[1]
    scale = 0.125
    G = q.shape[1] // Hkv
    every = np.broadcast_to(np.arange(B, dtype=np.int32), (S, Hkv, B)).copy()
    out, lse = ref.windowed_decode_attention(q, K, V, ids, every, 1, 31, scale, B)
    none = np.zeros((S, Hkv, 0), dtype=np.int32)
    wout, wlse = ref.windowed_decode_attention(q, K, V, ids, none, 1, 31, scale, B)
    for s in range(S):
        for hq in range(q.shape[1]):
            h = hq // G
            o, l = softmax_attention(q[s, hq], K[s, h], V[s, h], scale)
            np.testing.assert_allclose(out[s, hq], o, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(lse[s, hq], l, rtol=1e-12)
            keep = np.r_[0:1, Nt - 31:Nt]
            o, l = softmax_attention(q[s, hq], K[s, h][keep], V[s, h][keep], scale)
            np.testing.assert_allclose(wout[s, hq], o, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(wlse[s, hq], l, rtol=1e-12)


def check_state(off, ln, idx, Ks, Vs, res, K, V, ids, Nt, B, slack, n_sink, n_recent):
    """The index state against its position-based meaning, by brute force."""
    S, Hkv = ln.shape[:2]
    W = n_sink + n_recent
    pos = np.arange(Nt)
    resident = (pos < n_sink) | (pos >= Nt - n_recent)
    for s in range(S):
        for h in range(Hkv):
            o, l, ix = off[s, h], ln[s, h], idx[s, h]
            assert o[0] == 0 and o[B + 1] - o[B] == W
            assert l.sum() == Nt and l[B] == resident.sum()
            for b in range(B):
                want = pos[(~resident) & (ids[s, h, :Nt] == b)]
                got = ix[o[b]:o[b] + l[b]]
                np.testing.assert_array_equal(got, want)          # ascending position
                assert o[b] + l[b] <= o[b + 1]
                assert (ix[o[b] + l[b]:o[b + 1]] == -1).all()                    # free slots are marked
            got = ix[o[B]:o[B] + W]
            np.testing.assert_array_equal(np.sort(got[got >= 0]), pos[resident])
            for p in pos[resident]:
                r = p if p < n_sink else n_sink + (p - n_sink) % n_recent
                assert got[r] == p and res[s, h, r] == ids[s, h, p]
            members = ix >= 0
            # slots freed inside the ring never exist; every member slot holds its key's row
            rows = ix[members]
            live = np.zeros(len(ix), dtype=bool)
            for b in range(B + 1):
                cap = W if b == B else l[b]
                live[o[b]:o[b] + cap] = True
            live &= members
            np.testing.assert_array_equal(Ks[s, h][live], K[s, h][ix[live]])
            np.testing.assert_array_equal(Vs[s, h][live], V[s, h][ix[live]])
            assert len(np.unique(ix[live])) == live.sum() == Nt


@pytest.mark.parametrize("N,n_sink,n_recent,slack,steps", [(300, 1, 31, 40, 40), (300, 4, 16, 40, 40), (20, 2, 30, 40, 40),
                                                           (300, 0, 8, 40, 25), (300, 3, 0, 20, 20)])
def test_build_and_push_keep_the_position_meaning(N, n_sink, n_recent, slack, steps):
    x, K, V, cent, q, ids = make(3, N=N, extra=steps)
    S, Hkv, Nt, d = K.shape
    B = cent.shape[1]
    off, ln, idx, Ks, Vs, res = ref.build_windowed_index(ids[:, :, :N], K[:, :, :N], V[:, :, :N], B, slack, n_sink, n_recent)
    check_state(off, ln, idx, Ks, Vs, res, K, V, ids, N, B, slack, n_sink, n_recent)
    scale = float(np.float32(1.0 / np.sqrt(128.0)))   # the oracle takes the scale as a float
    rng = np.random.default_rng(9)
    for t in range(steps):
        pos = np.full((S,), N + t, dtype=np.int32)
        new_ids, flag = ref.window_push(x[:, :, N + t], K[:, :, N + t], V[:, :, N + t], pos, cent, None, off, ln, idx, Ks, Vs,
                                        res, n_sink, n_recent)
        assert flag == 0
        np.testing.assert_array_equal(new_ids, ids[:, :, N + t])       # library argmax on random data (no ties)
        if t % 7 == 0 or t == steps - 1:
            check_state(off, ln, idx, Ks, Vs, res, K, V, ids, N + t + 1, B, slack, n_sink, n_recent)
            # attention through the index (resident block = one more visited run) equals the
            # position-based definition
            sel = np.stack([np.stack([rng.permutation(B)[:3] for _ in range(Hkv)]) for _ in range(S)]).astype(np.int32)
            sel_plus = np.concatenate([sel, np.full((S, Hkv, 1), B, dtype=np.int32)], axis=2)
            Nt_now = N + t + 1
            a, al = ref.sparse_decode_attention(q, K[:, :, :Nt_now], V[:, :, :Nt_now], off, ln, idx, sel_plus, scale)
            b, bl = ref.windowed_decode_attention(q, K[:, :, :Nt_now], V[:, :, :Nt_now], ids[:, :, :Nt_now], sel, n_sink, n_recent,
                                                  scale, B)
            np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(al, bl, rtol=1e-12)


def test_push_into_a_full_bucket_changes_nothing_and_raises_the_flag():
    x, K, V, cent, q, ids = make(4, S=1, Hkv=1, Hq=1, N=100, extra=4)
    B = cent.shape[1]
    N = 100
    off, ln, idx, Ks, Vs, res = ref.build_windowed_index(ids[:, :, :N], K[:, :, :N], V[:, :, :N], B, 0, 1, 7)
    before = [a.copy() for a in (off, ln, idx, Ks, Vs, res)]
    pos = np.full((1,), N, dtype=np.int32)
    _, flag = ref.window_push(x[:, :, N], K[:, :, N], V[:, :, N], pos, cent, None, off, ln, idx, Ks, Vs, res, 1, 7)
    assert flag == 1
    for a, b in zip(before, (off, ln, idx, Ks, Vs, res)):
        np.testing.assert_array_equal(a, b)


def test_recompact_keeps_every_member_and_restores_the_slack():
    """After pushes have eaten the slack: the recompacted index holds the same keys in the same buckets in the
    same order (position meaning unchanged, by brute force), every bucket has its fresh slack again, the
    attention through it is unchanged, and a cache that is too small is refused."""
    N, n_sink, n_recent, slack, steps = 300, 2, 30, 12, 60
    x, K, V, cent, q, ids = make(6, N=N, extra=steps + 10)
    S, Hkv, Nt, d = K.shape
    B = cent.shape[1]
    off, ln, idx, Ks, Vs, res = ref.build_windowed_index(ids[:, :, :N], K[:, :, :N], V[:, :, :N], B, slack, n_sink, n_recent)
    t = 0
    while True:                                            # push until some bucket is full
        pos = np.full((S,), N + t, dtype=np.int32)
        state = [a.copy() for a in (ln, idx, Ks, Vs, res)]
        _, flag = ref.window_push(x[:, :, N + t], K[:, :, N + t], V[:, :, N + t], pos, cent, None, off, ln, idx, Ks, Vs, res,
                                  n_sink, n_recent)
        if flag:
            ln, idx, Ks, Vs, res = state               # a refused push changes nothing for its head; undo the others too
            break
        t += 1
        assert t < steps
    n_now = N + t
    W = n_sink + n_recent
    Ncap_new = n_now - W + B * 20 + W
    off2, idx2, K2, V2, flag = ref.recompact_index(off, ln, idx, Ks, Vs, 20, Ncap_new, resident=True)
    assert flag == 0
    check_state(off2, ln, idx2, K2, V2, res, K, V, ids, n_now, B, 20, n_sink, n_recent)
    for s in range(S):
        for h in range(Hkv):
            for b in range(B):
                assert off2[s, h, b + 1] - off2[s, h, b] == ln[s, h, b] + 20
    scale = 0.125
    sel = np.broadcast_to(np.array([1, 4, 6], dtype=np.int32), (S, Hkv, 3)).copy()
    sel_plus = np.concatenate([sel, np.full((S, Hkv, 1), B, dtype=np.int32)], axis=2)
    a, _ = ref.sparse_decode_attention(q, K[:, :, :n_now], V[:, :, :n_now], off, ln, idx, sel_plus, scale)
    b, _ = ref.sparse_decode_attention(q, K[:, :, :n_now], V[:, :, :n_now], off2, ln, idx2, sel_plus, scale)
    np.testing.assert_array_equal(a, b)
    # the push that was refused goes through now
    pos = np.full((S,), n_now, dtype=np.int32)
    _, flag = ref.window_push(x[:, :, n_now], K[:, :, n_now], V[:, :, n_now], pos, cent, None, off2, ln, idx2, K2, V2, res,
                              n_sink, n_recent)
    assert flag == 0
    _, _, _, _, flag = ref.recompact_index(off2, ln, idx2, K2, V2, 20, Ncap_new - 1 - B * 20, resident=True)
    assert flag == 1


def test_recompact_while_the_window_is_still_filling():
    """A context shorter than the window: the resident run keeps all its W slots through a re-compaction
    (not just the occupied ones), so later pushes still find their ring slots."""
    N, n_sink, n_recent, slack = 20, 2, 30, 3
    x, K, V, cent, q, ids = make(8, N=N, extra=60)
    S, Hkv, Nt, d = K.shape
    B = cent.shape[1]
    W = n_sink + n_recent
    off, ln, idx, Ks, Vs, res = ref.build_windowed_index(ids[:, :, :N], K[:, :, :N], V[:, :, :N], B, slack, n_sink, n_recent)

    def push(t, off):
        pos = np.full((S,), t, dtype=np.int32)
        _, flag = ref.window_push(x[:, :, t], K[:, :, t], V[:, :, t], pos, cent, None, off, ln, idx, Ks, Vs, res, n_sink, n_recent)
        assert flag == 0

    for t in range(N, N + 5):
        push(t, off)
    n_now = N + 5
    assert n_now < W and (ln[:, :, B] == n_now).all()
    off, idx, Ks, Vs, flag = ref.recompact_index(off, ln, idx, Ks, Vs, 9, B * 9 + W, resident=True)
    assert flag == 0
    check_state(off, ln, idx, Ks, Vs, res, K, V, ids, n_now, B, 9, n_sink, n_recent)
    for t in range(n_now, n_now + 40):                      # the window fills (at 32 keys), then slides
        push(t, off)
    check_state(off, ln, idx, Ks, Vs, res, K, V, ids, n_now + 40, B, 9, n_sink, n_recent)
