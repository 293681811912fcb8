"""GPU parity tests of the attention-sink + recent-key window (Section 3 "Per-head attention span",
Appendix F Algorithm 2 of arXiv 2502.08246): the index with a resident run, the per-step push and the
attention that always visits that run, against the CPU oracle.  Index state is compared bit for bit;
attention against the oracle's POSITION-based definition (no index on that side) within
    |gpu - ref| <= 2e-3 + 1e-2 |ref| (bf16),  1e-5 + 1e-5 |ref| (fp32)."""
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
    err = np.abs(got[fin] - want[fin])
    lim = atol + rtol * np.abs(want[fin])
    bad = err > lim
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"


def live_slots(off, ln, idx, W):
    """Boolean mask [S,Hkv,Ncap] of slots that hold a key."""
    S, Hkv, Ncap = idx.shape
    B = ln.shape[2] - 1
    live = np.zeros(idx.shape, dtype=bool)
    for s in range(S):
        for u in range(Hkv):
            for b in range(B + 1):
                live[s, u, off[s, u, b]:off[s, u, b] + ln[s, u, b]] = True
    return live & (idx >= 0)


def compare_state(gpu, want, W, what):
    off, ln, idx, Ks, Vs, res = gpu
    r_off, r_ln, r_idx, rKs, rVs, r_res = want
    g_off, g_ln, g_idx, g_res = (t.cpu().numpy() for t in (off, ln, idx, res))
    assert np.array_equal(g_off, r_off), f"{what}: off"
    assert np.array_equal(g_ln, r_ln), f"{what}: len"
    assert np.array_equal(g_idx, r_idx), f"{what}: idx"
    assert np.array_equal(g_res, r_res), f"{what}: resident ids"
    live = live_slots(r_off, r_ln, r_idx, W)
    assert np.array_equal(h(Ks)[live], rKs[live]), f"{what}: K rows"
    assert np.array_equal(h(Vs)[live], rVs[live]), f"{what}: V rows"


@pytest.mark.parametrize("dtype,S,Hq,Hkv,N,B,slack,n_sink,n_recent,steps", [
    ("bf16", 2, 8, 2, 6000, 32, 40, 1, 255, 300),     # the paper's 1 + (2^k - 1) shape; the ring wraps
    ("f32", 1, 2, 1, 3000, 16, 40, 4, 60, 90),
    ("bf16", 1, 4, 1, 40, 8, 64, 2, 100, 160),        # context shorter than the window: it fills, then slides
    ("bf16", 1, 4, 2, 2500, 16, 16, 0, 64, 70),       # no sink
    ("bf16", 1, 2, 1, 2100, 16, 16, 3, 0, 20),        # no ring: new keys go straight to their buckets
    # the other dense blocks the paper tries (Section 6.5, "Dense context size"): 128+512, 1+511, 1+63;
    # with no bucket visited (nprobe 0 in the loop below) the result is attention on sink + recent keys alone
    ("bf16", 1, 4, 1, 5000, 32, 24, 128, 512, 40),
    ("bf16", 1, 8, 2, 4000, 32, 24, 1, 511, 40),
    ("bf16", 2, 4, 1, 3000, 16, 24, 1, 63, 80),
])
def test_build_push_attend(saap, dtype, S, Hq, Hkv, N, B, slack, n_sink, n_recent, steps):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N + steps, B=B, nprobe=4, dtype=dtype, hidden=64)
    cache = gen.make_cache(cfg, 41, DEV)
    cent = gen.make_centroids(cfg, 41, DEV, cache, n_train=2048)
    _, q = gen.make_queries(cfg, 41, DEV, n_steps=4)
    W = n_sink + n_recent
    x, K, V = cache["x_keys"], cache["K"], cache["V"]
    ids_all = saap.assign_keys(x, cent)                    # ids of every position, also those pushed later
    ids0 = ids_all[:, :, :N].contiguous()
    K0, V0 = K[:, :, :N].contiguous(), V[:, :, :N].contiguous()
    state = saap.build_windowed_index(ids0, K0, V0, B, slack, n_sink, n_recent)
    torch.cuda.synchronize()
    h_ids = ids_all.cpu().numpy()
    assert np.array_equal(h_ids, ref.assign_keys(h(x), h(cent)))
    hK, hV, hx, hc = h(K), h(V), h(x), h(cent)
    want = list(ref.build_windowed_index(h_ids[:, :, :N], hK[:, :, :N], hV[:, :, :N], B, slack, n_sink, n_recent))
    compare_state(state, want, W, "after build")
    off, ln, idx, Ks, Vs, res = state
    flag = torch.zeros(4, dtype=torch.int32, device=DEV)
    rng = np.random.default_rng(7)
    check_at = {0, 1, steps // 3, steps // 2, steps - 1}
    for t in range(steps):
        pos = torch.full((S,), N + t, dtype=torch.int32, device=DEV)
        xn, kn, vn = (a[:, :, N + t].contiguous() for a in (x, K, V))
        nid, _ = saap.window_push(xn, kn, vn, pos, cent, None, off, ln, idx, Ks, Vs, res, n_sink, n_recent, overflow_flag=flag)
        rid, rflag = ref.window_push(hx[:, :, N + t], hK[:, :, N + t], hV[:, :, N + t], pos.cpu().numpy(), hc, None,
                                     want[0], want[1], want[2], want[3], want[4], want[5], n_sink, n_recent)
        assert rflag == 0, "test sizing: slack must absorb every displaced key"
        if t in check_at:
            torch.cuda.synchronize()
            assert np.array_equal(nid.cpu().numpy(), rid)
            compare_state(state, want, W, f"after push {t}")
            Nt = N + t + 1
            for nprobe in (0, 4, B):
                sel = np.stack([np.stack([rng.permutation(B)[:nprobe] for _ in range(Hkv)]) for _ in range(S)]).astype(np.int32)
                sel = sel.reshape(S, Hkv, nprobe)
                d_sel = torch.from_numpy(sel).to(DEV)
                out, lse = saap.windowed_decode_attention(q[t % 4], Ks, Vs, off, ln, d_sel, B, SCALE)
                torch.cuda.synchronize()
                ro, rl = ref.windowed_decode_attention(h(q[t % 4]), hK[:, :, :Nt], hV[:, :, :Nt], h_ids[:, :, :Nt], sel,
                                                       n_sink, n_recent, SCALE, B)
                assert_close(out.cpu().numpy(), ro, dtype, f"push {t} nprobe {nprobe} out")
                assert_close(lse.cpu().numpy(), rl, dtype, f"push {t} nprobe {nprobe} lse")
                if nprobe == B:       # every bucket + the window = every key: the dense definition
                    do, dl = ref.dense_decode_attention(h(q[t % 4]), hK[:, :, :Nt], hV[:, :, :Nt], SCALE)
                    assert_close(out.cpu().numpy(), do, dtype, f"push {t} all buckets vs dense")
    torch.cuda.synchronize()
    assert flag[0].item() == 0


def test_push_into_full_bucket_raises_flag_and_changes_nothing(saap):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=1, Hq=4, Hkv=2, N=1000 + 3, B=8, nprobe=2, hidden=64)
    cache = gen.make_cache(cfg, 43, DEV)
    cent = gen.make_centroids(cfg, 43, DEV, cache, n_train=2048)
    N, B, n_sink, n_recent = 1000, 8, 1, 31
    x, K, V = cache["x_keys"], cache["K"], cache["V"]
    ids = saap.assign_keys(x, cent)
    state = saap.build_windowed_index(ids[:, :, :N].contiguous(), K[:, :, :N].contiguous(), V[:, :, :N].contiguous(), B, 0,
                                      n_sink, n_recent)
    torch.cuda.synchronize()
    before = [t.clone() for t in state]
    off, ln, idx, Ks, Vs, res = state
    pos = torch.full((1,), N, dtype=torch.int32, device=DEV)
    _, flag = saap.window_push(x[:, :, N].contiguous(), K[:, :, N].contiguous(), V[:, :, N].contiguous(), pos, cent, None,
                               off, ln, idx, Ks, Vs, res, n_sink, n_recent)
    torch.cuda.synchronize()
    assert flag[0].item() == 1
    for a, b in zip(before, state):
        assert torch.equal(a, b)


def test_resident_run_minus_one_is_plain_sparse_attention(saap):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=1, Hq=8, Hkv=2, N=4000, B=32, nprobe=5, hidden=64)
    cache = gen.make_cache(cfg, 47, DEV)
    cent = gen.make_centroids(cfg, 47, DEV, cache, n_train=2048)
    _, q = gen.make_queries(cfg, 47, DEV)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, 0)
    sel = torch.stack([torch.randperm(cfg.B, device=DEV)[:5] for _ in range(2)]).reshape(1, 2, 5).to(torch.int32)
    a, al = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, sel, SCALE)
    b, bl = saap.windowed_decode_attention(q[0], Ks, Vs, off, ln, sel, -1, SCALE)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(al, bl)


@pytest.mark.parametrize("dtype,resident", [("bf16", True), ("f32", False)])
def test_recompact_index(saap, dtype, resident):
    """Slack runs out during generation; recompact_index lays the cache out afresh without re-assignment:
    state bit for bit against the oracle, attention unchanged, generation goes on."""
    S, Hq, Hkv, N, B, slack, steps = 2, 4, 2, 3000, 16, 6, 120
    n_sink, n_recent = (1, 63) if resident else (0, 0)
    W = n_sink + n_recent
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N + steps, B=B, nprobe=4, dtype=dtype, hidden=64)
    cache = gen.make_cache(cfg, 61, DEV)
    cent = gen.make_centroids(cfg, 61, DEV, cache, n_train=2048)
    _, q = gen.make_queries(cfg, 61, DEV, n_steps=2)
    x, K, V = cache["x_keys"], cache["K"], cache["V"]
    hK, hV, hx, hc = h(K), h(V), h(x), h(cent)
    ids_all = saap.assign_keys(x, cent)
    h_ids = ids_all.cpu().numpy()
    ids0, K0, V0 = (a[:, :, :N].contiguous() for a in (ids_all, K, V))
    if resident:
        off, ln, idx, Ks, Vs, res = saap.build_windowed_index(ids0, K0, V0, B, slack, n_sink, n_recent)
        want = list(ref.build_windowed_index(h_ids[:, :, :N], hK[:, :, :N], hV[:, :, :N], B, slack, n_sink, n_recent))
    else:
        off, ln, idx, Ks, Vs = saap.build_bucket_index(ids0, K0, V0, B, slack)
        want = list(ref.build_bucket_index(h_ids[:, :, :N], hK[:, :, :N], hV[:, :, :N], B, slack))

    def push(t, state, rstate):
        pos = torch.full((S,), N + t, dtype=torch.int32, device=DEV)
        xn, kn, vn = (a[:, :, N + t].contiguous() for a in (x, K, V))
        o, l, i, ks, vs = state[:5]
        if resident:
            _, flag = saap.window_push(xn, kn, vn, pos, cent, None, o, l, i, ks, vs, state[5], n_sink, n_recent)
            _, rflag = ref.window_push(hx[:, :, N + t], hK[:, :, N + t], hV[:, :, N + t], pos.cpu().numpy(), hc, None,
                                       rstate[0], rstate[1], rstate[2], rstate[3], rstate[4], rstate[5], n_sink, n_recent)
        else:
            _, flag = saap.append_keys(xn, kn, vn, pos, cent, None, o, l, i, ks, vs)
            _, rflag = ref.append_keys(hx[:, :, N + t], hK[:, :, N + t], hV[:, :, N + t], pos.cpu().numpy(), hc, None,
                                       rstate[0], rstate[1], rstate[2], rstate[3], rstate[4])
        torch.cuda.synchronize()
        assert (flag[0].item() != 0) == (rflag != 0)
        return rflag

    state = [off, ln, idx, Ks, Vs] + ([res] if resident else [])
    t = 0
    while not push(t, state, want):
        t += 1
        assert t < steps, "test sizing: the slack must run out"
    # the refused step left some heads pushed and one not: both sides are in that same state
    assert np.array_equal(ln.cpu().numpy(), want[1]) and np.array_equal(idx.cpu().numpy(), want[2])
    Ncap_new = int(want[1][..., :B].sum(axis=-1).max()) + B * 24 + W
    off2, idx2, K2, V2, flag = saap.recompact_index(off, ln, idx, Ks, Vs, 24, Ncap_new, resident=resident)
    torch.cuda.synchronize()
    r_off2, r_idx2, rK2, rV2, rflag = ref.recompact_index(want[0], want[1], want[2], want[3], want[4], 24, Ncap_new,
                                                          resident=resident)
    assert flag[0].item() == 0 and rflag == 0
    assert np.array_equal(off2.cpu().numpy(), r_off2) and np.array_equal(idx2.cpu().numpy(), r_idx2)
    live = r_idx2 >= 0
    assert np.array_equal(h(K2)[live], rK2[live]) and np.array_equal(h(V2)[live], rV2[live])
    # attention through the old and the new layout: same keys, same order inside every run -> same bits
    sel = torch.arange(3, dtype=torch.int32, device=DEV).repeat(S, Hkv, 1)
    a, al = saap.windowed_decode_attention(q[0], Ks, Vs, off, ln, sel, B if resident else -1, SCALE)
    b, bl = saap.windowed_decode_attention(q[0], K2, V2, off2, ln, sel, B if resident else -1, SCALE)
    torch.cuda.synchronize()
    assert_close(b.cpu().numpy(), a.cpu().numpy(), dtype, "attention after recompact")
    # generation goes on in the new layout
    state2 = [off2, ln, idx2, K2, V2] + ([res] if resident else [])
    want2 = [r_off2, want[1], r_idx2, rK2, rV2] + ([want[5]] if resident else [])
    for tt in range(t + 1, t + 11):
        assert push(tt, state2, want2) == 0
    assert np.array_equal(ln.cpu().numpy(), want2[1]) and np.array_equal(idx2.cpu().numpy(), want2[2])
    # a cache that cannot hold the keys is refused and nothing moves
    _, _, _, _, flag = saap.recompact_index(off2, ln, idx2, K2, V2, 24, 64, resident=resident)
    torch.cuda.synchronize()
    assert flag[0].item() == 1


def test_recompact_while_the_window_is_still_filling(saap):
    """A context shorter than the window: re-compaction keeps all W slots of the resident run, pushes go on
    in the new layout while the window fills and then slides; state bit for bit against the oracle."""
    S, Hq, Hkv, N, B, slack, n_sink, n_recent = 1, 4, 2, 20, 8, 3, 2, 30
    W = n_sink + n_recent
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N + 60, B=B, nprobe=2, hidden=64)
    cache = gen.make_cache(cfg, 89, DEV)
    cent = gen.make_centroids(cfg, 89, DEV, cache, n_train=2048)
    x, K, V = cache["x_keys"], cache["K"], cache["V"]
    hK, hV, hx, hc = h(K), h(V), h(x), h(cent)
    ids_all = saap.assign_keys(x, cent)
    h_ids = ids_all.cpu().numpy()
    state = list(saap.build_windowed_index(ids_all[:, :, :N].contiguous(), K[:, :, :N].contiguous(), V[:, :, :N].contiguous(),
                                           B, slack, n_sink, n_recent))
    want = list(ref.build_windowed_index(h_ids[:, :, :N], hK[:, :, :N], hV[:, :, :N], B, slack, n_sink, n_recent))

    def push(t):
        pos = torch.full((S,), t, dtype=torch.int32, device=DEV)
        xn, kn, vn = (a[:, :, t].contiguous() for a in (x, K, V))
        _, flag = saap.window_push(xn, kn, vn, pos, cent, None, *state, n_sink, n_recent)
        _, rflag = ref.window_push(hx[:, :, t], hK[:, :, t], hV[:, :, t], pos.cpu().numpy(), hc, None, *want, n_sink, n_recent)
        torch.cuda.synchronize()
        assert (flag[0].item(), rflag) == (0, 0), f"push {t}"

    for t in range(N, N + 5):
        push(t)
    compare_state(state, want, W, "before recompact")
    Ncap_new = B * 40 + W                                   # room for every key that the window will displace
    off2, idx2, K2, V2, flag = saap.recompact_index(state[0], state[1], state[2], state[3], state[4], 40, Ncap_new, resident=True)
    r_off2, r_idx2, rK2, rV2, rflag = ref.recompact_index(want[0], want[1], want[2], want[3], want[4], 40, Ncap_new, resident=True)
    torch.cuda.synchronize()
    assert flag[0].item() == 0 and rflag == 0
    state = [off2, state[1], idx2, K2, V2, state[5]]
    want = [r_off2, want[1], r_idx2, rK2, rV2, want[5]]
    assert int(r_off2[0, 0, B + 1] - r_off2[0, 0, B]) == W
    compare_state(state, want, W, "after recompact")
    for t in range(N + 5, N + 45):
        push(t)
    compare_state(state, want, W, "after the window filled and slid")
