"""GPU parity of the 8-bit K/V path: quantize_kv bit for bit against the oracle's encoder (codes and
scales), and the attention calls on the 8-bit cache against the oracle's attention on the decoded
values, within the bf16 tolerance |gpu - ref| <= 2e-3 + 1e-2 |ref| (bf16 queries, fp32 accumulation;
the decoded values are exact, so the tolerance covers the arithmetic only)."""
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


def assert_close(got, want, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    fin = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), fin), f"{what}: finiteness differs"
    err = np.abs(got[fin] - want[fin])
    lim = 2e-3 + 1e-2 * np.abs(want[fin])
    assert not (err > lim).any(), f"{what}: {(err > lim).sum()} of {err.size} outside tolerance, max err {err.max():.3e}"


def position_order(sorted_rows, idx):
    """Rows of a bucket-sorted array [S,Hkv,Ncap,d] back in position order [S,Hkv,N,d] (the oracle's
    attention reads keys by position through idx)."""
    S, Hkv, Ncap, d = sorted_rows.shape
    N = int(idx.max()) + 1
    out = np.zeros((S, Hkv, N, d), dtype=sorted_rows.dtype)
    for s in range(S):
        for hh in range(Hkv):
            m = idx[s, hh] >= 0
            out[s, hh, idx[s, hh][m]] = sorted_rows[s, hh][m]
    return out


def test_code_table_of_the_device(saap):
    """Every E4M3 code decoded by the attention kernel's conversion equals the oracle's table: one key
    per code, attended alone through a one-bucket list, value row = the code in every feature."""
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    n = len(codes)
    V8 = torch.from_numpy(np.repeat(codes[:, None], 128, axis=1).reshape(1, 1, n, 128).copy()).to(DEV)
    K8 = torch.zeros_like(V8)
    ks = torch.ones(1, 1, dtype=torch.float32, device=DEV)
    vs = torch.full((1, 1), 0.5, dtype=torch.float32, device=DEV)
    off = torch.arange(n + 1, dtype=torch.int32, device=DEV).reshape(1, 1, n + 1)
    ln = torch.ones(1, 1, n, dtype=torch.int32, device=DEV)
    q = torch.zeros(1, 1, 128, dtype=torch.bfloat16, device=DEV)
    table = np.array([ref.fp8_e4m3_decode(int(c)) for c in codes], dtype=np.float64)
    got = np.empty(n)
    for i in range(n):
        sel = torch.tensor([[[i]]], dtype=torch.int32, device=DEV)
        out, _ = saap.sparse_decode_attention_fp8(q, K8, V8, ks, vs, off, ln, sel, SCALE)
        o = out.cpu().numpy()[0, 0]
        assert (o == o[0]).all()
        got[i] = o[0]
    assert np.array_equal(got, 0.5 * table)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_quantize_kv_bit_exact(saap, dtype):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=2, Hq=4, Hkv=2, N=3000, B=16, nprobe=4, dtype=dtype)
    cache = gen.make_cache(cfg, 41, DEV)
    K, V = cache["K"].clone(), cache["V"].clone()
    # planted cases: exact ties between neighbouring codes, values below the smallest subnormal,
    # zeros of both signs, the unit maximum on a power-of-two boundary, an all-zero unit
    V[1, 1] = 0
    K[0, 0, 0, :8] = torch.tensor([448.0, -448.0, 0.0, -0.0, 1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10]).to(K.dtype)
    K[0, 0].clamp_(-448.0, 448.0)
    K[0, 0, 1, :4] = torch.tensor([2.0 ** -11, -(2.0 ** -11), 2.0 ** -9, 9 * 2.0 ** -10]).to(K.dtype)
    K8, V8, ks, vs = saap.quantize_kv(K, V)
    torch.cuda.synchronize()
    rK8, rks = ref.quantize_fp8(h(K))
    rV8, rvs = ref.quantize_fp8(h(V))
    assert np.array_equal(ks.cpu().numpy(), rks) and np.array_equal(vs.cpu().numpy(), rvs)
    assert float(ks[0, 0]) == 1.0
    for name, got, want in (("K", K8.cpu().numpy(), rK8), ("V", V8.cpu().numpy(), rV8)):
        diff = got != want
        assert not diff.any(), f"{name}: {diff.sum()} codes differ, first at {np.argwhere(diff)[0]}: {got[diff][0]:#x} vs {want[diff][0]:#x}"
    # the workspace header is zero again
    ws = saap.workspace(0, DEV)
    assert int(ws[:65536].view(torch.int32).abs().sum().item()) == 0


@pytest.mark.parametrize("S,Hq,Hkv,N,B,nprobe,mode", [
    (1, 8, 2, 5000, 32, 6, 0), (2, 4, 4, 3001, 16, 16, 0), (1, 8, 1, 4000, 64, 9, 0), (1, 4, 2, 2500, 16, 3, 1),
    (1, 2, 1, 777, 8, 0, 0),
])
def test_sparse_attention_fp8(saap, S, Hq, Hkv, N, B, nprobe, mode):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=nprobe, dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 43, DEV)
    cent = gen.make_centroids(cfg, 43, DEV, cache, n_train=2048)
    xq, q = gen.make_queries(cfg, 43, DEV, n_steps=3)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, 3)
    K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
    torch.cuda.synchronize()
    h_idx = idx.cpu().numpy()
    Kp = position_order(ref.dequantize_fp8(K8.cpu().numpy(), ks.cpu().numpy()), h_idx)
    Vp = position_order(ref.dequantize_fp8(V8.cpu().numpy(), vs.cpu().numpy()), h_idx)
    rng = np.random.default_rng(7)
    lists = Hq if mode == 1 else Hkv
    for t in range(3):
        sel_np = np.stack([np.stack([rng.permutation(B)[:nprobe] for _ in range(lists)]) for _ in range(S)]).astype(np.int32)
        sel = torch.from_numpy(sel_np).to(DEV)
        out, lse = saap.sparse_decode_attention_fp8(q[t], K8, V8, ks, vs, off, ln, sel, SCALE, mode=mode)
        torch.cuda.synchronize()
        r_out, r_lse = ref.sparse_decode_attention(h(q[t]), Kp, Vp, off.cpu().numpy(), ln.cpu().numpy(), h_idx, sel_np,
                                                   np.float32(SCALE), mode)
        assert_close(out.cpu().numpy(), r_out, "out")
        assert_close(lse.cpu().numpy(), r_lse, "lse")


def test_sparse_attention_fp8_query_ranges(saap):
    """Groups of four heads take their scores on the matrix cores, where the bf16 query row is scaled by a power of
    two and split into two rows of 8-bit codes: rows of zeros, tiny and huge rows, and a row whose elements span
    twenty binades must all come out within the tolerance."""
    S, Hq, Hkv, N, B, nprobe = 1, 8, 2, 6000, 32, 8
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=nprobe, dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 53, DEV)
    cent = gen.make_centroids(cfg, 53, DEV, cache, n_train=2048)
    xq, q = gen.make_queries(cfg, 53, DEV, n_steps=1)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, 3)
    K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
    qq = q[0].clone().float()                                    # [S, Hq, d]
    g = torch.Generator(device="cpu").manual_seed(5)
    qq[0, 0] = 0.0                                               # nothing to scale
    qq[0, 1] *= 1e-30                                            # below the range that is scaled
    qq[0, 2] *= 3e4                                              # scores in the thousands: one key takes all
    qq[0, 3] *= torch.exp2(-20.0 * torch.rand(128, generator=g)).to(DEV)     # elements from 1 down to 2^-20 of the largest
    qq[0, 5] = 0.0
    qq[0, 5, 17] = 1.0                                           # a single feature
    qq[0, 6] *= 2.0 ** -100
    qb = qq.to(torch.bfloat16)
    torch.cuda.synchronize()
    h_idx = idx.cpu().numpy()
    Kp = position_order(ref.dequantize_fp8(K8.cpu().numpy(), ks.cpu().numpy()), h_idx)
    Vp = position_order(ref.dequantize_fp8(V8.cpu().numpy(), vs.cpu().numpy()), h_idx)
    rng = np.random.default_rng(11)
    sel_np = np.stack([np.stack([rng.permutation(B)[:nprobe] for _ in range(Hkv)]) for _ in range(S)]).astype(np.int32)
    sel = torch.from_numpy(sel_np).to(DEV)
    out, lse = saap.sparse_decode_attention_fp8(qb, K8, V8, ks, vs, off, ln, sel, SCALE)
    torch.cuda.synchronize()
    r_out, r_lse = ref.sparse_decode_attention(h(qb), Kp, Vp, off.cpu().numpy(), ln.cpu().numpy(), h_idx, sel_np,
                                               np.float32(SCALE), 0)
    assert_close(out.cpu().numpy(), r_out, "out")
    assert_close(lse.cpu().numpy(), r_lse, "lse")


def test_dense_attention_fp8_and_all_buckets(saap):
    """Dense attention on the 8-bit cache, packed and bucket-sorted, and the sparse call with every
    bucket selected: all equal the oracle's dense attention on the decoded values."""
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=1, Hq=8, Hkv=2, N=6000, B=24, nprobe=24, dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 47, DEV)
    cent = gen.make_centroids(cfg, 47, DEV, cache, n_train=2048)
    xq, q = gen.make_queries(cfg, 47, DEV, n_steps=1)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, 2)
    K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
    P8, PV8, pks, pvs = saap.quantize_kv(cache["K"], cache["V"])          # the packed cache, position order
    torch.cuda.synchronize()
    h_idx = idx.cpu().numpy()
    Kp = position_order(ref.dequantize_fp8(K8.cpu().numpy(), ks.cpu().numpy()), h_idx)
    Vp = position_order(ref.dequantize_fp8(V8.cpu().numpy(), vs.cpu().numpy()), h_idx)
    r_out, r_lse = ref.dense_decode_attention(h(q[0]), Kp, Vp, np.float32(SCALE))
    out, lse = saap.dense_decode_attention_fp8(q[0], K8, V8, ks, vs, SCALE, off=off, ln=ln)
    assert_close(out.cpu().numpy(), r_out, "dense sorted out")
    assert_close(lse.cpu().numpy(), r_lse, "dense sorted lse")
    sel = torch.arange(cfg.B, dtype=torch.int32, device=DEV).repeat(1, cfg.Hkv, 1)
    out, lse = saap.sparse_decode_attention_fp8(q[0], K8, V8, ks, vs, off, ln, sel, SCALE)
    assert_close(out.cpu().numpy(), r_out, "all buckets out")
    assert_close(lse.cpu().numpy(), r_lse, "all buckets lse")
    # packed cache: the same keys in position order (the scales are those of the same values)
    assert torch.equal(pks, ks) and torch.equal(pvs, vs)
    out, lse = saap.dense_decode_attention_fp8(q[0], P8, PV8, pks, pvs, SCALE)
    assert_close(out.cpu().numpy(), r_out, "dense packed out")
    assert_close(lse.cpu().numpy(), r_lse, "dense packed lse")


def test_fp8_argument_checks(saap):
    q = torch.zeros(1, 4, 128, dtype=torch.bfloat16, device=DEV)
    K8 = torch.zeros(1, 1, 64, 128, dtype=torch.uint8, device=DEV)
    ks = torch.ones(1, 1, dtype=torch.float32, device=DEV)
    off = torch.zeros(1, 1, 3, dtype=torch.int32, device=DEV)
    ln = torch.zeros(1, 1, 2, dtype=torch.int32, device=DEV)
    sel = torch.zeros(1, 1, 1, dtype=torch.int32, device=DEV)
    with pytest.raises(TypeError):
        saap.sparse_decode_attention_fp8(q.float(), K8, K8, ks, ks, off, ln, sel, SCALE)
    with pytest.raises(saap.SaapError):
        saap.sparse_decode_attention_fp8(q, K8, K8, None, ks, off, ln, sel, SCALE)
    # the 16-bit entry point does not take the internal code of the 8-bit cache
    lib = saap.load_library()
    import ctypes
    ws = saap.workspace(1 << 20, DEV)
    out = torch.zeros(1, 4, 128, dtype=torch.float32, device=DEV)
    st = lib.saap_sparse_decode_attention(
        ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(K8.data_ptr()), ctypes.c_void_p(K8.data_ptr()),
        ctypes.c_void_p(off.data_ptr()), ctypes.c_void_p(ln.data_ptr()), ctypes.c_void_p(sel.data_ptr()), 1, 0,
        ctypes.c_float(SCALE), ctypes.c_void_p(out.data_ptr()), 0, ctypes.c_void_p(0), 1, 4, 1, 64, 2, 128, 2,
        ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel()), ctypes.c_void_p(0))
    assert st != 0


@pytest.mark.parametrize("n_sink,n_recent,nprobe", [(1, 255, 5), (4, 60, 0), (0, 64, 16)])
def test_windowed_attention_fp8(saap, n_sink, n_recent, nprobe):
    """The always-visited run (attention sink + recent keys) on the 8-bit cache, against the oracle's
    position-based definition on the decoded values."""
    S, Hq, Hkv, N, B = 1, 8, 2, 5000, 16
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=max(nprobe, 1), dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 53, DEV)
    cent = gen.make_centroids(cfg, 53, DEV, cache, n_train=2048)
    _, q = gen.make_queries(cfg, 53, DEV, n_steps=2)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs, res = saap.build_windowed_index(ids, cache["K"], cache["V"], B, 4, n_sink, n_recent)
    K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
    torch.cuda.synchronize()
    h_idx = idx.cpu().numpy()
    Kp = position_order(ref.dequantize_fp8(K8.cpu().numpy(), ks.cpu().numpy()), h_idx)
    Vp = position_order(ref.dequantize_fp8(V8.cpu().numpy(), vs.cpu().numpy()), h_idx)
    assert Kp.shape[2] == N
    rng = np.random.default_rng(3)
    for t in range(2):
        sel_np = np.stack([np.stack([rng.permutation(B)[:nprobe] for _ in range(Hkv)]) for _ in range(S)]).astype(np.int32)
        sel_np = sel_np.reshape(S, Hkv, nprobe)
        out, lse = saap.windowed_decode_attention_fp8(q[t], K8, V8, ks, vs, off, ln, torch.from_numpy(sel_np).to(DEV), B, SCALE)
        torch.cuda.synchronize()
        ro, rl = ref.windowed_decode_attention(h(q[t]), Kp, Vp, ids.cpu().numpy(), sel_np, n_sink, n_recent, np.float32(SCALE), B)
        assert_close(out.cpu().numpy(), ro, "out")
        assert_close(lse.cpu().numpy(), rl, "lse")


def _live(off, ln, idx):
    """Boolean mask [S,Hkv,Ncap] of the slots that hold a key."""
    live = np.zeros(idx.shape, dtype=bool)
    S, Hkv, _ = idx.shape
    for s in range(S):
        for u in range(Hkv):
            for b in range(ln.shape[2]):
                live[s, u, off[s, u, b]:off[s, u, b] + ln[s, u, b]] = True
    return live & (idx >= 0)


def _oracle_scales(rKs, rVs, live):
    """Scales of a cache as quantize_kv fixes them: free slots hold zeros."""
    rKs = np.where(live[..., None], rKs, 0).astype(np.float32)
    rVs = np.where(live[..., None], rVs, 0).astype(np.float32)
    return ref.quantize_fp8(rKs)[1], ref.quantize_fp8(rVs)[1]


def _as_stored(x, scale):
    """Values a row has once it is in the 8-bit cache: decoded codes of x / scale (saturated)."""
    return ref.dequantize_fp8(ref.quantize_fp8_scaled(x, scale), scale)


@pytest.mark.parametrize("S,Hkv,N,B,slack,n_sink,n_recent,steps", [
    (2, 2, 3000, 16, 100, 1, 63, 150),                     # the ring wraps twice: displaced rows move as bytes
    (1, 2, 2100, 16, 16, 3, 0, 20),                        # no ring: new rows go straight to their buckets
    (1, 1, 40, 8, 64, 2, 100, 130),                        # the window fills first, then slides
])
def test_window_push_fp8(saap, S, Hkv, N, B, slack, n_sink, n_recent, steps):
    """Generation on an 8-bit cache: index state bit for bit, stored codes bit for bit against the oracle's
    encoder with the cache's scales, attention on the grown cache against the oracle on the decoded values."""
    Hq = 2 * Hkv
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N + steps, B=B, nprobe=4, dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 67, DEV)
    cent = gen.make_centroids(cfg, 67, DEV, cache, n_train=2048)
    _, q = gen.make_queries(cfg, 67, DEV, n_steps=3)
    x, K, V = cache["x_keys"], cache["K"].clone(), cache["V"].clone()
    # two later rows leave the range that the prefill keys fixed: their features saturate at +-448 * scale
    K[0, 0, N + 5, :4] = torch.tensor([3e4, -3e4, 1e30, -1e30]).to(K.dtype)
    V[0, 0, N + 7, 9] = -5e4
    ids_all = saap.assign_keys(x, cent)
    ids0, K0, V0 = (a[:, :, :N].contiguous() for a in (ids_all, K, V))
    off, ln, idx, Ks, Vs, res = saap.build_windowed_index(ids0, K0, V0, B, slack, n_sink, n_recent)
    K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
    torch.cuda.synchronize()
    # the oracle's side, from the inputs alone
    h_ids, hK, hV, hx, hc = ids_all.cpu().numpy(), h(K), h(V), h(x), h(cent)
    assert np.array_equal(h_ids, ref.assign_keys(hx, hc))
    r0 = ref.build_windowed_index(h_ids[:, :, :N], hK[:, :, :N], hV[:, :, :N], B, slack, n_sink, n_recent)
    rks, rvs = _oracle_scales(r0[3], r0[4], _live(r0[0], r0[1], r0[2]))
    assert np.array_equal(ks.cpu().numpy(), rks) and np.array_equal(vs.cpu().numpy(), rvs)
    Kq, Vq = _as_stored(hK, rks), _as_stored(hV, rvs)      # every position as the cache will hold it
    want = list(ref.build_windowed_index(h_ids[:, :, :N], Kq[:, :, :N], Vq[:, :, :N], B, slack, n_sink, n_recent))

    def compare(what):
        torch.cuda.synchronize()
        for name, got, exp in (("off", off, want[0]), ("len", ln, want[1]), ("idx", idx, want[2]), ("resident", res, want[5])):
            assert np.array_equal(got.cpu().numpy(), exp), f"{what}: {name}"
        live = _live(want[0], want[1], want[2])
        for name, got, exp, sc in (("K", K8, want[3], rks), ("V", V8, want[4], rvs)):
            codes = ref.quantize_fp8_scaled(exp, sc)        # exact: the oracle's rows are decoded codes
            assert np.array_equal(ref.dequantize_fp8(codes, sc)[live], exp[live])
            assert np.array_equal(got.cpu().numpy()[live], codes[live]), f"{what}: {name} codes"

    compare("after build")
    flag = torch.zeros(4, dtype=torch.int32, device=DEV)
    rng = np.random.default_rng(5)
    check_at = {0, 5, 7, 8, steps // 2, steps - 1}
    for t in range(steps):
        pos = torch.full((S,), N + t, dtype=torch.int32, device=DEV)
        xn, kn, vn = (a[:, :, N + t].contiguous() for a in (x, K, V))
        nid, _ = saap.window_push_fp8(xn, kn, vn, pos, cent, None, off, ln, idx, K8, V8, ks, vs, res, n_sink, n_recent,
                                      overflow_flag=flag)
        rid, rflag = ref.window_push(hx[:, :, N + t], Kq[:, :, N + t], Vq[:, :, N + t], pos.cpu().numpy(), hc, None,
                                     want[0], want[1], want[2], want[3], want[4], want[5], n_sink, n_recent)
        assert rflag == 0, "test sizing: slack must absorb every displaced key"
        if t in check_at:
            compare(f"after push {t}")
            assert np.array_equal(nid.cpu().numpy(), rid)
            Nt = N + t + 1
            for nprobe in (0, 4, B):
                sel = np.stack([np.stack([rng.permutation(B)[:nprobe] for _ in range(Hkv)]) for _ in range(S)]).astype(np.int32)
                sel = sel.reshape(S, Hkv, nprobe)
                out, lse = saap.windowed_decode_attention_fp8(q[t % 3], K8, V8, ks, vs, off, ln, torch.from_numpy(sel).to(DEV),
                                                              B, SCALE)
                torch.cuda.synchronize()
                ro, rl = ref.windowed_decode_attention(h(q[t % 3]), Kq[:, :, :Nt], Vq[:, :, :Nt], h_ids[:, :, :Nt], sel,
                                                       n_sink, n_recent, np.float32(SCALE), B)
                assert_close(out.cpu().numpy(), ro, f"push {t} nprobe {nprobe} out")
                assert_close(lse.cpu().numpy(), rl, f"push {t} nprobe {nprobe} lse")
    torch.cuda.synchronize()
    assert flag[0].item() == 0
    # the planted rows did saturate
    assert float(np.abs(Kq[0, 0, N + 5, :4]).max()) == 448.0 * float(rks[0, 0])
    assert float(Vq[0, 0, N + 7, 9]) == -448.0 * float(rvs[0, 0])


def test_append_keys_fp8(saap):
    """The index without a resident run: appended rows, their codes, and the overflow flag once a bucket's
    slack has run out (nothing changes for that unit then)."""
    S, Hkv, N, B, slack, steps = 2, 2, 2000, 32, 2, 6
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=8, Hkv=Hkv, N=N, B=B, nprobe=B, dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 71, DEV)
    cent = gen.make_centroids(cfg, 71, DEV, cache, n_train=2048)
    _, q = gen.make_queries(cfg, 71, DEV)
    new = gen.make_cache(cfg.replace(N=steps), 73, DEV)
    new["x_keys"][0, 0, :] = (4.0 * cent[0, 3].float()).to(new["x_keys"].dtype)   # one bucket takes every new key of unit (0,0)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, slack)
    K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
    torch.cuda.synchronize()
    h_ids = ids.cpu().numpy()
    hK, hV = h(cache["K"]), h(cache["V"])
    r0 = ref.build_bucket_index(h_ids, hK, hV, B, slack)
    rks, rvs = _oracle_scales(r0[3], r0[4], _live(r0[0], r0[1], r0[2]))
    assert np.array_equal(ks.cpu().numpy(), rks) and np.array_equal(vs.cpu().numpy(), rvs)
    Kq, Vq = _as_stored(hK, rks), _as_stored(hV, rvs)
    nKq, nVq = _as_stored(h(new["K"]), rks), _as_stored(h(new["V"]), rvs)
    r_off, r_ln, r_idx, rKs, rVs = ref.build_bucket_index(h_ids, Kq, Vq, B, slack)
    flags = []
    for t in range(steps):
        pos = torch.full((S,), N + t, dtype=torch.int32, device=DEV)
        xn, kn, vn = (new[k][:, :, t].contiguous() for k in ("x_keys", "K", "V"))
        nid, flag = saap.append_keys_fp8(xn, kn, vn, pos, cent, None, off, ln, idx, K8, V8, ks, vs)
        torch.cuda.synchronize()
        rid, rflag = ref.append_keys(h(xn), nKq[:, :, t], nVq[:, :, t], pos.cpu().numpy(), h(cent), None, r_off, r_ln, r_idx,
                                     rKs, rVs)
        flags.append(rflag)
        assert np.array_equal(nid.cpu().numpy(), rid)
        assert (flag[0].item() != 0) == (rflag != 0)
        assert np.array_equal(ln.cpu().numpy(), r_ln) and np.array_equal(idx.cpu().numpy(), r_idx)
    assert flags[0] == 0 and flags[-1] == 1
    live = _live(r_off, r_ln, r_idx)
    assert np.array_equal(K8.cpu().numpy()[live], ref.quantize_fp8_scaled(rKs, rks)[live])
    assert np.array_equal(V8.cpu().numpy()[live], ref.quantize_fp8_scaled(rVs, rvs)[live])
    # attention over every bucket of the grown cache
    sel = torch.arange(B, dtype=torch.int32, device=DEV).repeat(S, Hkv, 1)
    out, lse = saap.sparse_decode_attention_fp8(q[0], K8, V8, ks, vs, off, ln, sel, SCALE)
    torch.cuda.synchronize()
    Kall = position_order(rKs, r_idx)
    Vall = position_order(rVs, r_idx)
    ro, rl = ref.sparse_decode_attention(h(q[0]), Kall, Vall, r_off, r_ln, r_idx, sel.cpu().numpy(), SCALE)
    assert_close(out.cpu().numpy(), ro, "attention after append")
    assert_close(lse.cpu().numpy(), rl, "lse after append")
