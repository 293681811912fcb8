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
