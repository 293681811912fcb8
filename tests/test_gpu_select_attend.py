"""GPU parity of select_attend: selection and attention in one call.  The lists must equal those of
select_buckets_from_logits bit for bit (which the parity suite pins to the oracle), and the attention must meet
the oracle's sparse attention on those lists within the bf16 tolerance |gpu - ref| <= 2e-3 + 1e-2 |ref|; shapes the
one-launch kernels do not take must give the same results through the two calls."""
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


def assert_close(got, want, what, atol=2e-3, rtol=1e-2):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    fin = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), fin), f"{what}: finiteness differs"
    err = np.abs(got[fin] - want[fin])
    lim = atol + rtol * np.abs(want[fin])
    assert not (err > lim).any(), f"{what}: {(err > lim).sum()} of {err.size} outside tolerance, max err {err.max():.3e}"


@pytest.mark.parametrize("dtype,S,Hq,Hkv,N,B,nprobe,slack", [
    ("bf16", 1, 32, 8, 20000, 1024, 51, 0),       # the benchmark's shape: one launch, 2 buckets per thread
    ("bf16", 2, 8, 2, 9000, 2048, 100, 3),        # 4 buckets per thread, slack behind the buckets
    ("bf16", 1, 8, 1, 9000, 4096, 410, 0),        # eight heads, 8 buckets per thread, a long list
    ("bf16", 3, 4, 4, 3000, 64, 7, 2),            # one head per KV head, the smallest bucket count taken in one launch
    ("bf16", 1, 4, 2, 5000, 1000, 33, 0),         # a bucket count that is no power of two
    ("bf16", 1, 8, 2, 4000, 32, 6, 0),            # fewer buckets than one launch takes: the two calls
    ("bf16", 1, 8, 2, 4000, 128, 100, 0),         # a list too long for the radix selection: refused like the selection itself
    ("f32", 1, 8, 2, 3000, 256, 12, 0),           # fp32 cache: the two calls
])
def test_select_attend(saap, dtype, S, Hq, Hkv, N, B, nprobe, slack):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=nprobe, dtype=dtype, hidden=64)
    cache = gen.make_cache(cfg, 71, DEV)
    cent = gen.make_centroids(cfg, 71, DEV, cache, n_train=4096)
    _, q = gen.make_queries(cfg, 71, DEV, n_steps=3)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, slack)
    g = torch.Generator(device=DEV)
    g.manual_seed(5 * B + nprobe)
    for t in range(3):
        logits = 3 * torch.randn(S, Hq, B, generator=g, device=DEV)
        logits[:, :, B // 2] = logits[:, :, 1]                     # planted ties
        n_sort, n_pow2 = 2, 2
        while n_sort < nprobe:
            n_sort *= 2
        while n_pow2 < B:
            n_pow2 *= 2
        if not n_sort < n_pow2:
            with pytest.raises(saap.SaapError):
                saap.select_attend(logits, q[t], Ks, Vs, off, ln, nprobe, SCALE)
            return
        want_sel = saap.select_buckets_from_logits(logits, Hkv, nprobe)
        sel, out, lse = saap.select_attend(logits, q[t], Ks, Vs, off, ln, nprobe, SCALE)
        two_out, two_lse = saap.sparse_decode_attention(q[t], Ks, Vs, off, ln, want_sel, SCALE)
        torch.cuda.synchronize()
        assert torch.equal(sel, want_sel)
        r_out, r_lse = ref.sparse_decode_attention(h(q[t]), h(cache["K"]), h(cache["V"]), off.cpu().numpy(), ln.cpu().numpy(),
                                                   idx.cpu().numpy(), sel.cpu().numpy(), np.float32(SCALE), 0)
        tol = dict(atol=1e-5, rtol=1e-5) if dtype == "f32" else {}
        assert_close(out.cpu().numpy(), r_out, "out", **tol)
        assert_close(lse.cpu().numpy(), r_lse, "lse", **tol)
        # the same lists, the same dealing of the keys: the two routes agree to the last bit
        assert torch.equal(out, two_out) and torch.equal(lse, two_lse)
    # the workspace header is zero again
    ws = saap.workspace(0, DEV)
    assert int(ws[:65536].view(torch.int32).abs().sum().item()) == 0


def test_select_attend_fp8(saap):
    S, Hq, Hkv, N, B, nprobe = 1, 8, 2, 12000, 1024, 51
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=nprobe, dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 73, DEV)
    cent = gen.make_centroids(cfg, 73, DEV, cache, n_train=4096)
    _, q = gen.make_queries(cfg, 73, DEV, n_steps=1)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, 0)
    K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
    g = torch.Generator(device=DEV)
    g.manual_seed(9)
    logits = 3 * torch.randn(S, Hq, B, generator=g, device=DEV)
    want_sel = saap.select_buckets_from_logits(logits, Hkv, nprobe)
    sel, out, lse = saap.select_attend_fp8(logits, q[0], K8, V8, ks, vs, off, ln, nprobe, SCALE)
    two_out, two_lse = saap.sparse_decode_attention_fp8(q[0], K8, V8, ks, vs, off, ln, want_sel, SCALE)
    torch.cuda.synchronize()
    assert torch.equal(sel, want_sel)
    assert torch.equal(out, two_out) and torch.equal(lse, two_lse)


def test_select_attend_under_graph_replay(saap):
    """Captured once, replayed with new logits and queries in place: every replay equals the eager result."""
    S, Hq, Hkv, N, B, nprobe = 1, 32, 8, 16000, 1024, 51
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=nprobe, dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 79, DEV)
    cent = gen.make_centroids(cfg, 79, DEV, cache, n_train=4096)
    _, q = gen.make_queries(cfg, 79, DEV, n_steps=4)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, 0)
    g = torch.Generator(device=DEV)
    g.manual_seed(21)
    all_logits = [3 * torch.randn(S, Hq, B, generator=g, device=DEV) for _ in range(4)]
    logits, qq = all_logits[0].clone(), q[0].clone()
    sel = torch.empty(S, Hkv, nprobe, dtype=torch.int32, device=DEV)
    out = torch.empty(S, Hq, 128, dtype=torch.float32, device=DEV)
    lse = torch.empty(S, Hq, dtype=torch.float32, device=DEV)
    saap.select_attend(logits, qq, Ks, Vs, off, ln, nprobe, SCALE, selected=sel, out=out, lse=lse)   # workspace exists
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        saap.select_attend(logits, qq, Ks, Vs, off, ln, nprobe, SCALE, selected=sel, out=out, lse=lse)
    for t in range(4):
        logits.copy_(all_logits[t])
        qq.copy_(q[t])
        graph.replay()
        torch.cuda.synchronize()
        e_sel, e_out, e_lse = saap.select_attend(all_logits[t], q[t], Ks, Vs, off, ln, nprobe, SCALE)
        torch.cuda.synchronize()
        assert torch.equal(sel, e_sel) and torch.equal(out, e_out) and torch.equal(lse, e_lse)


@pytest.mark.parametrize("n_sink,n_recent,nprobe,B", [(1, 255, 20, 256), (4, 60, 0, 128), (1, 2047, 51, 1024)])
def test_select_attend_with_a_resident_run(saap, n_sink, n_recent, nprobe, B):
    """Over a windowed index the always-visited run is attended after the selected buckets: lists as the selection
    alone gives them, attention bit for bit as windowed_decode_attention on those lists, and within the tolerance of
    the oracle's position-based definition."""
    S, Hq, Hkv, N = 1, 8, 2, 9000
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=max(nprobe, 1), dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 83, DEV)
    cent = gen.make_centroids(cfg, 83, DEV, cache, n_train=4096)
    _, q = gen.make_queries(cfg, 83, DEV, n_steps=1)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs, res = saap.build_windowed_index(ids, cache["K"], cache["V"], B, 4, n_sink, n_recent)
    g = torch.Generator(device=DEV)
    g.manual_seed(31)
    logits = 3 * torch.randn(S, Hq, B, generator=g, device=DEV)
    sel, out, lse = saap.select_attend(logits, q[0], Ks, Vs, off, ln, nprobe, SCALE, resident_run=B)
    if nprobe > 0:
        want_sel = saap.select_buckets_from_logits(logits, Hkv, nprobe)
    else:
        want_sel = torch.empty(S, Hkv, 0, dtype=torch.int32, device=DEV)
    two_out, two_lse = saap.windowed_decode_attention(q[0], Ks, Vs, off, ln, want_sel, B, SCALE)
    torch.cuda.synchronize()
    assert torch.equal(sel, want_sel)
    assert torch.equal(out, two_out) and torch.equal(lse, two_lse)
    r_out, r_lse = ref.windowed_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), ids.cpu().numpy(), sel.cpu().numpy(),
                                                 n_sink, n_recent, np.float32(SCALE), B)
    assert_close(out.cpu().numpy(), r_out, "out")
    assert_close(lse.cpu().numpy(), r_lse, "lse")
