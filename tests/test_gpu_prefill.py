"""GPU parity of prefill-time sparse attention (one visit plan per prompt token and KV head, then the planned
attention) against the oracle's position-based definition, which knows neither index nor plans."""
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


def setup(saap, dtype, S, Hq, Hkv, Nt, B, Tq, seed, slack=0):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=Nt, B=B, nprobe=1, dtype=dtype, alpha=0.3, hidden=64)
    cache = gen.make_cache(cfg, seed, DEV)
    cent = gen.make_centroids(cfg, seed, DEV, cache, n_train=2048)
    ids = saap.assign_keys(cache["x_keys"], cent)
    index = saap.build_bucket_index(ids, cache["K"], cache["V"], B, slack)
    g = torch.Generator(device=DEV).manual_seed(seed)
    q = torch.randn(S, Tq, Hq, 128, generator=g, device=DEV).to(gen.torch_dtype(dtype))
    return cache, ids, index, q


@pytest.mark.parametrize("dtype,S,Hq,Hkv,Nt,B,Tq,nprobe,n_sink,n_recent,pos0", [
    ("bf16", 2, 8, 2, 3000, 32, 40, 4, 2, 64, (1000, 2960)),
    ("bf16", 1, 4, 1, 5000, 64, 96, 7, 1, 255, (0,)),            # the block opens the prompt: first tokens see few keys
    ("f32", 1, 2, 2, 900, 16, 24, 3, 0, 16, (700,)),
    ("bf16", 1, 8, 1, 2000, 32, 16, 5, 4, 0, (1500,)),           # G = 8, no recent window
    ("bf16", 3, 2, 2, 1200, 16, 8, 0, 1, 31, (0, 600, 1192)),    # empty lists: sink and recent keys alone
    ("bf16", 1, 4, 2, 1500, 24, 32, 24, 0, 0, (1468,)),          # every bucket listed: causal attention
])
def test_prefill_sparse_attention(saap, dtype, S, Hq, Hkv, Nt, B, Tq, nprobe, n_sink, n_recent, pos0):
    cache, ids, (off, ln, idx, Ks, Vs), q = setup(saap, dtype, S, Hq, Hkv, Nt, B, Tq, 21 + Tq, slack=1)
    rng = np.random.default_rng(Tq + nprobe)
    sel = np.stack([rng.permutation(B)[:nprobe] for _ in range(S * Hkv * Tq)]).reshape(S, Hkv, Tq, nprobe).astype(np.int32)
    p0 = np.array(pos0, dtype=np.int32)
    out, lse = saap.prefill_sparse_attention(q, cache["K"], cache["V"], Ks, Vs, off, ln, idx, torch.from_numpy(sel).to(DEV),
                                             torch.from_numpy(p0).to(DEV), n_sink, n_recent, SCALE)
    out16, _ = saap.prefill_sparse_attention(q, cache["K"], cache["V"], Ks, Vs, off, ln, idx, torch.from_numpy(sel).to(DEV),
                                             torch.from_numpy(p0).to(DEV), n_sink, n_recent, SCALE, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    ro, rl = ref.prefill_sparse_attention(h(q), h(cache["K"]), h(cache["V"]), ids.cpu().numpy(), sel, p0, n_sink, n_recent,
                                          SCALE, B)
    assert_close(out.cpu().numpy(), ro, dtype, "prefill out")
    assert_close(lse.cpu().numpy(), rl, dtype, "prefill lse")
    assert_close(out16.float().cpu().numpy(), ro, "bf16", "prefill out (bf16 store)")


def test_prefill_block_at_the_end_agrees_with_the_decode_step(saap):
    """The last token of the prompt as a block of one: the same keys as the decode-time attention with sink and recent
    keys sees on an index whose resident run holds them."""
    S, Hq, Hkv, Nt, B = 1, 8, 2, 4000, 32
    cache, ids, (off, ln, idx, Ks, Vs), q = setup(saap, "bf16", S, Hq, Hkv, Nt, B, 1, 9)
    rng = np.random.default_rng(2)
    sel = np.stack([rng.permutation(B)[:5] for _ in range(S * Hkv)]).reshape(S, Hkv, 1, 5).astype(np.int32)
    p0 = torch.full((S,), Nt - 1, dtype=torch.int32, device=DEV)
    out, lse = saap.prefill_sparse_attention(q, cache["K"], cache["V"], Ks, Vs, off, ln, idx, torch.from_numpy(sel).to(DEV), p0,
                                             2, 100, SCALE)
    w_off, w_ln, w_idx, w_Ks, w_Vs, _ = saap.build_windowed_index(ids, cache["K"], cache["V"], B, 0, 2, 100)
    wo, wl = saap.windowed_decode_attention(q[:, 0].contiguous(), w_Ks, w_Vs, w_off, w_ln,
                                            torch.from_numpy(sel[:, :, 0]).contiguous().to(DEV), B, SCALE)
    torch.cuda.synchronize()
    assert torch.allclose(out[:, 0], wo, rtol=1e-4, atol=1e-5) and torch.allclose(lse[:, 0], wl, rtol=1e-5)


def test_prefill_rejects_blocks_beyond_its_limits(saap):
    q = torch.zeros(1, 600, 32, 128, dtype=torch.bfloat16, device=DEV)         # 600 tokens * 8 KV heads > 4096 plans
    K = torch.zeros(1, 8, 700, 128, dtype=torch.bfloat16, device=DEV)
    off = torch.zeros(1, 8, 5, dtype=torch.int32, device=DEV)
    ln = torch.zeros(1, 8, 4, dtype=torch.int32, device=DEV)
    idx = torch.zeros(1, 8, 700, dtype=torch.int32, device=DEV)
    sel = torch.zeros(1, 8, 600, 2, dtype=torch.int32, device=DEV)
    with pytest.raises(saap.SaapError) as e:
        saap.prefill_sparse_attention(q, K, K, K, K, off, ln, idx, sel, torch.zeros(1, dtype=torch.int32, device=DEV), 1, 8, SCALE)
    assert e.value.status == -2
