"""GPU parity of bucket_attention_mass (the training target of the query model, Eq. 1) against the
oracle, which works on position-ordered keys and bucket ids and knows nothing of the sorted cache.
Tolerance: the probabilities are fp32 results of bf16 / fp32 inputs, |gpu - ref| <= 1e-6 + 2e-3 |ref|
(bf16) or 1e-7 + 1e-4 |ref| (fp32); lse within the attention tolerances."""
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


@pytest.mark.parametrize("dtype,S,Hq,Hkv,N,B", [
    ("bf16", 1, 8, 2, 6000, 37), ("bf16", 2, 4, 4, 3001, 16), ("f32", 1, 2, 1, 2500, 9), ("bf16", 1, 8, 1, 5000, 130),
    ("f32", 1, 4, 4, 900, 5),
])
def test_mass_against_the_oracle(saap, dtype, S, Hq, Hkv, N, B):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=min(4, B), dtype=dtype, hidden=64)
    cache = gen.make_cache(cfg, 71, DEV)
    cent = gen.make_centroids(cfg, 71, DEV, cache, n_train=2048)
    xq, q = gen.make_queries(cfg, 71, DEV, n_steps=2)
    ids = saap.assign_keys(cache["x_keys"], cent)
    ids[:, :, : N // 3] = torch.clamp(ids[:, :, : N // 3], max=B - 3)     # leaves the last buckets thin or empty
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, 2)
    torch.cuda.synchronize()
    atol, rtol = (1e-6, 2e-3) if dtype == "bf16" else (1e-7, 1e-4)
    for t in range(2):
        mass, lse = saap.bucket_attention_mass(q[t], Ks, off, ln, SCALE)
        torch.cuda.synchronize()
        want = ref.bucket_attention_mass(h(q[t]), h(cache["K"]), ids.cpu().numpy(), np.float32(SCALE), B)
        got = mass.cpu().numpy().astype(np.float64)
        err = np.abs(got - want)
        assert (err <= atol + rtol * want).all(), f"max err {err.max():.3e}"
        np.testing.assert_allclose(got.sum(-1), 1.0, rtol=1e-5)
        _, want_lse = ref.dense_decode_attention(h(q[t]), h(cache["K"]), h(cache["V"]), np.float32(SCALE))
        np.testing.assert_allclose(lse.cpu().numpy(), want_lse, rtol=1e-2 if dtype == "bf16" else 1e-5, atol=2e-3 if dtype == "bf16" else 1e-5)


def test_mass_of_a_selection_is_the_ratio_of_the_attention_sums(saap):
    """sum of mass over the selected buckets = exp(lse of sparse attention - lse of dense attention),
    all three from the library."""
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=2, Hq=8, Hkv=2, N=8000, B=64, nprobe=8, dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 73, DEV)
    cent = gen.make_centroids(cfg, 73, DEV, cache, n_train=4096)
    xq, q = gen.make_queries(cfg, 73, DEV, n_steps=1)
    W1, b1, W2, b2 = gen.make_classifier(cfg, 73, DEV)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, 0)
    probs = saap.classify_queries(xq[0], W1, b1, W2, b2, cfg.Hkv)
    sel = saap.select_buckets(probs, cfg.Hkv, cfg.nprobe)
    mass, lse_all = saap.bucket_attention_mass(q[0], Ks, off, ln, SCALE)
    _, lse_sel = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, sel, SCALE)
    _, lse_dense = saap.dense_decode_attention(q[0], Ks, Vs, SCALE, off=off, ln=ln)
    torch.cuda.synchronize()
    G = cfg.Hq // cfg.Hkv
    sel_q = sel.repeat_interleave(G, dim=1).to(torch.int64)                # the group's list for each of its heads
    captured = torch.gather(mass, 2, sel_q).sum(-1)
    np.testing.assert_allclose(captured.cpu().numpy(), torch.exp(lse_sel - lse_dense).cpu().numpy(), rtol=2e-3)
    np.testing.assert_allclose(lse_all.cpu().numpy(), lse_dense.cpu().numpy(), rtol=1e-5, atol=1e-5)


def test_mass_argument_checks(saap):
    q = torch.zeros(1, 4, 128, dtype=torch.bfloat16, device=DEV)
    Ks = torch.zeros(1, 1, 64, 128, dtype=torch.bfloat16, device=DEV)
    off = torch.zeros(1, 1, 3, dtype=torch.int32, device=DEV)
    ln = torch.zeros(1, 1, 2, dtype=torch.int32, device=DEV)
    mass, lse = saap.bucket_attention_mass(q, Ks, off, ln, SCALE)          # a head without keys: zeros, -inf
    assert not mass.any() and torch.isinf(lse).all()
    with pytest.raises(saap.SaapError):
        saap.bucket_attention_mass(q[:, :3], Ks, off, ln, SCALE)           # 3 heads on 1 KV head: unsupported group
    small = torch.zeros(65536 + 8, dtype=torch.uint8, device=DEV)
    with pytest.raises(saap.SaapError):
        saap.bucket_attention_mass(q, Ks, off, ln, SCALE, ws=small)


@pytest.mark.parametrize("S,Hkv,R,N,B", [(1, 2, 200, 6000, 37), (2, 1, 33, 3001, 16), (1, 1, 129, 2500, 130)])
def test_batched_mass_against_the_oracle(saap, S, Hkv, R, N, B):
    """R queries per KV head through the matrix-core kernels, against the oracle (which sees them as R heads
    sharing the KV head) and against the decode-step kernel on the first 8 of them."""
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hkv, Hkv=Hkv, N=N, B=B, nprobe=min(4, B), dtype="bf16", hidden=64)
    cache = gen.make_cache(cfg, 79, DEV)
    cent = gen.make_centroids(cfg, 79, DEV, cache, n_train=2048)
    ids = saap.assign_keys(cache["x_keys"], cent)
    ids[:, :, : N // 3] = torch.clamp(ids[:, :, : N // 3], max=B - 3)      # thin and empty buckets at the end
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], B, 2)
    g = torch.Generator(device="cpu").manual_seed(5)
    q = (2.0 * torch.randn(S, Hkv, R, 128, generator=g)).to(torch.bfloat16).to(DEV)
    mass, lse = saap.bucket_attention_mass_batch(q, Ks, off, ln, SCALE)
    torch.cuda.synchronize()
    want = ref.bucket_attention_mass(h(q).reshape(S, Hkv * R, 128), h(cache["K"]), ids.cpu().numpy(), np.float32(SCALE), B)
    got = mass.cpu().numpy().astype(np.float64).reshape(S, Hkv * R, B)
    err = np.abs(got - want)
    assert (err <= 1e-6 + 2e-3 * want).all(), f"max err {err.max():.3e}"
    np.testing.assert_allclose(got.sum(-1), 1.0, rtol=1e-5)
    m8, l8 = saap.bucket_attention_mass(q[:, :, :8].reshape(S, Hkv * 8, 128).contiguous(), Ks, off, ln, SCALE)
    torch.cuda.synchronize()
    np.testing.assert_allclose(mass[:, :, :8].cpu().numpy().reshape(S, Hkv * 8, B), m8.cpu().numpy(), rtol=2e-3, atol=1e-6)
    np.testing.assert_allclose(lse[:, :, :8].cpu().numpy().reshape(S, Hkv * 8), l8.cpu().numpy(), rtol=1e-5, atol=1e-4)
