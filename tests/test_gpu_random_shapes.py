"""Seeded sweep over odd shapes: every call of the decode path on small random configurations
(ragged N, bucket counts that are no power of two, empty buckets, G in {1,2,4,8}, both dtypes, slack,
nprobe from 0 to B, both routing modes, with and without a resident run; the attention mass per bucket; the
8-bit copy of the cache and the attention on it) against the oracle.
Integer results bit for bit, attention within the tolerances of test_gpu_parity.py."""
import math

import numpy as np
import pytest
import torch

from oracle import ref
from synth import gen

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SCALE = 1.0 / math.sqrt(128.0)
TOL = {"bf16": (2e-3, 1e-2), "f32": (1e-5, 1e-5)}


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


def close(got, want, dtype, what):
    atol, rtol = TOL[dtype]
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    fin = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), fin), f"{what}: finiteness differs"
    err = np.abs(got[fin] - want[fin])
    assert (err <= atol + rtol * np.abs(want[fin])).all(), f"{what}: max err {err.max():.3e}"


def draw(rng):
    G = int(rng.choice([1, 2, 4, 8]))
    Hkv = int(rng.choice([1, 2, 3]))
    B = int(rng.choice([16, 48, 80, 112, 208, 1008]))
    return dict(dtype=str(rng.choice(["bf16", "f32"], p=[0.7, 0.3])), S=int(rng.choice([1, 2, 3])), Hkv=Hkv, Hq=Hkv * G,
                N=int(rng.integers(1, 7000)), B=B, slack=int(rng.choice([0, 0, 1, 5])),
                nprobe=int(rng.choice([0, 1, 2, 7, B // 3, B - 1, B])), mode=int(rng.choice([0, 0, 1])),
                window=bool(rng.random() < 0.35), hidden=int(rng.choice([32, 96, 160])))


@pytest.mark.parametrize("case", range(96))
def test_random_shape(saap, case):
    rng = np.random.default_rng(1000 + case)
    c = draw(rng)
    dtype, S, Hq, Hkv, N, B, slack, nprobe, mode = (c[k] for k in ("dtype", "S", "Hq", "Hkv", "N", "B", "slack", "nprobe", "mode"))
    print(c, flush=True)
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=max(nprobe, 1), dtype=dtype,
                                                   hidden=c["hidden"], alpha=0.3)
    cache = gen.make_cache(cfg, case, DEV)
    cent = gen.make_centroids(cfg, case, DEV, cache, n_train=max(B, 1024))
    xq, q = gen.make_queries(cfg, case, DEV)
    W1, b1, W2, b2 = gen.make_classifier(cfg, case, DEV)
    x, K, V = cache["x_keys"], cache["K"], cache["V"]
    hK, hV = h(K), h(V)

    ids = saap.assign_keys(x, cent)
    torch.cuda.synchronize()
    r_ids = ref.assign_keys(h(x), h(cent))
    assert np.array_equal(ids.cpu().numpy(), r_ids), "bucket ids"

    n_sink, n_recent = (int(rng.integers(0, 5)), int(rng.integers(1, 200))) if c["window"] else (0, 0)
    if c["window"]:
        off, ln, idx, Ks, Vs, res = saap.build_windowed_index(ids, K, V, B, slack, n_sink, n_recent)
        want = ref.build_windowed_index(r_ids, hK, hV, B, slack, n_sink, n_recent)
        r_res = want[5]
    else:
        off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, K, V, B, slack)
        want = ref.build_bucket_index(r_ids, hK, hV, B, slack)
    torch.cuda.synchronize()
    r_off, r_ln, r_idx = want[0], want[1], want[2]
    assert np.array_equal(off.cpu().numpy(), r_off) and np.array_equal(ln.cpu().numpy(), r_ln), "off / len"
    assert np.array_equal(idx.cpu().numpy(), r_idx), "idx"
    if c["window"]:
        assert np.array_equal(res.cpu().numpy(), r_res), "resident ids"
    live = r_idx >= 0
    assert np.array_equal(h(Ks)[live], want[3][live]) and np.array_equal(h(Vs)[live], want[4][live]), "sorted rows"

    logits = saap.classify_queries(xq[0], W1, b1, W2, b2, Hkv, output_kind=saap.LOGITS)
    probs = saap.classify_queries(xq[0], W1, b1, W2, b2, Hkv)
    torch.cuda.synchronize()
    np.testing.assert_allclose(logits.cpu().numpy(), ref.classify_queries(h(xq[0]), h(W1), h(b1), h(W2), h(b2), Hkv, output_kind=1),
                               rtol=2e-5, atol=5e-5)
    sel = saap.select_buckets(probs, Hkv, nprobe, mode)
    torch.cuda.synchronize()
    r_sel = ref.select_buckets(probs.cpu().numpy(), Hkv, nprobe, mode)
    if nprobe > 0:
        assert np.array_equal(sel.cpu().numpy(), r_sel), "selected"
    d_sel = torch.from_numpy(r_sel).to(DEV)

    resident = B if c["window"] else -1
    out, lse = saap.windowed_decode_attention(q[0], Ks, Vs, off, ln, d_sel, resident, SCALE, mode=mode)
    torch.cuda.synchronize()
    if c["window"]:
        ro, rl = ref.windowed_decode_attention(h(q[0]), hK, hV, r_ids, r_sel, n_sink, n_recent, SCALE, B, mode=mode)
    else:
        ro, rl = ref.sparse_decode_attention(h(q[0]), hK, hV, r_off, r_ln, r_idx, r_sel, SCALE, mode=mode)
    close(out.cpu().numpy(), ro, dtype, "attention out")
    close(lse.cpu().numpy(), rl, dtype, "attention lse")

    # selection and attention in one call: the lists of the selection from logits, the attention of the separate
    # call on those lists to the last bit (group lists only; a list as long as the padded bucket count is refused
    # like the selection from logits itself)
    n_sort, n_pow2 = 2, 2
    while n_sort < nprobe:
        n_sort *= 2
    while n_pow2 < B:
        n_pow2 *= 2
    if mode == 0 and 0 < nprobe and n_sort < n_pow2:
        want_sel = saap.select_buckets_from_logits(logits, Hkv, nprobe)
        two_out, two_lse = saap.windowed_decode_attention(q[0], Ks, Vs, off, ln, want_sel, resident, SCALE)
        sa_sel, sa_out, sa_lse = saap.select_attend(logits, q[0], Ks, Vs, off, ln, nprobe, SCALE, resident_run=resident)
        torch.cuda.synchronize()
        assert torch.equal(sa_sel, want_sel), "select_attend lists"
        assert torch.equal(sa_out, two_out) and torch.equal(sa_lse, two_lse), "select_attend attention"

    # the attention mass per bucket (plain index only: the resident run is no bucket)
    if not c["window"]:
        mass, mlse = saap.bucket_attention_mass(q[0], Ks, off, ln, SCALE)
        torch.cuda.synchronize()
        r_mass = ref.bucket_attention_mass(h(q[0]), hK, r_ids, np.float32(SCALE), B)
        atol, rtol = (1e-6, 2e-3) if dtype == "bf16" else (1e-7, 1e-4)
        err = np.abs(mass.cpu().numpy() - r_mass)
        assert (err <= atol + rtol * r_mass).all(), f"bucket mass: max err {err.max():.3e}"

    # the same attention on the 8-bit copy of the cache, against the oracle on the decoded values
    if dtype == "bf16":
        K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
        torch.cuda.synchronize()
        # free slots of the sorted cache hold zeros, so the scales are those of the position-ordered tensors
        rK8, rks = ref.quantize_fp8(hK)
        rV8, rvs = ref.quantize_fp8(hV)
        assert np.array_equal(ks.cpu().numpy(), rks) and np.array_equal(vs.cpu().numpy(), rvs), "8-bit scales"
        for s_ in range(S):
            for hh in range(Hkv):
                m = r_idx[s_, hh] >= 0
                assert np.array_equal(K8.cpu().numpy()[s_, hh][m], rK8[s_, hh][r_idx[s_, hh][m]]), "K codes"
                assert np.array_equal(V8.cpu().numpy()[s_, hh][m], rV8[s_, hh][r_idx[s_, hh][m]]), "V codes"
        Kd, Vd = ref.dequantize_fp8(rK8, rks), ref.dequantize_fp8(rV8, rvs)
        out8, lse8 = saap.windowed_decode_attention_fp8(q[0], K8, V8, ks, vs, off, ln, d_sel, resident, SCALE, mode=mode)
        torch.cuda.synchronize()
        if c["window"]:
            ro, rl = ref.windowed_decode_attention(h(q[0]), Kd, Vd, r_ids, r_sel, n_sink, n_recent, SCALE, B, mode=mode)
        else:
            ro, rl = ref.sparse_decode_attention(h(q[0]), Kd, Vd, r_off, r_ln, r_idx, r_sel, SCALE, mode=mode)
        close(out8.cpu().numpy(), ro, dtype, "8-bit attention out")
        close(lse8.cpu().numpy(), rl, dtype, "8-bit attention lse")
