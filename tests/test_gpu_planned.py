"""GPU parity of the visit-plan path: the selection writes the attention's work list and the attention
deals the keys of ALL lists to the workgroups in equal shares.  The plan is compared bit for bit with the
one numpy builds from the oracle's index and lists; the attention element by element with the oracle's
restricted softmax (which knows neither plans nor workgroups), with units of wildly unequal sizes."""
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


def plan_by_hand(sel, off, ln, G_lists, resident=-1):
    """The documented plan layout written out with numpy: sel [S,lists,nprobe], off/ln per (sequence, KV head);
    G_lists = lists per KV head (1 for group lists)."""
    S, lists, nprobe = sel.shape
    nruns = nprobe + (1 if resident >= 0 else 0)
    ps = (2 * nruns + 2 + 3) // 4 * 4
    plan = np.zeros((S * lists, ps), dtype=np.int32)
    for s in range(S):
        for li in range(lists):
            hk = li // G_lists
            runs = list(sel[s, li]) + ([resident] if resident >= 0 else [])
            lens = np.array([ln[s, hk, b] for b in runs], dtype=np.int64)
            row = plan[s * lists + li]
            row[0] = lens.sum()
            row[1] = 0
            row[2:2 + nruns] = np.cumsum(lens)
            row[nruns + 2:2 * nruns + 2] = [off[s, hk, b] for b in runs]
    return plan, ps, nruns


def used_part(plan_flat, units, ps, nruns):
    """Entries of a device plan that the layout defines (the stride's padding is unspecified)."""
    return plan_flat[:units * ps].reshape(units, ps)[:, :2 * nruns + 2]


def make_index(saap, cfg, seed, slack=0):
    cache = gen.make_cache(cfg, seed, DEV)
    cent = gen.make_centroids(cfg, seed, DEV, cache, n_train=min(8192, max(4 * cfg.B, 2048)))
    ids = saap.assign_keys(cache["x_keys"], cent)
    index = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, slack)
    cache["ids"] = ids
    return cache, index


# ------------------------------------------------------------------------------ the plan itself
@pytest.mark.parametrize("S,Hq,Hkv,B,nprobe,mode,kind", [
    (1, 32, 8, 1024, 51, 0, "logits"), (2, 8, 2, 4096, 410, 0, "logits"), (1, 1, 1, 64, 8, 0, "probs"),
    (1, 8, 2, 100, 100, 0, "probs"), (2, 8, 2, 300, 17, 1, "logits"), (1, 4, 1, 8192, 1, 0, "probs"),
    (1, 4, 4, 48, 5, 0, "logits"), (3, 16, 2, 2048, 700, 0, "logits"), (1, 4, 2, 96, 0, 0, "probs"),
    (1, 8, 2, 4096, 2100, 0, "probs"),
])
def test_select_buckets_planned(saap, S, Hq, Hkv, B, nprobe, mode, kind):
    """Lists equal to the oracle's selection bit for bit (same fp32 scores), plan equal to the hand-made one."""
    rng = np.random.default_rng(B * 31 + nprobe)
    logits = (rng.standard_normal((S, Hq, B)) * 3).astype(np.float32)
    ln = rng.integers(0, 300, size=(S, Hkv, B)).astype(np.int32)
    ln[:, :, ::5] = 0
    off = np.zeros((S, Hkv, B + 1), dtype=np.int32)
    off[:, :, 1:] = np.cumsum(ln + 2, axis=2)
    d_off, d_ln = torch.from_numpy(off).to(DEV), torch.from_numpy(ln).to(DEV)
    if kind == "logits":
        probs = torch.empty(S, Hq, B, dtype=torch.float32, device=DEV)
        sel, plan = saap.select_buckets_planned(torch.from_numpy(logits).to(DEV), d_off, d_ln, Hkv, nprobe,
                                                input_kind=saap.LOGITS, mode=mode, probs=probs)
        torch.cuda.synchronize()
        scores = probs.cpu().numpy() if nprobe > 0 else logits
    else:
        e = np.exp(logits - logits.max(-1, keepdims=True))
        scores = (e / e.sum(-1, keepdims=True)).astype(np.float32)
        sel, plan = saap.select_buckets_planned(torch.from_numpy(scores).to(DEV), d_off, d_ln, Hkv, nprobe, mode=mode)
        torch.cuda.synchronize()
    r_sel = ref.select_buckets(scores, Hkv, nprobe, mode=mode)
    assert np.array_equal(sel.cpu().numpy(), r_sel)
    want, ps, nruns = plan_by_hand(r_sel, off, ln, Hq // Hkv if mode == 1 else 1)
    assert np.array_equal(used_part(plan.cpu().numpy(), want.shape[0], ps, nruns), want[:, :2 * nruns + 2])


@pytest.mark.parametrize("S,Hq,Hkv,B,nprobe,mode,resident", [
    (2, 8, 2, 200, 13, 0, -1), (1, 8, 2, 64, 9, 1, -1), (2, 4, 2, 50, 7, 0, 50), (1, 4, 1, 30, 0, 0, 30), (1, 2, 1, 9000, 8000, 0, -1),
])
def test_build_visit_plan(saap, S, Hq, Hkv, B, nprobe, mode, resident):
    rng = np.random.default_rng(B + nprobe)
    runs = B + (1 if resident >= 0 else 0)
    ln = rng.integers(0, 50, size=(S, Hkv, runs)).astype(np.int32)
    off = np.zeros((S, Hkv, runs + 1), dtype=np.int32)
    off[:, :, 1:] = np.cumsum(ln + 1, axis=2)
    lists = Hq if mode == 1 else Hkv
    sel = np.stack([rng.permutation(B)[:nprobe] for _ in range(S * lists)]).reshape(S, lists, nprobe).astype(np.int32)
    plan = saap.build_visit_plan(torch.from_numpy(sel).to(DEV), torch.from_numpy(off).to(DEV), torch.from_numpy(ln).to(DEV),
                                 Hq, mode=mode, resident_run=resident)
    torch.cuda.synchronize()
    want, ps, nruns = plan_by_hand(sel, off, ln, Hq // Hkv if mode == 1 else 1, resident)
    assert np.array_equal(used_part(plan.cpu().numpy(), want.shape[0], ps, nruns), want[:, :2 * nruns + 2])


# ------------------------------------------------------------------------------ attention from a plan
@pytest.mark.parametrize("dtype,S,Hq,Hkv,N,B,nprobe,slack,alpha", [
    ("bf16", 1, 4, 1, 6000, 64, 8, 0, None),
    ("bf16", 2, 8, 2, 5003, 128, 13, 2, 0.3),
    ("f32", 1, 1, 1, 4096, 64, 8, 0, None),
    ("f32", 1, 4, 2, 2500, 32, 5, 1, 0.3),
    ("bf16", 1, 8, 1, 3000, 32, 32, 0, None),       # G = 8, all buckets
    ("bf16", 1, 2, 1, 3000, 32, 1, 0, 0.3),         # G = 2, one bucket
    ("bf16", 3, 12, 3, 40000, 256, 40, 0, 0.3),     # many workgroups per unit, skewed buckets
    ("bf16", 37, 4, 1, 900, 16, 3, 0, None),        # more units than the keys need workgroups
])
def test_planned_attention(saap, dtype, S, Hq, Hkv, N, B, nprobe, slack, alpha):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=nprobe, dtype=dtype, alpha=alpha,
                                                   hidden=64)
    cache, (off, ln, idx, Ks, Vs) = make_index(saap, cfg, 7, slack)
    _, q = gen.make_queries(cfg, 7, DEV)
    rng = np.random.default_rng(N + nprobe)
    sel = np.stack([rng.permutation(B)[:nprobe] for _ in range(S * Hkv)]).reshape(S, Hkv, nprobe).astype(np.int32)
    plan = saap.build_visit_plan(torch.from_numpy(sel).to(DEV), off, ln, Hq)
    out, lse = saap.planned_decode_attention(q[0], Ks, Vs, plan, nprobe, SCALE)
    out16, _ = saap.planned_decode_attention(q[0], Ks, Vs, plan, nprobe, SCALE, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    ro, rl = ref.sparse_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), off.cpu().numpy(), ln.cpu().numpy(),
                                         idx.cpu().numpy(), sel, SCALE)
    assert_close(out.cpu().numpy(), ro, dtype, "planned out")
    assert_close(lse.cpu().numpy(), rl, dtype, "planned lse")
    assert_close(out16.float().cpu().numpy(), ro, "bf16", "planned out (bf16 store)")


@pytest.mark.parametrize("S,Hkv,G,seed", [(3, 3, 4, 0), (5, 7, 2, 1), (1, 9, 4, 2), (11, 1, 8, 3)])
def test_planned_attention_with_wildly_unequal_units(saap, S, Hkv, G, seed):
    """Units without any visited key, units ten times the mean, a unit count that divides nothing: the lists
    are planted so that list sizes differ by orders of magnitude, and every unit must still get exactly the
    softmax over its own keys."""
    N, B = 30000, 64
    Hq = Hkv * G
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=S, Hq=Hq, Hkv=Hkv, N=N, B=B, nprobe=8, alpha=0.3, hidden=64)
    cache, (off, ln, idx, Ks, Vs) = make_index(saap, cfg, 40 + seed)
    _, q = gen.make_queries(cfg, 40 + seed, DEV)
    h_ln = ln.cpu().numpy().copy()
    rng = np.random.default_rng(seed)
    nprobe = 8
    sel = np.zeros((S, Hkv, nprobe), dtype=np.int32)
    units = S * Hkv
    big, empty = rng.choice(units, 2, replace=False)
    for u in range(units):
        s, hk = divmod(u, Hkv)
        order = np.argsort(h_ln[s, hk], kind="stable")
        if u == big:
            sel[s, hk] = order[-nprobe:]                    # the eight largest buckets
        elif u == empty:
            sel[s, hk] = order[:nprobe]
            h_ln[s, hk, order[:nprobe]] = 0                 # ... made empty: this unit visits no key
        else:
            sel[s, hk] = rng.permutation(B)[:nprobe] if rng.random() < 0.5 else order[:nprobe]   # typical, or the smallest
    d_ln = torch.from_numpy(h_ln).to(DEV)
    totals = np.take_along_axis(h_ln, sel, axis=2).sum(-1).reshape(-1)
    assert totals[empty] == 0 and totals[big] >= 5 * max(1, np.median(totals))
    plan = saap.build_visit_plan(torch.from_numpy(sel).to(DEV), off, d_ln, Hq)
    out, lse = saap.planned_decode_attention(q[0], Ks, Vs, plan, nprobe, SCALE)
    torch.cuda.synchronize()
    ro, rl = ref.sparse_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), off.cpu().numpy(), h_ln, idx.cpu().numpy(),
                                         sel, SCALE)
    assert_close(out.cpu().numpy(), ro, "bf16", "unequal units out")
    assert_close(lse.cpu().numpy(), rl, "bf16", "unequal units lse")
    s_e, h_e = divmod(int(empty), Hkv)
    assert (out[s_e, h_e * G:(h_e + 1) * G] == 0).all() and torch.isneginf(lse[s_e, h_e * G:(h_e + 1) * G]).all()
    # and the same launch twice more on the same workspace (arrival counters must come back to zero).  Which
    # wave takes which batch of keys depends on timing, so a repeat agrees in value, not bit for bit.
    for _ in range(2):
        o2, l2 = saap.planned_decode_attention(q[0], Ks, Vs, plan, nprobe, SCALE)
    torch.cuda.synchronize()
    assert_close(o2.cpu().numpy(), ro, "bf16", "repeat out")
    assert torch.allclose(o2, out, rtol=1e-4, atol=1e-5) and torch.allclose(l2[torch.isfinite(lse)], lse[torch.isfinite(lse)], rtol=1e-5)


def test_planned_attention_independent_lists_and_resident_run(saap):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=2, Hq=8, Hkv=2, N=4000, B=64, nprobe=6, hidden=64)
    cache, (off, ln, idx, Ks, Vs) = make_index(saap, cfg, 13)
    _, q = gen.make_queries(cfg, 13, DEV)
    rng = np.random.default_rng(5)
    sel = np.stack([rng.permutation(cfg.B)[:6] for _ in range(2 * 8)]).reshape(2, 8, 6).astype(np.int32)
    plan = saap.build_visit_plan(torch.from_numpy(sel).to(DEV), off, ln, cfg.Hq, mode=saap.INDEPENDENT)
    out, lse = saap.planned_decode_attention(q[0], Ks, Vs, plan, 6, SCALE, mode=saap.INDEPENDENT)
    torch.cuda.synchronize()
    ro, rl = ref.sparse_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), off.cpu().numpy(), ln.cpu().numpy(),
                                         idx.cpu().numpy(), sel, SCALE, mode=1)
    assert_close(out.cpu().numpy(), ro, "bf16", "independent out")
    assert_close(lse.cpu().numpy(), rl, "bf16", "independent lse")

    # sink + recent keys as the always-visited run: the position-based oracle knows no run at all
    n_sink, n_recent = 4, 250
    ids = cache["ids"]
    w_off, w_ln, w_idx, w_Ks, w_Vs, _ = saap.build_windowed_index(ids, cache["K"], cache["V"], cfg.B, 2, n_sink, n_recent)
    gsel = sel[:, ::4, :].copy()
    plan = saap.build_visit_plan(torch.from_numpy(gsel).to(DEV), w_off, w_ln, cfg.Hq, resident_run=cfg.B)
    out, lse = saap.planned_decode_attention(q[0], w_Ks, w_Vs, plan, 7, SCALE)
    torch.cuda.synchronize()
    ro, rl = ref.windowed_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), ids.cpu().numpy(), gsel, n_sink, n_recent,
                                           SCALE, cfg.B)
    assert_close(out.cpu().numpy(), ro, "bf16", "windowed out")
    assert_close(lse.cpu().numpy(), rl, "bf16", "windowed lse")


def test_planned_attention_all_buckets_is_dense_and_nothing_selected(saap):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=1, Hq=8, Hkv=2, N=7001, B=96, nprobe=96, hidden=64)
    cache, (off, ln, idx, Ks, Vs) = make_index(saap, cfg, 11, slack=2)
    _, q = gen.make_queries(cfg, 11, DEV)
    g = torch.Generator(device="cpu").manual_seed(1)
    sel = torch.stack([torch.randperm(cfg.B, generator=g) for _ in range(2)]).view(1, 2, cfg.B).to(torch.int32).to(DEV)
    plan = saap.build_visit_plan(sel, off, ln, cfg.Hq)
    out, lse = saap.planned_decode_attention(q[0], Ks, Vs, plan, cfg.B, SCALE)
    empty = saap.build_visit_plan(torch.empty(1, 2, 0, dtype=torch.int32, device=DEV), off, ln, cfg.Hq)
    o0, l0 = saap.planned_decode_attention(q[0], Ks, Vs, empty, 0, SCALE)
    torch.cuda.synchronize()
    ro, rl = ref.dense_decode_attention(h(q[0]), h(cache["K"]), h(cache["V"]), SCALE)
    assert_close(out.cpu().numpy(), ro, "bf16", "nprobe = B")
    assert_close(lse.cpu().numpy(), rl, "bf16", "nprobe = B lse")
    assert (o0 == 0).all() and torch.isneginf(l0).all()


def test_planned_attention_fp8(saap):
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=2, Hq=8, Hkv=2, N=9000, B=64, nprobe=9, alpha=0.3, hidden=64)
    cache, (off, ln, idx, Ks, Vs) = make_index(saap, cfg, 3)
    _, q = gen.make_queries(cfg, 3, DEV)
    K8, V8, ks, vs = saap.quantize_kv(Ks, Vs)
    rng = np.random.default_rng(9)
    sel = np.stack([rng.permutation(cfg.B)[:9] for _ in range(4)]).reshape(2, 2, 9).astype(np.int32)
    plan = saap.build_visit_plan(torch.from_numpy(sel).to(DEV), off, ln, cfg.Hq)
    out, lse = saap.planned_decode_attention_fp8(q[0], K8, V8, ks, vs, plan, 9, SCALE)
    want, wl = saap.sparse_decode_attention_fp8(q[0], K8, V8, ks, vs, off, ln, torch.from_numpy(sel).to(DEV), SCALE)
    torch.cuda.synchronize()
    # oracle on the decoded cache (the decoded values are exact in fp32), position-ordered through idx
    h_idx = idx.cpu().numpy()
    Kd = ref.dequantize_fp8(K8.cpu().numpy(), ks.cpu().numpy())
    Vd = ref.dequantize_fp8(V8.cpu().numpy(), vs.cpu().numpy())
    Kp, Vp = np.zeros_like(h(cache["K"])), np.zeros_like(h(cache["V"]))
    for s in range(2):
        for hk in range(2):
            m = h_idx[s, hk] >= 0
            Kp[s, hk, h_idx[s, hk][m]] = Kd[s, hk][m]
            Vp[s, hk, h_idx[s, hk][m]] = Vd[s, hk][m]
    ro, rl = ref.sparse_decode_attention(h(q[0]), Kp, Vp, off.cpu().numpy(), ln.cpu().numpy(), h_idx, sel, SCALE)
    assert_close(out.cpu().numpy(), ro, "bf16", "planned fp8 out")
    assert_close(lse.cpu().numpy(), rl, "bf16", "planned fp8 lse")
    assert_close(want.cpu().numpy(), ro, "bf16", "list fp8 out")


def test_planned_attention_rejects_what_it_does_not_cover(saap):
    q = torch.zeros(1, 4, 128, dtype=torch.bfloat16, device=DEV)
    K = torch.zeros(1, 1, 64, 128, dtype=torch.bfloat16, device=DEV)
    plan = torch.zeros(64, dtype=torch.int32, device=DEV)
    with pytest.raises(ValueError):
        saap.planned_decode_attention(q, K, K, plan[:2], 5, SCALE)         # plan buffer too short
    with pytest.raises(saap.SaapError) as e:
        saap.planned_decode_attention(q[:, :3], K, K, plan, 5, SCALE)      # 3 heads per KV head
    assert e.value.status == -2
