"""The decode step under HIP graph capture: the three calls of a step are recorded once and replayed
with new inputs several times, with eager work and synchronisations between the replays; every
replay must give exactly what the same calls give when launched eagerly (the library takes its
scratch from the caller's workspace, allocates nothing and records no memset, so nothing in it
should depend on how it is launched)."""
import math

import pytest
import torch

from synth import gen

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
SCALE = 1.0 / math.sqrt(128.0)


def test_step_replays_match_eager_launches():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the -m gpu tests need a real device")
    import paper_2502_08246_amd as saap
    saap.load_library()
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(N=16384, B=256, nprobe=13, hidden=128)
    cache = gen.make_cache(cfg, 5, DEV)
    cent = gen.make_centroids(cfg, 5, DEV, cache, n_train=4096)
    xq, q = gen.make_queries(cfg, 5, DEV, n_steps=6)
    W1, b1, W2, b2 = gen.make_classifier(cfg, 5, DEV)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, 0)

    x_in, q_in = xq[0].clone(), q[0].clone()
    logits = torch.empty(cfg.S, cfg.Hq, cfg.B, dtype=torch.float32, device=DEV)
    sel = torch.empty(cfg.S, cfg.Hkv, cfg.nprobe, dtype=torch.int32, device=DEV)
    out = torch.empty(cfg.S, cfg.Hq, cfg.d, dtype=torch.float32, device=DEV)
    lse = torch.empty(cfg.S, cfg.Hq, dtype=torch.float32, device=DEV)

    def step():
        saap.classify_queries(x_in, W1, b1, W2, b2, cfg.Hkv, output_kind=saap.LOGITS, out=logits)
        saap.select_buckets_from_logits(logits, cfg.Hkv, cfg.nprobe, out=sel)
        saap.sparse_decode_attention(q_in, Ks, Vs, off, ln, sel, SCALE, out=out, lse=lse)

    step()                                   # sizes the binding's workspace before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()

    for t in range(1, 6):
        x_in.copy_(xq[t])
        q_in.copy_(q[t])
        graph.replay()
        torch.cuda.synchronize()
        got = [a.clone() for a in (logits, sel, out, lse)]
        # eager work of the program itself between the replays: the same step, launched directly
        for a in (logits, sel, out, lse):
            a.zero_()
        step()
        torch.cuda.synchronize()
        for g, w, name in zip(got, (logits, sel, out, lse), ("logits", "selected", "out", "lse")):
            assert torch.equal(g, w), f"replay {t}: {name} differs from the eager launch"
        ws = saap.workspace(0, DEV)
        assert int(ws[:65536].view(torch.int64).abs().sum().item()) == 0, "arrival counters must be zero between calls"


def test_own_workspace_on_a_side_stream():
    """A caller-provided workspace that starts with a dirty header is reset by workspace_reset, and the decode
    calls run with it on a stream of the caller's; the results equal those of the default workspace and stream."""
    import paper_2502_08246_amd as saap
    saap.load_library()
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=2, Hq=8, Hkv=2, N=5000, B=32, nprobe=6, hidden=64)
    cache = gen.make_cache(cfg, 61, DEV)
    cent = gen.make_centroids(cfg, 61, DEV, cache, n_train=2048)
    xq, q = gen.make_queries(cfg, 61, DEV, n_steps=1)
    W1, b1, W2, b2 = gen.make_classifier(cfg, 61, DEV)
    ids = saap.assign_keys(cache["x_keys"], cent)
    off, ln, idx, Ks, Vs = saap.build_bucket_index(ids, cache["K"], cache["V"], cfg.B, 0)
    logits = saap.classify_queries(xq[0], W1, b1, W2, b2, cfg.Hkv, output_kind=saap.LOGITS)
    sel = saap.select_buckets_from_logits(logits, cfg.Hkv, cfg.nprobe)
    want, want_lse = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, sel, SCALE)
    torch.cuda.synchronize()
    need = saap.workspace_bytes(saap.binding.OP_SPARSE_DECODE_ATTENTION, S=cfg.S, Hq=cfg.Hq, Hkv=cfg.Hkv, mode=0)
    ws = torch.full((need,), 0xAB, dtype=torch.uint8, device=DEV)          # arrival counters full of garbage
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        saap.workspace_reset(ws)
        assert int(ws[:65536].view(torch.int32).abs().sum().item()) == 0
        lg = saap.classify_queries(xq[0], W1, b1, W2, b2, cfg.Hkv, output_kind=saap.LOGITS, ws=ws)
        sl = saap.select_buckets_from_logits(lg, cfg.Hkv, cfg.nprobe, ws=ws)
        got, got_lse = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, sl, SCALE, ws=ws)
        got2, _ = saap.sparse_decode_attention(q[0], Ks, Vs, off, ln, sl, SCALE, ws=ws)      # the header was left clean
    side.synchronize()
    assert torch.equal(sl, sel) and torch.equal(got, want) and torch.equal(got_lse, want_lse) and torch.equal(got2, want)
    assert int(ws[:65536].view(torch.int32).abs().sum().item()) == 0


def test_generation_on_the_8bit_cache_replayed_and_eager():
    """A generation step that changes state (classify, select, attention over the selected buckets and the
    resident window of an 8-bit cache, then the push of the token's key into that cache): one copy of the state
    is advanced by replaying a captured graph, a second copy by launching the same calls directly; outputs and
    both states agree bit for bit after every step."""
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the -m gpu tests need a real device")
    import paper_2502_08246_amd as saap
    saap.load_library()
    steps, n_sink, n_recent = 12, 1, 31
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=2, N=6000 + steps, B=64, nprobe=7, hidden=128)
    N = 6000
    cache = gen.make_cache(cfg, 7, DEV)
    cent = gen.make_centroids(cfg, 7, DEV, cache, n_train=4096)
    xq, q = gen.make_queries(cfg, 7, DEV, n_steps=steps)
    W1, b1, W2, b2 = gen.make_classifier(cfg, 7, DEV)
    x, K, V = cache["x_keys"], cache["K"], cache["V"]
    ids = saap.assign_keys(x, cent)
    built = saap.build_windowed_index(ids[:, :, :N].contiguous(), K[:, :, :N].contiguous(), V[:, :, :N].contiguous(), cfg.B, 32,
                                      n_sink, n_recent)
    off, ln0, idx0, Ks, Vs, res0 = built
    K8_0, V8_0, ks, vs = saap.quantize_kv(Ks, Vs)
    torch.cuda.synchronize()

    def fresh():
        return dict(ln=ln0.clone(), idx=idx0.clone(), K8=K8_0.clone(), V8=V8_0.clone(), res=res0.clone(),
                    logits=torch.empty(cfg.S, cfg.Hq, cfg.B, dtype=torch.float32, device=DEV),
                    sel=torch.empty(cfg.S, cfg.Hkv, cfg.nprobe, dtype=torch.int32, device=DEV),
                    out=torch.empty(cfg.S, cfg.Hq, cfg.d, dtype=torch.float32, device=DEV),
                    lse=torch.empty(cfg.S, cfg.Hq, dtype=torch.float32, device=DEV),
                    nid=torch.empty(cfg.S, cfg.Hkv, dtype=torch.int32, device=DEV),
                    flag=torch.zeros(4, dtype=torch.int32, device=DEV))

    x_in, q_in = xq[0].clone(), q[0].clone()
    xn, kn, vn = (a[:, :, N].clone() for a in (x, K, V))
    pos = torch.full((cfg.S,), N, dtype=torch.int32, device=DEV)

    def step(st):
        saap.classify_queries(x_in, W1, b1, W2, b2, cfg.Hkv, output_kind=saap.LOGITS, out=st["logits"])
        saap.select_buckets_from_logits(st["logits"], cfg.Hkv, cfg.nprobe, out=st["sel"])
        saap.windowed_decode_attention_fp8(q_in, st["K8"], st["V8"], ks, vs, off, st["ln"], st["sel"], cfg.B, SCALE,
                                           out=st["out"], lse=st["lse"])
        saap.window_push_fp8(xn, kn, vn, pos, cent, None, off, st["ln"], st["idx"], st["K8"], st["V8"], ks, vs, st["res"],
                             n_sink, n_recent, overflow_flag=st["flag"], new_ids=st["nid"])

    warm = fresh()
    step(warm)                               # sizes the binding's workspace before the capture
    torch.cuda.synchronize()
    a, b = fresh(), fresh()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(a)
    torch.cuda.synchronize()
    for k in a:                              # the capture itself launched nothing: a is still the fresh state
        assert torch.equal(a[k], b[k]) or k in ("logits", "sel", "out", "lse", "nid")
    for t in range(steps):
        x_in.copy_(xq[t])
        q_in.copy_(q[t])
        for dst, src in ((xn, x), (kn, K), (vn, V)):
            dst.copy_(src[:, :, N + t])
        pos.fill_(N + t)
        graph.replay()
        torch.cuda.synchronize()
        step(b)
        torch.cuda.synchronize()
        for k in a:
            assert torch.equal(a[k], b[k]), f"step {t}: {k} differs between the replay and the eager launch"
        assert a["flag"][0].item() == 0
    assert int(a["ln"][..., :cfg.B].sum().item()) == int(ln0[..., :cfg.B].sum().item()) + steps * cfg.S * cfg.Hkv
