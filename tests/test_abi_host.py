"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol that
include/saap.h declares, sizes workspaces, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2502_08246_amd as saap
from paper_2502_08246_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return saap.load_library()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "saap.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(saap_[a-z0-9_]+)\s*\(", header))
    assert {"saap_assign_keys", "saap_build_bucket_index", "saap_classify_queries", "saap_select_buckets",
            "saap_sparse_decode_attention", "saap_dense_decode_attention", "saap_append_keys"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.EXPORTS)


def test_status_strings(lib):
    assert binding.status_string(0) == "ok"
    for st in (-1, -2, -3, -4, -5, -99):
        assert isinstance(binding.status_string(st), str) and binding.status_string(st)


def test_workspace_bytes_arithmetic():
    hdr = binding.WS_HEADER_BYTES
    # attention: header + units * 128 partial slots * G heads * (d + 2) floats
    got = saap.workspace_bytes(binding.OP_SPARSE_DECODE_ATTENTION, S=1, Hq=32, Hkv=8, mode=0)
    assert got == hdr + 8 * 128 * 4 * 130 * 4
    got = saap.workspace_bytes(binding.OP_SPARSE_DECODE_ATTENTION, S=2, Hq=32, Hkv=8, mode=1)
    assert got == hdr + 64 * 128 * 1 * 130 * 4
    assert saap.workspace_bytes(binding.OP_DENSE_DECODE_ATTENTION, S=1, Hq=4, Hkv=4) == hdr + 4 * 128 * 130 * 4
    assert saap.workspace_bytes(binding.OP_SELECT_BUCKETS) == hdr
    assert saap.workspace_bytes(binding.OP_BUILD_BUCKET_INDEX, S=1, Hkv=8, N=131072, B=1024) == hdr + 8 * 64 * 1024 * 4
    assert saap.workspace_bytes(binding.OP_ASSIGN_KEYS, S=1, Hkv=2, N=1000) == hdr + 16384 + 2000 * 4
    assert saap.workspace_bytes(binding.OP_SPARSE_DECODE_ATTENTION, S=1, Hq=5, Hkv=2) == 0   # Hq % Hkv != 0
    assert saap.workspace_bytes(99, S=1) == 0


def _fake(n=1):
    """Aligned non-null fake device pointers: argument validation must fail before any is used."""
    return [ctypes.c_void_p(4096 * (i + 1)) for i in range(n)]


def test_invalid_arguments_are_rejected_on_the_host(lib):
    q, K, V, off, ln, sel, out, lse, ws = _fake(9)
    i32, f32 = ctypes.c_int32, ctypes.c_float
    big = ctypes.c_size_t(1 << 30)

    def sparse(**kw):
        a = dict(q=q, K=K, V=V, off=off, ln=ln, sel=sel, nprobe=4, mode=0, scale=0.1, out=out, odt=0, lse=lse,
                 S=1, Hq=4, Hkv=1, Ncap=100, B=8, d=128, dt=1, ws=ws, wsb=big)
        a.update(kw)
        return lib.saap_sparse_decode_attention(a["q"], a["K"], a["V"], a["off"], a["ln"], a["sel"], i32(a["nprobe"]),
                                                i32(a["mode"]), f32(a["scale"]), a["out"], i32(a["odt"]), a["lse"],
                                                i32(a["S"]), i32(a["Hq"]), i32(a["Hkv"]), i32(a["Ncap"]), i32(a["B"]),
                                                i32(a["d"]), i32(a["dt"]), a["ws"], a["wsb"], None)

    assert sparse(q=None) == -1
    assert sparse(q=ctypes.c_void_p(4100)) == -1            # misaligned
    assert sparse(nprobe=9) == -1                           # nprobe > B
    assert sparse(nprobe=-1) == -1
    assert sparse(Hq=5, Hkv=2) == -1
    assert sparse(d=64) == -2
    assert sparse(Hq=3, Hkv=1) == -2                        # G = 3 unsupported
    assert sparse(dt=7) == -1
    assert sparse(mode=2) == -1
    assert sparse(wsb=ctypes.c_size_t(1024)) == -3

    def select(**kw):
        a = dict(sc=q, sel=sel, S=1, Hq=4, Hkv=1, B=64, nprobe=8, mode=0)
        a.update(kw)
        return lib.saap_select_buckets(a["sc"], a["sel"], i32(a["S"]), i32(a["Hq"]), i32(a["Hkv"]), i32(a["B"]),
                                       i32(a["nprobe"]), i32(a["mode"]), ws, big, None)

    assert select(nprobe=65) == -1
    assert select(B=1 << 20, nprobe=8) == -2
    assert select(sc=None) == -1
    assert select(nprobe=0) == 0                            # nothing to do, nothing launched

    st = lib.saap_build_bucket_index(q, K, V, off, ln, sel, out, lse, i32(1), i32(1), i32(100), i32(99), i32(8),
                                     i32(128), i32(1), i32(0), ws, big, None)
    assert st == -1                                         # Ncap != N + B*slack
    st = lib.saap_assign_keys(q, K, None, sel, i32(1), i32(1), i32(100), i32(8), i32(128), i32(1), ws,
                              ctypes.c_size_t(16), None)
    assert st == -3
    st = lib.saap_classify_queries(q, K, None, V, None, i32(3), out, i32(1), i32(4), i32(2), i32(128), i32(64),
                                   i32(64), i32(1), i32(0), ws, big, None)
    assert st == -1                                         # Hw must be 1, Hkv or Hq
    st = lib.saap_classify_queries(q, K, None, V, None, i32(1), out, i32(1), i32(4), i32(2), i32(128), i32(40),
                                   i32(64), i32(1), i32(0), ws, big, None)
    assert st == -2                                         # hidden % 32
    st = lib.saap_dense_decode_attention(q, K, V, off, None, i32(8), f32(0.1), out, i32(0), lse, i32(1), i32(4),
                                         i32(1), i32(100), i32(128), i32(1), ws, big, None)
    assert st == -1                                         # off without len

    def windowed(**kw):
        a = dict(nprobe=4, resident=8, runs=9)
        a.update(kw)
        return lib.saap_windowed_decode_attention(q, K, V, off, ln, sel, i32(a["nprobe"]), i32(0), i32(a["resident"]),
                                                  f32(0.1), out, i32(0), lse, i32(1), i32(4), i32(1), i32(100),
                                                  i32(a["runs"]), i32(128), i32(1), ws, big, None)

    assert windowed(resident=9) == -1                       # the resident run must be one of the runs
    assert windowed(resident=-2) == -1
    assert windowed(nprobe=9) == -1                         # nprobe + the resident run > runs
    st = lib.saap_build_windowed_index(q, K, V, off, ln, sel, out, lse, sel, i32(1), i32(1), i32(100), i32(100), i32(8),
                                       i32(128), i32(1), i32(2), i32(1), i32(15), ws, big, None)
    assert st == -1                                         # Ncap != N - W + B*slack + W = 116
    st = lib.saap_build_windowed_index(q, K, V, off, ln, sel, out, lse, None, i32(1), i32(1), i32(100), i32(116), i32(8),
                                       i32(128), i32(1), i32(2), i32(1), i32(15), ws, big, None)
    assert st == -1                                         # resident_ids missing
    st = lib.saap_window_push(q, K, V, None, q, None, off, ln, sel, out, lse, sel, sel, sel, i32(1), i32(1), i32(116),
                              i32(8), i32(128), i32(1), i32(1), i32(15), ws, big, None)
    assert st == -1                                         # pos_new missing
    st = lib.saap_window_push(q, K, V, sel, q, None, off, ln, sel, out, lse, sel, sel, sel, i32(1), i32(1), i32(10),
                              i32(8), i32(128), i32(1), i32(1), i32(15), ws, big, None)
    assert st == -1                                         # window larger than the cache
    st = lib.saap_window_push(q, K, V, sel, q, None, off, ln, sel, out, lse, sel, sel, sel, i32(1), i32(1), i32(116),
                              i32(8), i32(128), i32(1), i32(1), i32(15), ws, ctypes.c_size_t(100), None)
    assert st == -3


def test_binding_refuses_host_tensors():
    import torch
    x = torch.zeros(1, 1, 8, 128)
    c = torch.zeros(1, 4, 128)
    with pytest.raises(ValueError):
        saap.assign_keys(x, c, out=torch.zeros(1, 1, 8, dtype=torch.int32), ws=torch.zeros(1 << 20, dtype=torch.uint8))


def test_invalid_arguments_of_the_later_calls_are_rejected_on_the_host(lib):
    """8-bit cache, bucket attention mass and the training calls: argument checks fail before anything is enqueued."""
    q, K, V, off, ln, sel, out, lse, ws, ks, vs = _fake(11)
    i32, f32 = ctypes.c_int32, ctypes.c_float
    big, small = ctypes.c_size_t(1 << 30), ctypes.c_size_t(1024)

    def quant(**kw):
        a = dict(K=K, ks=ks, S=1, Hkv=2, Ncap=64, d=128, dt=1, wsb=big)
        a.update(kw)
        return lib.saap_quantize_kv(a["K"], V, out, lse, a["ks"], vs, i32(a["S"]), i32(a["Hkv"]), i32(a["Ncap"]), i32(a["d"]),
                                    i32(a["dt"]), ws, a["wsb"], None)

    assert quant(K=None) == -1 and quant(ks=None) == -1 and quant(Ncap=0) == -1 and quant(dt=2) == -1
    assert quant(d=64) == -2 and quant(S=70000) == -2 and quant(wsb=small) == -3

    def sparse8(**kw):
        a = dict(ks=ks, nprobe=4, mode=0, Hq=4, Hkv=1, B=8, odt=0, wsb=big)
        a.update(kw)
        return lib.saap_sparse_decode_attention_fp8(q, K, V, a["ks"], vs, off, ln, sel, i32(a["nprobe"]), i32(a["mode"]),
                                                    f32(0.1), out, i32(a["odt"]), lse, i32(1), i32(a["Hq"]), i32(a["Hkv"]),
                                                    i32(100), i32(a["B"]), i32(128), ws, a["wsb"], None)

    assert sparse8(ks=None) == -1 and sparse8(nprobe=9) == -1 and sparse8(mode=3) == -1 and sparse8(odt=5) == -1
    assert sparse8(Hq=3) == -2 and sparse8(wsb=small) == -3
    st = lib.saap_dense_decode_attention_fp8(q, K, V, ks, None, None, None, i32(0), f32(0.1), out, i32(0), lse, i32(1), i32(4),
                                             i32(1), i32(100), i32(128), ws, big, None)
    assert st == -1                                         # vscale missing
    st = lib.saap_windowed_decode_attention_fp8(q, K, V, ks, vs, off, ln, sel, i32(4), i32(0), i32(9), f32(0.1), out, i32(0),
                                                lse, i32(1), i32(4), i32(1), i32(100), i32(9), i32(128), ws, big, None)
    assert st == -1                                         # the resident run must be one of the runs
    # the 16-bit entry points do not accept the internal code of the 8-bit cache
    st = lib.saap_sparse_decode_attention(q, K, V, off, ln, sel, i32(4), i32(0), f32(0.1), out, i32(0), lse, i32(1), i32(4),
                                          i32(1), i32(100), i32(8), i32(128), i32(2), ws, big, None)
    assert st == -1

    def push8(**kw):
        a = dict(ks=ks, pos=sel, res=sel, Ncap=116, B=8, d=128, wsb=big)
        a.update(kw)
        return lib.saap_window_push_fp8(q, K, V, a["pos"], q, None, off, ln, sel, out, lse, a["ks"], vs, a["res"], sel, sel,
                                        i32(1), i32(1), i32(a["Ncap"]), i32(a["B"]), i32(a["d"]), i32(1), i32(15), ws,
                                        a["wsb"], None)

    assert push8(ks=None) == -1 and push8(pos=None) == -1 and push8(res=None) == -1 and push8(Ncap=10) == -1
    assert push8(d=64) == -2 and push8(wsb=ctypes.c_size_t(100)) == -3
    st = lib.saap_append_keys_fp8(q, K, V, None, q, None, off, ln, sel, out, lse, ks, None, sel, sel, i32(1), i32(1), i32(116),
                                  i32(8), i32(128), ws, big, None)
    assert st == -1                                         # vscale missing

    def mass(**kw):
        a = dict(q=q, m=out, Hq=4, Hkv=1, B=8, d=128, dt=1, wsb=big)
        a.update(kw)
        return lib.saap_bucket_attention_mass(a["q"], K, off, ln, f32(0.1), a["m"], lse, i32(1), i32(a["Hq"]), i32(a["Hkv"]),
                                              i32(100), i32(a["B"]), i32(a["d"]), i32(a["dt"]), ws, a["wsb"], None)

    assert mass(q=None) == -1 and mass(m=None) == -1 and mass(B=0) == -1 and mass(Hq=5, Hkv=2) == -1 and mass(dt=3) == -1
    assert mass(d=64) == -2 and mass(Hq=3) == -2 and mass(wsb=small) == -3

    def mass_batch(**kw):
        a = dict(q=q, R=100, B=8, d=128, dt=1, wsb=big)
        a.update(kw)
        return lib.saap_bucket_attention_mass_batch(a["q"], K, off, ln, f32(0.1), out, lse, i32(1), i32(2), i32(a["R"]),
                                                    i32(100), i32(a["B"]), i32(a["d"]), i32(a["dt"]), ws, a["wsb"], None)

    assert mass_batch(q=None) == -1 and mass_batch(R=0) == -1 and mass_batch(B=0) == -1 and mass_batch(dt=4) == -1
    assert mass_batch(d=64) == -2 and mass_batch(dt=0) == -2 and mass_batch(wsb=small) == -3
    assert saap.workspace_bytes(binding.OP_BUCKET_ATTENTION_MASS_BATCH, S=1, Hkv=2, N=100, B=8) == binding.WS_HEADER_BYTES + 2 * 100 * 8 * 8

    params = binding._MlpF32(*(p.value for p in _fake(4)))
    holes = binding._MlpF32(4096, None, 8192, 12288)

    def grads(**kw):
        a = dict(x=q, p=params, g=params, Hw=2, R=16, d=128, hidden=64, B=32, dt=1, wsb=big)
        a.update(kw)
        return lib.saap_query_model_loss_grads(a["x"], K, ctypes.byref(a["p"]), ctypes.byref(a["g"]), lse, i32(a["Hw"]),
                                               i32(a["R"]), i32(a["d"]), i32(a["hidden"]), i32(a["B"]), i32(a["dt"]), ws,
                                               a["wsb"], None)

    assert grads(x=None) == -1 and grads(p=holes) == -1 and grads(g=holes) == -1 and grads(R=0) == -1 and grads(dt=2) == -1
    assert grads(Hw=70000) == -2 and grads(wsb=small) == -3
    need = saap.workspace_bytes(binding.OP_QUERY_MODEL_LOSS_GRADS, Hkv=2, N=16, d=128, hidden=64, B=32)
    assert need == binding.WS_HEADER_BYTES + 2 * 16 * (128 + 3 * 64 + 32 + 1) * 4 + 2 * 4 * 64 * 4

    def bn_struct(**kw):
        a = dict(gamma=4096, beta=8192, gg=12288, gb=16384, rm=None, rv=None, mom=0.1, eps=1e-5)
        a.update(kw)
        return binding._BatchNormF32(a["gamma"], a["beta"], a["gg"], a["gb"], a["rm"], a["rv"], a["mom"], a["eps"])

    def grads_bn(bn, **kw):
        a = dict(R=16, wsb=big)
        a.update(kw)
        return lib.saap_query_model_bn_loss_grads(q, K, ctypes.byref(params), ctypes.byref(params),
                                                  ctypes.byref(bn) if bn is not None else None, lse, i32(2), i32(a["R"]),
                                                  i32(128), i32(64), i32(32), i32(1), ws, a["wsb"], None)

    assert grads_bn(None) == -1 and grads_bn(bn_struct(gamma=None)) == -1 and grads_bn(bn_struct(gb=None)) == -1
    assert grads_bn(bn_struct(rm=4096)) == -1                # running mean without running variance
    assert grads_bn(bn_struct(eps=0.0)) == -1 and grads_bn(bn_struct(mom=1.5)) == -1
    assert grads_bn(bn_struct(), R=1) == -1 and grads_bn(bn_struct(), wsb=small) == -3
    fold = lambda **kw: lib.saap_fold_batch_norm(kw.get("W1", q), K, K, K, K, K, f32(kw.get("eps", 1e-5)), out, lse, i32(2),
                                                 i32(kw.get("hidden", 64)), i32(128), i32(kw.get("dt", 1)), None)
    assert fold(W1=None) == -1 and fold(eps=0.0) == -1 and fold(hidden=0) == -1 and fold(dt=2) == -1
    assert saap.workspace_bytes(binding.OP_BUCKET_ATTENTION_MASS, S=1, Hq=32, Hkv=8, B=1024) == binding.WS_HEADER_BYTES + 8 * 1024 * 4 * 8

    def adam(**kw):
        a = dict(p=q, n=100, step=1, b1=0.9, b2=0.999)
        a.update(kw)
        return lib.saap_adam_update(a["p"], K, V, out, ctypes.c_size_t(a["n"]), i32(a["step"]), f32(1e-3), f32(a["b1"]),
                                    f32(a["b2"]), f32(1e-8), None)

    assert adam(p=None) == -1 and adam(n=0) == -1 and adam(step=0) == -1 and adam(b1=1.0) == -1 and adam(b2=-0.1) == -1


def test_invalid_arguments_of_select_attend_prefill_and_the_probe_are_rejected_on_the_host(lib):
    """Selection inside the attention launch, prefill-time sparse attention, the matrix-rate probe and the
    no-allocation entry point: every argument check fails before anything is enqueued."""
    logits, q, K, V, off, ln, sel, out, lse, ws, ks, vs, idx, pos0 = _fake(14)
    i32, f32 = ctypes.c_int32, ctypes.c_float
    big, small = ctypes.c_size_t(1 << 30), ctypes.c_size_t(1024)

    def attend(**kw):
        a = dict(logits=logits, off=off, sel=sel, nprobe=4, Hq=4, Hkv=1, Ncap=1000, B=64, d=128, dt=1, odt=0, wsb=big)
        a.update(kw)
        return lib.saap_select_attend(a["logits"], q, K, V, a["off"], ln, i32(a["nprobe"]), f32(0.1), a["sel"], out,
                                      i32(a["odt"]), lse, i32(1), i32(a["Hq"]), i32(a["Hkv"]), i32(a["Ncap"]), i32(a["B"]),
                                      i32(a["d"]), i32(a["dt"]), ws, a["wsb"], None)

    assert attend(logits=None) == -1 and attend(off=None) == -1 and attend(sel=None) == -1
    assert attend(nprobe=65) == -1 and attend(nprobe=-1) == -1 and attend(B=0) == -1 and attend(Ncap=0) == -1
    assert attend(odt=5) == -1
    assert attend(dt=2) == -2                                         # the 8-bit cache has an entry point of its own
    assert attend(logits=ctypes.c_void_p(4100)) == -1                 # rows of logits are read 16 bytes at a time
    assert attend(d=64) == -2 and attend(Hq=3) == -2
    assert attend(wsb=small) == -3

    def attend_w(res):
        return lib.saap_select_attend_windowed(logits, q, K, V, off, ln, i32(4), i32(res), f32(0.1), sel, out, i32(0), lse,
                                               i32(1), i32(4), i32(1), i32(1000), i32(64), i32(128), i32(1), ws, big, None)

    assert attend_w(3) == -1 and attend_w(65) == -1 and attend_w(-2) == -1   # the resident run is run B, or there is none

    def attend8(**kw):
        a = dict(ks=ks, vs=vs, nprobe=4, wsb=big)
        a.update(kw)
        return lib.saap_select_attend_fp8(logits, q, K, V, a["ks"], a["vs"], off, ln, i32(a["nprobe"]), f32(0.1), sel, out,
                                          i32(0), lse, i32(1), i32(4), i32(1), i32(1000), i32(64), i32(128), ws, a["wsb"], None)

    assert attend8(ks=None) == -1 and attend8(vs=None) == -1 and attend8(nprobe=65) == -1 and attend8(wsb=small) == -3

    def prefill(**kw):
        a = dict(K=K, idx=idx, pos0=pos0, sel=sel, nprobe=4, sink=1, recent=15, Tq=8, Nt=100, B=8, d=128, dt=1, wsb=big)
        a.update(kw)
        return lib.saap_prefill_sparse_attention(q, a["K"], V, K, V, off, ln, a["idx"], a["sel"], a["pos0"], i32(a["nprobe"]),
                                                 i32(a["sink"]), i32(a["recent"]), f32(0.1), out, i32(0), lse, i32(1), i32(4),
                                                 i32(1), i32(a["Tq"]), i32(a["Nt"]), i32(116), i32(a["B"]), i32(a["d"]),
                                                 i32(a["dt"]), ws, a["wsb"], None)

    assert prefill(K=None) == -1 and prefill(idx=None) == -1 and prefill(pos0=None) == -1 and prefill(sel=None) == -1
    assert prefill(Tq=0) == -1 and prefill(Nt=0) == -1 and prefill(nprobe=9) == -1 and prefill(sink=-1) == -1
    assert prefill(recent=-1) == -1 and prefill(dt=2) == -1
    assert prefill(d=64) == -2 and prefill(wsb=small) == -3

    flop = ctypes.c_double(0.0)

    def probe(**kw):
        a = dict(ops=q, bytes=4096, iters=10, per_cu=1, sink=out)
        a.update(kw)
        return lib.saap_mfma_rate_probe(a["ops"], ctypes.c_size_t(a["bytes"]), i32(a["iters"]), i32(a["per_cu"]), a["sink"],
                                        ctypes.byref(flop), None)

    assert probe(ops=None) == -1 and probe(sink=None) == -1 and probe(bytes=32) == -1 and probe(iters=0) == -1
    assert probe(per_cu=0) == -1 and probe(ops=ctypes.c_void_p(4100)) == -1

    def noalloc(**kw):
        a = dict(q=q, sel=sel, nprobe=4, mode=0, Hq=4, Hkv=1, B=8, d=128, dt=1)
        a.update(kw)
        return lib.saap_sparse_decode_attention_noalloc(a["q"], K, V, off, ln, a["sel"], i32(a["nprobe"]), i32(a["mode"]),
                                                        f32(0.1), out, i32(0), lse, i32(1), i32(a["Hq"]), i32(a["Hkv"]),
                                                        i32(100), i32(a["B"]), i32(a["d"]), i32(a["dt"]), None)

    assert noalloc(q=None) == -1 and noalloc(sel=None) == -1 and noalloc(nprobe=9) == -1 and noalloc(mode=3) == -1
    assert noalloc(d=64) == -2 and noalloc(Hq=3) == -2


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and not r.stdout.strip()
