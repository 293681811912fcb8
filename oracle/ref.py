"""ctypes front end of the CPU oracle (oracle/saap_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module.

Every function takes and returns numpy arrays on the host.  Floating-point
inputs are converted to float32 (exact for bf16 and fp32 data); attention
results come back in float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# SAAP_ORACLE_SRC names another copy of the source (the mutation test plants mistakes in such a copy
# and expects the pins to fail); the library is then built next to that copy.
_SRC = os.environ.get("SAAP_ORACLE_SRC") or os.path.join(_HERE, "saap_ref.c")
_LIB = os.path.join(os.path.dirname(os.path.abspath(_SRC)), "libsaap_ref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile saap_ref.c with gcc into oracle/libsaap_ref.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.ref_selectivity.restype = ctypes.c_double
        _lib.ref_get_threads.restype = ctypes.c_int
        _lib.ref_append_keys.restype = ctypes.c_int
        _lib.ref_window_push.restype = ctypes.c_int
        _lib.ref_recompact_index.restype = ctypes.c_int
        _lib.ref_fp8_e4m3_decode.restype = ctypes.c_float
        _lib.ref_fp8_e4m3_decode.argtypes = [ctypes.c_uint8]
        _lib.ref_fp8_e4m3_encode.restype = ctypes.c_uint8
        _lib.ref_fp8_e4m3_encode.argtypes = [ctypes.c_float]
    return _lib


def _f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def set_threads(n: int) -> None:
    lib().ref_set_threads(int(n))


def get_threads() -> int:
    return int(lib().ref_get_threads())


def assign_keys(x, centroids, bias=None):
    """x [S,Hkv,N,d], centroids [Hkv,B,d], bias [Hkv,B] or None -> ids int32 [S,Hkv,N]."""
    x = _f32(x)
    c = _f32(centroids)
    S, Hkv, N, d = x.shape
    B = c.shape[1]
    assert c.shape == (Hkv, B, d)
    bias = None if bias is None else _f32(bias)
    ids = np.empty((S, Hkv, N), dtype=np.int32)
    lib().ref_assign_keys(_p(x), _p(c), _p(bias), _p(ids), S, Hkv, N, B, d)
    return ids


def build_bucket_index(ids, K, V, B, slack=0):
    """-> off [S,Hkv,B+1], len [S,Hkv,B], idx [S,Hkv,Ncap], Ks, Vs [S,Hkv,Ncap,d] (float32)."""
    ids = _i32(ids)
    K = _f32(K)
    V = _f32(V)
    S, Hkv, N, d = K.shape
    Ncap = N + B * slack
    off = np.empty((S, Hkv, B + 1), dtype=np.int32)
    ln = np.empty((S, Hkv, B), dtype=np.int32)
    idx = np.empty((S, Hkv, Ncap), dtype=np.int32)
    Ks = np.zeros((S, Hkv, Ncap, d), dtype=np.float32)
    Vs = np.zeros((S, Hkv, Ncap, d), dtype=np.float32)
    lib().ref_build_bucket_index(_p(ids), _p(K), _p(V), _p(off), _p(ln), _p(idx), _p(Ks), _p(Vs),
                                 S, Hkv, N, Ncap, B, d, slack)
    return off, ln, idx, Ks, Vs


def append_keys(x_new, k_new, v_new, pos_new, centroids, bias, off, ln, idx, Ks, Vs):
    """In-place append on (ln, idx, Ks, Vs); -> (new_ids [S,Hkv], overflow flag)."""
    x_new = _f32(x_new)
    k_new = _f32(k_new)
    v_new = _f32(v_new)
    c = _f32(centroids)
    bias = None if bias is None else _f32(bias)
    pos = None if pos_new is None else _i32(pos_new)
    S, Hkv, d = x_new.shape
    B = c.shape[1]
    Ncap = idx.shape[2]
    for a, dt in ((off, np.int32), (ln, np.int32), (idx, np.int32), (Ks, np.float32), (Vs, np.float32)):
        assert a.dtype == dt and a.flags["C_CONTIGUOUS"]
    new_ids = np.empty((S, Hkv), dtype=np.int32)
    flag = lib().ref_append_keys(_p(x_new), _p(k_new), _p(v_new), _p(pos), _p(c), _p(bias), _p(off), _p(ln),
                                 _p(idx), _p(Ks), _p(Vs), _p(new_ids), S, Hkv, Ncap, B, d)
    return new_ids, int(flag)


def windowed_capacity(N, B, slack, n_sink, n_recent):
    """Rows of the sorted cache with a resident block: non-resident keys + slack + the block itself."""
    W = n_sink + n_recent
    return max(N - W, 0) + B * slack + W


def build_windowed_index(ids, K, V, B, slack, n_sink, n_recent):
    """-> off [S,Hkv,B+2], len [S,Hkv,B+1], idx [S,Hkv,Ncap], Ks, Vs [S,Hkv,Ncap,d], res_ids [S,Hkv,W]."""
    ids = _i32(ids)
    K = _f32(K)
    V = _f32(V)
    S, Hkv, N, d = K.shape
    W = n_sink + n_recent
    Ncap = windowed_capacity(N, B, slack, n_sink, n_recent)
    off = np.empty((S, Hkv, B + 2), dtype=np.int32)
    ln = np.empty((S, Hkv, B + 1), dtype=np.int32)
    idx = np.empty((S, Hkv, Ncap), dtype=np.int32)
    Ks = np.zeros((S, Hkv, Ncap, d), dtype=np.float32)
    Vs = np.zeros((S, Hkv, Ncap, d), dtype=np.float32)
    res = np.empty((S, Hkv, W), dtype=np.int32)
    lib().ref_build_windowed_index(_p(ids), _p(K), _p(V), _p(off), _p(ln), _p(idx), _p(Ks), _p(Vs), _p(res),
                                   S, Hkv, N, Ncap, B, d, slack, n_sink, n_recent)
    return off, ln, idx, Ks, Vs, res


def window_push(x_new, k_new, v_new, pos_new, centroids, bias, off, ln, idx, Ks, Vs, res_ids, n_sink, n_recent):
    """In-place push on (ln, idx, Ks, Vs, res_ids); -> (new_ids [S,Hkv], overflow flag)."""
    x_new = _f32(x_new)
    k_new = _f32(k_new)
    v_new = _f32(v_new)
    c = _f32(centroids)
    bias = None if bias is None else _f32(bias)
    pos = _i32(pos_new)
    S, Hkv, d = x_new.shape
    B = c.shape[1]
    Ncap = idx.shape[2]
    for a, dt in ((off, np.int32), (ln, np.int32), (idx, np.int32), (Ks, np.float32), (Vs, np.float32),
                  (res_ids, np.int32)):
        assert a.dtype == dt and a.flags["C_CONTIGUOUS"]
    assert off.shape[2] == B + 2 and ln.shape[2] == B + 1 and res_ids.shape[2] == n_sink + n_recent
    new_ids = np.empty((S, Hkv), dtype=np.int32)
    flag = lib().ref_window_push(_p(x_new), _p(k_new), _p(v_new), _p(pos), _p(c), _p(bias), _p(off), _p(ln),
                                 _p(idx), _p(Ks), _p(Vs), _p(res_ids), _p(new_ids), S, Hkv, Ncap, B, d,
                                 n_sink, n_recent)
    return new_ids, int(flag)


def windowed_decode_attention(q, K, V, ids, selected, n_sink, n_recent, scale, B, mode=0):
    """Position-ordered K,V [S,Hkv,Nt,d], ids [S,Hkv,Nt] -> out float64 [S,Hq,d], lse float64 [S,Hq]."""
    q = _f32(q)
    K = _f32(K)
    V = _f32(V)
    ids = _i32(ids)
    selected = _i32(selected)
    S, Hq, d = q.shape
    _, Hkv, Nt, _ = K.shape
    nprobe = selected.shape[2]
    out = np.empty((S, Hq, d), dtype=np.float64)
    lse = np.empty((S, Hq), dtype=np.float64)
    lib().ref_windowed_decode_attention(_p(q), _p(K), _p(V), _p(ids), _p(selected), nprobe, mode, n_sink,
                                        n_recent, ctypes.c_float(scale), _p(out), _p(lse), S, Hq, Hkv, Nt, B, d)
    return out, lse


def prefill_sparse_attention(q, K, V, ids, selected, pos0, n_sink, n_recent, scale, B):
    """q [S,Tq,Hq,d]; position-ordered K,V [S,Hkv,Nt,d], ids [S,Hkv,Nt]; selected [S,Hkv,Tq,nprobe]; pos0 [S]
    -> out float64 [S,Tq,Hq,d], lse float64 [S,Tq,Hq]."""
    q = _f32(q)
    K = _f32(K)
    V = _f32(V)
    ids = _i32(ids)
    selected = _i32(selected)
    pos0 = _i32(pos0)
    S, Tq, Hq, d = q.shape
    _, Hkv, Nt, _ = K.shape
    nprobe = selected.shape[3]
    assert selected.shape[:3] == (S, Hkv, Tq) and pos0.shape == (S,) and int(pos0.max()) + Tq <= Nt
    out = np.empty((S, Tq, Hq, d), dtype=np.float64)
    lse = np.empty((S, Tq, Hq), dtype=np.float64)
    lib().ref_prefill_sparse_attention(_p(q), _p(K), _p(V), _p(ids), _p(selected), _p(pos0), nprobe, n_sink, n_recent,
                                       ctypes.c_float(scale), _p(out), _p(lse), S, Hq, Hkv, Tq, Nt, B, d)
    return out, lse


def recompact_index(off, ln, idx, Ks, Vs, slack_new, Ncap_new, resident=False):
    """-> (off_new, idx_new, Ks_new, Vs_new, overflow flag); ln stays valid."""
    S, Hkv, Ncap, d = Ks.shape
    runs = ln.shape[2]
    B = runs - (1 if resident else 0)
    for a, dt in ((off, np.int32), (ln, np.int32), (idx, np.int32), (Ks, np.float32), (Vs, np.float32)):
        assert a.dtype == dt and a.flags["C_CONTIGUOUS"]
    off_new = np.zeros_like(off)
    idx_new = np.full((S, Hkv, Ncap_new), -1, dtype=np.int32)
    Kn = np.zeros((S, Hkv, Ncap_new, d), dtype=np.float32)
    Vn = np.zeros((S, Hkv, Ncap_new, d), dtype=np.float32)
    flag = lib().ref_recompact_index(_p(off), _p(ln), _p(idx), _p(Ks), _p(Vs), _p(off_new), _p(idx_new), _p(Kn), _p(Vn),
                                     S, Hkv, Ncap, Ncap_new, B, 1 if resident else 0, d, slack_new)
    return off_new, idx_new, Kn, Vn, int(flag)


def update_centroids(x, ids, centroids_old, normalize=True):
    """x [S,Hkv,N,d] position-ordered features, ids [S,Hkv,N] -> new centroids float64 [Hkv,B,d]."""
    x = _f32(x)
    ids = _i32(ids)
    c = _f32(centroids_old)
    S, Hkv, N, d = x.shape
    B = c.shape[1]
    out = np.empty((Hkv, B, d), dtype=np.float64)
    lib().ref_update_centroids(_p(x), _p(ids), _p(c), _p(out), S, Hkv, N, B, d, 1 if normalize else 0)
    return out


def fp8_e4m3_decode(code: int) -> float:
    return float(lib().ref_fp8_e4m3_decode(int(code)))


def fp8_e4m3_encode(x: float) -> int:
    return int(lib().ref_fp8_e4m3_encode(float(x)))


def quantize_fp8(x):
    """x [S,Hkv,rows,d] -> codes uint8 [S,Hkv,rows,d], scale float32 [S,Hkv] (one power of two per unit)."""
    x = _f32(x)
    S, Hkv, rows, d = x.shape
    codes = np.empty(x.shape, dtype=np.uint8)
    scale = np.empty((S, Hkv), dtype=np.float32)
    lib().ref_quantize_fp8(_p(x), _p(codes), _p(scale), ctypes.c_longlong(S * Hkv), ctypes.c_longlong(rows), d)
    return codes, scale


def quantize_fp8_scaled(x, scale):
    """x [S,Hkv,rows,d] with the units' scales [S,Hkv] given -> codes uint8, saturated at +-448."""
    x = _f32(x)
    scale = _f32(scale)
    S, Hkv, rows, d = x.shape
    assert scale.shape == (S, Hkv)
    codes = np.empty(x.shape, dtype=np.uint8)
    lib().ref_quantize_fp8_scaled(_p(x), _p(scale), _p(codes), ctypes.c_longlong(S * Hkv), ctypes.c_longlong(rows), d)
    return codes


def dequantize_fp8(codes, scale):
    """codes uint8 [S,Hkv,rows,d], scale [S,Hkv] -> float32 [S,Hkv,rows,d] = scale * value(code), exact."""
    codes = np.ascontiguousarray(np.asarray(codes, dtype=np.uint8))
    scale = _f32(scale)
    S, Hkv, rows, d = codes.shape
    x = np.empty(codes.shape, dtype=np.float32)
    lib().ref_dequantize_fp8(_p(codes), _p(scale), _p(x), ctypes.c_longlong(S * Hkv), ctypes.c_longlong(rows), d)
    return x


def classify_queries(xq, W1, b1, W2, b2, Hkv, output_kind=0):
    """xq [S,Hq,d]; W1 [Hw,hidden,d]; W2 [Hw,B,hidden] -> scores float32 [S,Hq,B].
    W1 = None: the one-layer model, W2 [Hw,B,d]."""
    xq = _f32(xq)
    W2 = _f32(W2)
    b2 = None if b2 is None else _f32(b2)
    S, Hq, d = xq.shape
    if W1 is None:
        Hw, B, hidden = W2.shape[0], W2.shape[1], 0
        assert W2.shape == (Hw, B, d) and Hw in (1, Hkv, Hq)
        b1 = None
    else:
        W1 = _f32(W1)
        b1 = None if b1 is None else _f32(b1)
        Hw, hidden, _ = W1.shape
        B = W2.shape[1]
        assert W2.shape == (Hw, B, hidden) and Hw in (1, Hkv, Hq)
    scores = np.empty((S, Hq, B), dtype=np.float32)
    lib().ref_classify_queries(_p(xq), _p(W1), _p(b1), _p(W2), _p(b2), Hw, _p(scores), S, Hq, Hkv, d,
                               hidden, B, output_kind)
    return scores


def select_buckets(scores, Hkv, nprobe, mode=0):
    """scores float32 [S,Hq,B] -> selected int32 [S,Hkv or Hq,nprobe]."""
    scores = _f32(scores)
    S, Hq, B = scores.shape
    lists = Hq if mode == 1 else Hkv
    sel = np.empty((S, lists, nprobe), dtype=np.int32)
    lib().ref_select_buckets(_p(scores), _p(sel), S, Hq, Hkv, B, nprobe, mode)
    return sel


def sparse_decode_attention(q, K, V, off, ln, idx, selected, scale, mode=0):
    """q [S,Hq,d]; K,V position-ordered [S,Hkv,Nrows,d]; -> out float64 [S,Hq,d], lse float64 [S,Hq]."""
    q = _f32(q)
    K = _f32(K)
    V = _f32(V)
    off = _i32(off)
    ln = _i32(ln)
    idx = _i32(idx)
    selected = _i32(selected)
    S, Hq, d = q.shape
    _, Hkv, Nrows, _ = K.shape
    B = ln.shape[2]
    Ncap = idx.shape[2]
    nprobe = selected.shape[2]
    if idx.size and int(idx.max()) >= Nrows:
        raise ValueError(f"idx names position {int(idx.max())}, K holds {Nrows} rows")
    out = np.empty((S, Hq, d), dtype=np.float64)
    lse = np.empty((S, Hq), dtype=np.float64)
    lib().ref_sparse_decode_attention(_p(q), _p(K), _p(V), _p(off), _p(ln), _p(idx), _p(selected), nprobe,
                                      mode, ctypes.c_float(scale), _p(out), _p(lse), S, Hq, Hkv, Nrows,
                                      Ncap, B, d)
    return out, lse


def dense_decode_attention(q, K, V, scale):
    q = _f32(q)
    K = _f32(K)
    V = _f32(V)
    S, Hq, d = q.shape
    _, Hkv, N, _ = K.shape
    out = np.empty((S, Hq, d), dtype=np.float64)
    lse = np.empty((S, Hq), dtype=np.float64)
    lib().ref_dense_decode_attention(_p(q), _p(K), _p(V), ctypes.c_float(scale), _p(out), _p(lse), S, Hq,
                                     Hkv, N, d)
    return out, lse


def bucket_attention_mass(q, K, ids, scale, B):
    """q [S,Hq,d], K [S,Hkv,N,d] position order, ids [S,Hkv,N] -> mass float64 [S,Hq,B]: the share of each
    query's softmax attention that falls into each bucket (the training target of the query model)."""
    q, K, ids = _f32(q), _f32(K), _i32(ids)
    S, Hq, d = q.shape
    _, Hkv, N, _ = K.shape
    mass = np.empty((S, Hq, B), dtype=np.float64)
    lib().ref_bucket_attention_mass(_p(q), _p(K), _p(ids), ctypes.c_float(scale), _p(mass), S, Hq, Hkv, N, B, d)
    return mass


def selectivity(ln, selected, n_keys):
    """ln [lists,B], selected [lists,nprobe] -> mean fraction of keys visited."""
    ln = _i32(ln)
    selected = _i32(selected)
    lists, B = ln.shape
    nprobe = selected.shape[1]
    return float(lib().ref_selectivity(_p(ln), _p(selected), lists, B, nprobe, ctypes.c_long(int(n_keys))))
