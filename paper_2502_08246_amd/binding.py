"""ctypes binding of libsaap.so (declared in include/saap.h).

Argument marshalling only: shapes are read off the tensors, pointers and the current HIP
stream are handed to the C entry points, status codes become exceptions.  Outputs are
allocated with torch (device memory) unless the caller passes them in.
"""
from __future__ import annotations

import ctypes
import os

import torch

F32, BF16 = 0, 1
GROUP_SUM, INDEPENDENT = 0, 1
PROBS, LOGITS = 0, 1
OP_ASSIGN_KEYS, OP_BUILD_BUCKET_INDEX, OP_CLASSIFY_QUERIES, OP_SELECT_BUCKETS = 0, 1, 2, 3
OP_SPARSE_DECODE_ATTENTION, OP_DENSE_DECODE_ATTENTION, OP_APPEND_KEYS, OP_WINDOW_PUSH = 4, 5, 6, 7
OP_BUCKET_ATTENTION_MASS, OP_QUERY_MODEL_LOSS_GRADS, OP_BUCKET_ATTENTION_MASS_BATCH = 8, 9, 10
OP_PLANNED_DECODE_ATTENTION, OP_PREFILL_SPARSE_ATTENTION = 11, 12
WS_HEADER_BYTES = 65536

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsaap.so")
_lib = None

EXPORTS = (
    "saap_workspace_bytes", "saap_workspace_reset", "saap_status_string", "saap_device_compute_units",
    "saap_assign_keys", "saap_build_bucket_index", "saap_append_keys", "saap_classify_queries",
    "saap_select_buckets", "saap_sparse_decode_attention", "saap_dense_decode_attention", "saap_stream_read_probe", "saap_mfma_rate_probe",
    "saap_build_windowed_index", "saap_window_push", "saap_windowed_decode_attention",
    "saap_append_keys_fp8", "saap_window_push_fp8",
    "saap_select_buckets_from_logits", "saap_update_centroids", "saap_recompact_index",
    "saap_quantize_kv", "saap_sparse_decode_attention_fp8", "saap_dense_decode_attention_fp8",
    "saap_windowed_decode_attention_fp8",
    "saap_bucket_attention_mass", "saap_query_model_loss_grads", "saap_adam_update",
    "saap_bucket_attention_mass_batch", "saap_query_model_bn_loss_grads", "saap_fold_batch_norm",
    "saap_build_visit_plan", "saap_select_buckets_planned", "saap_planned_decode_attention",
    "saap_planned_decode_attention_fp8", "saap_visit_plan_bytes", "saap_sparse_decode_attention_noalloc",
    "saap_prefill_sparse_attention", "saap_classify_select", "saap_select_attend", "saap_select_attend_fp8", "saap_select_attend_windowed",
)


class SaapError(RuntimeError):
    def __init__(self, call: str, status: int):
        self.status = status
        super().__init__(f"{call} failed: {status_string(status)} ({status})")


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("S", "Hq", "Hkv", "N", "B", "nprobe", "d", "hidden", "dtype", "mode")]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built library; build it first (python -m paper_2502_08246_amd.build) if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build
            _build.build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.saap_workspace_bytes.restype = ctypes.c_size_t
        lib.saap_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.POINTER(_Shape)]
        lib.saap_status_string.restype = ctypes.c_char_p
        lib.saap_status_string.argtypes = [ctypes.c_int32]
        for name in EXPORTS[4:] + ("saap_workspace_reset", "saap_device_compute_units"):
            getattr(lib, name).restype = ctypes.c_int32
        lib.saap_visit_plan_bytes.restype = ctypes.c_size_t
        lib.saap_visit_plan_bytes.argtypes = [ctypes.c_int32] * 5
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().saap_status_string(int(status)).decode()


def _check(call: str, status: int) -> None:
    if status != 0:
        raise SaapError(call, status)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise ValueError("SAAP tensors must live in GPU memory; there is no CPU path")
    if not t.is_contiguous():
        raise ValueError("SAAP tensors must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _i32(v):
    return ctypes.c_int32(int(v))


def workspace_bytes(op: int, **shape) -> int:
    sh = _Shape(**{k: int(v) for k, v in shape.items()})
    return int(load_library().saap_workspace_bytes(op, ctypes.byref(sh)))


class _Workspace:
    """Device scratch handed to the calls.  Zero-filled once at allocation, which is what the
    header of arrival counters needs; grown (and zero-filled again) on demand.

    A HIP graph that captured a call holds the RAW ADDRESS of the buffer it was given.  A buffer that has
    been handed out is therefore never freed: when a larger one replaces it, the old one is kept alive, so a
    graph captured earlier still replays into memory that belongs to the workspace.  Growing while the
    current stream is capturing is refused (allocating there would also break the capture): run the call
    once eagerly first, or pass ws= explicitly."""

    def __init__(self):
        self.buf = None
        self.retired = []

    def get(self, nbytes: int, device) -> torch.Tensor:
        if self.buf is None or self.buf.numel() < nbytes or self.buf.device != torch.device(device):
            if torch.cuda.is_current_stream_capturing():
                raise RuntimeError("the shared SAAP workspace would have to grow during stream capture: call the "
                                   "operation once eagerly before capturing, or pass ws=")
            if self.buf is not None:
                self.retired.append(self.buf)
            self.buf = torch.zeros(max(nbytes, WS_HEADER_BYTES), dtype=torch.uint8, device=device)
        return self.buf


_default_ws = _Workspace()


def workspace(nbytes: int, device) -> torch.Tensor:
    """The binding's shared workspace buffer, at least nbytes long."""
    return _default_ws.get(nbytes, device)


def _ws(op, device, ws, **shape):
    need = workspace_bytes(op, **shape)
    if need == 0:
        raise SaapError("saap_workspace_bytes", -1)
    if ws is None:
        ws = workspace(need, device)
    return ws, ctypes.c_size_t(ws.numel())


def workspace_reset(ws: torch.Tensor) -> None:
    """Zeroes the header of a caller-provided workspace (needed once before its first use, or after a
    call was abandoned midway)."""
    st = load_library().saap_workspace_reset(_ptr(ws), ctypes.c_size_t(ws.numel()), _stream())
    _check("saap_workspace_reset", st)


def stream_read_probe(src: torch.Tensor, sink: torch.Tensor) -> None:
    """Measurement aid: one pass of non-temporal 16-byte loads over `src` (see saap_stream_read_probe)."""
    st = load_library().saap_stream_read_probe(_ptr(src), ctypes.c_size_t(src.numel() * src.element_size()), _ptr(sink),
                                               ctypes.c_size_t(sink.numel() * sink.element_size()), _stream())
    _check("saap_stream_read_probe", st)


def mfma_rate_probe(operands: torch.Tensor, iters: int, sink: torch.Tensor, wgs_per_cu: int = 2) -> float:
    """Measurement aid: enqueues the bare matrix-instruction loop on `operands` (bf16 values) and returns the
    floating-point operations of the launch (see saap_mfma_rate_probe)."""
    flop = ctypes.c_double(0.0)
    st = load_library().saap_mfma_rate_probe(_ptr(operands), ctypes.c_size_t(operands.numel() * operands.element_size()),
                                             ctypes.c_int32(iters), ctypes.c_int32(wgs_per_cu), _ptr(sink), ctypes.byref(flop),
                                             _stream())
    _check("saap_mfma_rate_probe", st)
    return flop.value


def assign_keys(x, centroids, bias=None, out=None, ws=None):
    """x [S,Hkv,N,d], centroids [Hkv,B,d], bias [Hkv,B] fp32 or None -> bucket_ids int32 [S,Hkv,N]."""
    S, Hkv, N, d = x.shape
    B = centroids.shape[1]
    if centroids.shape != (Hkv, B, d) or centroids.dtype != x.dtype:
        raise ValueError("centroids must be [Hkv,B,d] in the dtype of x")
    ids = out if out is not None else torch.empty(S, Hkv, N, dtype=torch.int32, device=x.device)
    ws, wsb = _ws(OP_ASSIGN_KEYS, x.device, ws, S=S, Hkv=Hkv, N=N, B=B, d=d)
    st = load_library().saap_assign_keys(_ptr(x), _ptr(centroids), _ptr(bias), _ptr(ids), _i32(S), _i32(Hkv),
                                         _i32(N), _i32(B), _i32(d), _i32(_dtype_code(x)), _ptr(ws), wsb, _stream())
    _check("saap_assign_keys", st)
    return ids


def build_bucket_index(bucket_ids, K, V, B, slack=0, ws=None):
    """-> off [S,Hkv,B+1], len [S,Hkv,B], idx [S,Hkv,Ncap] (int32), Ksorted, Vsorted [S,Hkv,Ncap,d]."""
    S, Hkv, N, d = K.shape
    Ncap = N + B * slack
    dev = K.device
    off = torch.empty(S, Hkv, B + 1, dtype=torch.int32, device=dev)
    ln = torch.empty(S, Hkv, B, dtype=torch.int32, device=dev)
    idx = torch.empty(S, Hkv, Ncap, dtype=torch.int32, device=dev)
    alloc = torch.zeros if slack > 0 else torch.empty
    Ks = alloc(S, Hkv, Ncap, d, dtype=K.dtype, device=dev)
    Vs = alloc(S, Hkv, Ncap, d, dtype=K.dtype, device=dev)
    ws, wsb = _ws(OP_BUILD_BUCKET_INDEX, dev, ws, S=S, Hkv=Hkv, N=N, B=B)
    st = load_library().saap_build_bucket_index(_ptr(bucket_ids), _ptr(K), _ptr(V), _ptr(off), _ptr(ln), _ptr(idx),
                                                _ptr(Ks), _ptr(Vs), _i32(S), _i32(Hkv), _i32(N), _i32(Ncap), _i32(B),
                                                _i32(d), _i32(_dtype_code(K)), _i32(slack), _ptr(ws), wsb, _stream())
    _check("saap_build_bucket_index", st)
    return off, ln, idx, Ks, Vs


def append_keys(x_new, k_new, v_new, pos_new, centroids, bias, off, ln, idx, Ks, Vs, overflow_flag=None, new_ids=None,
                ws=None):
    """In-place append of one key per (sequence, KV head). -> (new_bucket_ids [S,Hkv], overflow_flag [1])."""
    S, Hkv, d = x_new.shape
    B = centroids.shape[1]
    Ncap = idx.shape[2]
    dev = x_new.device
    if new_ids is None:
        new_ids = torch.empty(S, Hkv, dtype=torch.int32, device=dev)
    if overflow_flag is None:
        overflow_flag = torch.zeros(4, dtype=torch.int32, device=dev)
    ws, wsb = _ws(OP_APPEND_KEYS, dev, ws, S=S, Hkv=Hkv, B=B)
    st = load_library().saap_append_keys(_ptr(x_new), _ptr(k_new), _ptr(v_new), _ptr(pos_new), _ptr(centroids),
                                         _ptr(bias), _ptr(off), _ptr(ln), _ptr(idx), _ptr(Ks), _ptr(Vs),
                                         _ptr(new_ids), _ptr(overflow_flag), _i32(S), _i32(Hkv), _i32(Ncap), _i32(B),
                                         _i32(d), _i32(_dtype_code(x_new)), _ptr(ws), wsb, _stream())
    _check("saap_append_keys", st)
    return new_ids, overflow_flag


def _bf16_only(name, *tensors):
    for t in tensors:
        if t.dtype != torch.bfloat16:
            raise TypeError(f"{name}: bf16 features and rows expected, got {t.dtype}")


def append_keys_fp8(x_new, k_new, v_new, pos_new, centroids, bias, off, ln, idx, K8, V8, kscale, vscale,
                    overflow_flag=None, new_ids=None, ws=None):
    """append_keys on an 8-bit cache (K8, V8 uint8 with the scales of quantize_kv), in place."""
    _bf16_only("append_keys_fp8", x_new, k_new, v_new, centroids)
    S, Hkv, d = x_new.shape
    B = centroids.shape[1]
    Ncap = idx.shape[2]
    dev = x_new.device
    if new_ids is None:
        new_ids = torch.empty(S, Hkv, dtype=torch.int32, device=dev)
    if overflow_flag is None:
        overflow_flag = torch.zeros(4, dtype=torch.int32, device=dev)
    ws, wsb = _ws(OP_APPEND_KEYS, dev, ws, S=S, Hkv=Hkv, B=B)
    st = load_library().saap_append_keys_fp8(
        _ptr(x_new), _ptr(k_new), _ptr(v_new), _ptr(pos_new), _ptr(centroids), _ptr(bias), _ptr(off), _ptr(ln),
        _ptr(idx), _ptr(K8), _ptr(V8), _ptr(kscale), _ptr(vscale), _ptr(new_ids), _ptr(overflow_flag), _i32(S),
        _i32(Hkv), _i32(Ncap), _i32(B), _i32(d), _ptr(ws), wsb, _stream())
    _check("saap_append_keys_fp8", st)
    return new_ids, overflow_flag


def window_push_fp8(x_new, k_new, v_new, pos_new, centroids, bias, off, ln, idx, K8, V8, kscale, vscale, resident_ids,
                    n_sink, n_recent, overflow_flag=None, new_ids=None, ws=None):
    """window_push on an 8-bit cache (K8, V8 uint8 with the scales of quantize_kv), in place."""
    _bf16_only("window_push_fp8", x_new, k_new, v_new, centroids)
    S, Hkv, d = x_new.shape
    B = centroids.shape[1]
    Ncap = idx.shape[2]
    dev = x_new.device
    if new_ids is None:
        new_ids = torch.empty(S, Hkv, dtype=torch.int32, device=dev)
    if overflow_flag is None:
        overflow_flag = torch.zeros(4, dtype=torch.int32, device=dev)
    ws, wsb = _ws(OP_WINDOW_PUSH, dev, ws, S=S, Hkv=Hkv, B=B)
    st = load_library().saap_window_push_fp8(
        _ptr(x_new), _ptr(k_new), _ptr(v_new), _ptr(pos_new), _ptr(centroids), _ptr(bias), _ptr(off), _ptr(ln),
        _ptr(idx), _ptr(K8), _ptr(V8), _ptr(kscale), _ptr(vscale), _ptr(resident_ids), _ptr(new_ids),
        _ptr(overflow_flag), _i32(S), _i32(Hkv), _i32(Ncap), _i32(B), _i32(d), _i32(n_sink), _i32(n_recent), _ptr(ws),
        wsb, _stream())
    _check("saap_window_push_fp8", st)
    return new_ids, overflow_flag


def classify_queries(xq, W1, b1, W2, b2, Hkv, output_kind=PROBS, out=None, ws=None):
    """xq [S,Hq,d]; W1 [Hw,hidden,d]; W2 [Hw,B,hidden]; b1,b2 fp32 or None -> scores fp32 [S,Hq,B].
    W1 = None: the one-layer model z = W2 x + b2 with W2 [Hw,B,d]."""
    S, Hq, d = xq.shape
    if W1 is None:
        Hw, B, hidden = W2.shape[0], W2.shape[1], 0
        if W2.shape != (Hw, B, d) or W2.dtype != xq.dtype:
            raise ValueError("one-layer model: W2 must be [Hw,B,d] in xq's dtype")
        b1 = None
    else:
        Hw, hidden, _ = W1.shape
        B = W2.shape[1]
        if W2.shape != (Hw, B, hidden) or W1.dtype != xq.dtype or W2.dtype != xq.dtype:
            raise ValueError("W1 [Hw,hidden,d] and W2 [Hw,B,hidden] must match xq's dtype")
    scores = out if out is not None else torch.empty(S, Hq, B, dtype=torch.float32, device=xq.device)
    ws, wsb = _ws(OP_CLASSIFY_QUERIES, xq.device, ws, S=S, Hq=Hq, hidden=hidden)
    st = load_library().saap_classify_queries(_ptr(xq), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _i32(Hw),
                                              _ptr(scores), _i32(S), _i32(Hq), _i32(Hkv), _i32(d), _i32(hidden),
                                              _i32(B), _i32(_dtype_code(xq)), _i32(output_kind), _ptr(ws), wsb,
                                              _stream())
    _check("saap_classify_queries", st)
    return scores


def classify_select(xq, W1, b1, W2, b2, Hkv, nprobe, off=None, ln=None, resident_run=-1, want_plan=False, logits=None,
                    probs=None, out=None, plan=None, ws=None):
    """classify_queries (logits) + the group selection in one call. -> (logits [S,Hq,B], selected [S,Hkv,nprobe], plan
    or None).  want_plan (or plan=) also writes the lists' visit plan, which needs off and ln."""
    S, Hq, d = xq.shape
    Hw, hidden, _ = W1.shape
    B = W2.shape[1]
    if W2.shape != (Hw, B, hidden) or W1.dtype != xq.dtype or W2.dtype != xq.dtype:
        raise ValueError("W1 [Hw,hidden,d] and W2 [Hw,B,hidden] must match xq's dtype")
    dev = xq.device
    logits = logits if logits is not None else torch.empty(S, Hq, B, dtype=torch.float32, device=dev)
    sel = out if out is not None else torch.empty(S, Hkv, nprobe, dtype=torch.int32, device=dev)
    if want_plan or plan is not None:
        if off is None or ln is None:
            raise ValueError("a visit plan needs off and ln")
        plan = _plan_buffer(plan, S, Hq, Hkv, nprobe + (1 if resident_run >= 0 else 0), GROUP_SUM, dev)
    ws, wsb = _ws(OP_CLASSIFY_QUERIES, dev, ws, S=S, Hq=Hq, hidden=hidden)
    st = load_library().saap_classify_select(
        _ptr(xq), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _i32(Hw), _ptr(logits), _ptr(probs), _ptr(sel), _ptr(off),
        _ptr(ln), _i32(resident_run), _ptr(plan), _i32(S), _i32(Hq), _i32(Hkv), _i32(d), _i32(hidden), _i32(B),
        _i32(nprobe), _i32(_dtype_code(xq)), _ptr(ws), wsb, _stream())
    _check("saap_classify_select", st)
    return logits, sel, plan


def select_buckets(scores, Hkv, nprobe, mode=GROUP_SUM, out=None, ws=None):
    """scores fp32 [S,Hq,B] -> selected int32 [S,Hkv,nprobe] (GROUP_SUM) or [S,Hq,nprobe] (INDEPENDENT)."""
    S, Hq, B = scores.shape
    lists = Hq if mode == INDEPENDENT else Hkv
    sel = out if out is not None else torch.empty(S, lists, nprobe, dtype=torch.int32, device=scores.device)
    ws, wsb = _ws(OP_SELECT_BUCKETS, scores.device, ws)
    st = load_library().saap_select_buckets(_ptr(scores), _ptr(sel), _i32(S), _i32(Hq), _i32(Hkv), _i32(B),
                                            _i32(nprobe), _i32(mode), _ptr(ws), wsb, _stream())
    _check("saap_select_buckets", st)
    return sel


def select_buckets_from_logits(logits, Hkv, nprobe, mode=GROUP_SUM, probs=None, out=None, ws=None):
    """logits fp32 [S,Hq,B] (classify_queries with LOGITS) -> selected; `probs` (optional fp32 [S,Hq,B]) receives
    the softmax the selection was made from."""
    S, Hq, B = logits.shape
    lists = Hq if mode == INDEPENDENT else Hkv
    sel = out if out is not None else torch.empty(S, lists, nprobe, dtype=torch.int32, device=logits.device)
    ws, wsb = _ws(OP_SELECT_BUCKETS, logits.device, ws)
    st = load_library().saap_select_buckets_from_logits(_ptr(logits), _ptr(probs), _ptr(sel), _i32(S), _i32(Hq),
                                                        _i32(Hkv), _i32(B), _i32(nprobe), _i32(mode), _ptr(ws), wsb,
                                                        _stream())
    _check("saap_select_buckets_from_logits", st)
    return sel


def sparse_decode_attention(q, Ks, Vs, off, ln, selected, scale, mode=GROUP_SUM, out_dtype=torch.float32,
                            out=None, lse=None, ws=None):
    """q [S,Hq,d]; Ks,Vs [S,Hkv,Ncap,d]; off,ln from build_bucket_index; selected from select_buckets
    -> out [S,Hq,d] (out_dtype), lse fp32 [S,Hq]."""
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = Ks.shape
    B = ln.shape[2]
    nprobe = selected.shape[2]
    dev = q.device
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_SPARSE_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, mode=mode)
    st = load_library().saap_sparse_decode_attention(
        _ptr(q), _ptr(Ks), _ptr(Vs), _ptr(off), _ptr(ln), _ptr(selected) if nprobe > 0 else ctypes.c_void_p(0),
        _i32(nprobe), _i32(mode), ctypes.c_float(scale), _ptr(out), _i32(_dtype_code(out)), _ptr(lse), _i32(S),
        _i32(Hq), _i32(Hkv), _i32(Ncap), _i32(B), _i32(d), _i32(_dtype_code(q)), _ptr(ws), wsb, _stream())
    _check("saap_sparse_decode_attention", st)
    return out, lse


def visit_plan_ints(S, Hq, Hkv, nruns, mode=GROUP_SUM) -> int:
    """int32 elements of the visit plan of S*Hkv (GROUP_SUM) or S*Hq (INDEPENDENT) lists of nruns runs."""
    nbytes = int(load_library().saap_visit_plan_bytes(int(S), int(Hq), int(Hkv), int(nruns), int(mode)))
    if nbytes == 0:
        raise SaapError("saap_visit_plan_bytes", -1)
    return nbytes // 4


def _plan_buffer(plan, S, Hq, Hkv, nruns, mode, device):
    n = visit_plan_ints(S, Hq, Hkv, nruns, mode)
    if plan is None:
        plan = torch.empty(n, dtype=torch.int32, device=device)
    elif plan.dtype != torch.int32 or plan.numel() < n:
        raise ValueError(f"plan must be int32 with at least {n} elements")
    return plan


def build_visit_plan(selected, off, ln, Hq, mode=GROUP_SUM, resident_run=-1, plan=None):
    """selected int32 [S,lists,nprobe]; off [S,Hkv,runs+1], ln [S,Hkv,runs] -> plan (int32, flat)."""
    S, _, nprobe = selected.shape
    Hkv, runs = ln.shape[1], ln.shape[2]
    nruns = nprobe + (1 if resident_run >= 0 else 0)
    plan = _plan_buffer(plan, S, Hq, Hkv, nruns, mode, ln.device)
    st = load_library().saap_build_visit_plan(_ptr(selected) if nprobe > 0 else ctypes.c_void_p(0), _ptr(off), _ptr(ln),
                                              _i32(nprobe), _i32(mode), _i32(resident_run), _ptr(plan), _i32(S), _i32(Hq),
                                              _i32(Hkv), _i32(runs), _stream())
    _check("saap_build_visit_plan", st)
    return plan


def select_buckets_planned(scores, off, ln, Hkv, nprobe, input_kind=PROBS, mode=GROUP_SUM, resident_run=-1, probs=None,
                           out=None, plan=None, ws=None):
    """select_buckets (PROBS) or select_buckets_from_logits (LOGITS) that also writes the lists' visit plan.
    -> (selected, plan)."""
    S, Hq, B = scores.shape
    lists = Hq if mode == INDEPENDENT else Hkv
    sel = out if out is not None else torch.empty(S, lists, nprobe, dtype=torch.int32, device=scores.device)
    plan = _plan_buffer(plan, S, Hq, Hkv, nprobe + (1 if resident_run >= 0 else 0), mode, scores.device)
    ws, wsb = _ws(OP_SELECT_BUCKETS, scores.device, ws)
    st = load_library().saap_select_buckets_planned(
        _ptr(scores), _i32(input_kind), _ptr(probs), _ptr(off), _ptr(ln), _i32(resident_run), _ptr(sel), _ptr(plan),
        _i32(S), _i32(Hq), _i32(Hkv), _i32(B), _i32(nprobe), _i32(mode), _ptr(ws), wsb, _stream())
    _check("saap_select_buckets_planned", st)
    return sel, plan


def planned_decode_attention(q, Ks, Vs, plan, nruns, scale, mode=GROUP_SUM, out_dtype=torch.float32, out=None, lse=None,
                             ws=None):
    """q [S,Hq,d]; Ks,Vs [S,Hkv,Ncap,d]; plan from select_buckets_planned / build_visit_plan -> out, lse."""
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = Ks.shape
    dev = q.device
    _plan_buffer(plan, S, Hq, Hkv, nruns, mode, dev)
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_PLANNED_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, mode=mode)
    st = load_library().saap_planned_decode_attention(
        _ptr(q), _ptr(Ks), _ptr(Vs), _ptr(plan), _i32(nruns), _i32(mode), ctypes.c_float(scale), _ptr(out),
        _i32(_dtype_code(out)), _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(Ncap), _i32(d), _i32(_dtype_code(q)),
        _ptr(ws), wsb, _stream())
    _check("saap_planned_decode_attention", st)
    return out, lse


def planned_decode_attention_fp8(q, K8, V8, kscale, vscale, plan, nruns, scale, mode=GROUP_SUM, out_dtype=torch.float32,
                                 out=None, lse=None, ws=None):
    """planned_decode_attention on a cache written by quantize_kv; q bf16 [S,Hq,d]."""
    if q.dtype != torch.bfloat16 or K8.dtype != torch.uint8 or V8.dtype != torch.uint8:
        raise TypeError("q must be bf16, K8 and V8 uint8")
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = K8.shape
    dev = q.device
    _plan_buffer(plan, S, Hq, Hkv, nruns, mode, dev)
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_PLANNED_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, mode=mode)
    st = load_library().saap_planned_decode_attention_fp8(
        _ptr(q), _ptr(K8), _ptr(V8), _ptr(kscale), _ptr(vscale), _ptr(plan), _i32(nruns), _i32(mode),
        ctypes.c_float(scale), _ptr(out), _i32(_dtype_code(out)), _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(Ncap),
        _i32(d), _ptr(ws), wsb, _stream())
    _check("saap_planned_decode_attention_fp8", st)
    return out, lse


def prefill_sparse_attention(q, K, V, Ks, Vs, off, ln, idx, selected, pos0, n_sink, n_recent, scale,
                             out_dtype=torch.float32, out=None, lse=None, ws=None):
    """q [S,Tq,Hq,d]; position-ordered K,V [S,Hkv,Nt,d]; Ks,Vs,off,ln,idx from build_bucket_index over them;
    selected int32 [S,Hkv,Tq,nprobe]; pos0 int32 [S] -> out [S,Tq,Hq,d], lse fp32 [S,Tq,Hq]."""
    S, Tq, Hq, d = q.shape
    _, Hkv, Nt, _ = K.shape
    Ncap = Ks.shape[2]
    B = ln.shape[2]
    nprobe = selected.shape[3]
    dev = q.device
    out = out if out is not None else torch.empty(S, Tq, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Tq, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_PREFILL_SPARSE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, N=Tq, nprobe=nprobe)
    st = load_library().saap_prefill_sparse_attention(
        _ptr(q), _ptr(K), _ptr(V), _ptr(Ks), _ptr(Vs), _ptr(off), _ptr(ln), _ptr(idx),
        _ptr(selected) if nprobe > 0 else ctypes.c_void_p(0), _ptr(pos0), _i32(nprobe), _i32(n_sink), _i32(n_recent),
        ctypes.c_float(scale), _ptr(out), _i32(_dtype_code(out)), _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(Tq),
        _i32(Nt), _i32(Ncap), _i32(B), _i32(d), _i32(_dtype_code(q)), _ptr(ws), wsb, _stream())
    _check("saap_prefill_sparse_attention", st)
    return out, lse


def sparse_decode_attention_noalloc(q, Ks, Vs, off, ln, selected, scale, out, lse, mode=GROUP_SUM):
    """sparse_decode_attention without a workspace argument: the library's built-in scratch array serves.  The
    caller passes every output; nothing is allocated here or in the library."""
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = Ks.shape
    B = ln.shape[2]
    nprobe = selected.shape[2]
    st = load_library().saap_sparse_decode_attention_noalloc(
        _ptr(q), _ptr(Ks), _ptr(Vs), _ptr(off), _ptr(ln), _ptr(selected) if nprobe > 0 else ctypes.c_void_p(0),
        _i32(nprobe), _i32(mode), ctypes.c_float(scale), _ptr(out), _i32(_dtype_code(out)), _ptr(lse), _i32(S),
        _i32(Hq), _i32(Hkv), _i32(Ncap), _i32(B), _i32(d), _i32(_dtype_code(q)), _stream())
    _check("saap_sparse_decode_attention_noalloc", st)
    return out, lse


def bucket_attention_mass(q, Ks, off, ln, scale, out=None, lse=None, ws=None):
    """q [S,Hq,d]; Ks [S,Hkv,Ncap,d]; off, ln from build_bucket_index -> mass fp32 [S,Hq,B], lse fp32 [S,Hq]."""
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = Ks.shape
    B = ln.shape[2]
    dev = q.device
    mass = out if out is not None else torch.empty(S, Hq, B, dtype=torch.float32, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_BUCKET_ATTENTION_MASS, dev, ws, S=S, Hq=Hq, Hkv=Hkv, B=B)
    st = load_library().saap_bucket_attention_mass(
        _ptr(q), _ptr(Ks), _ptr(off), _ptr(ln), ctypes.c_float(scale), _ptr(mass), _ptr(lse), _i32(S), _i32(Hq),
        _i32(Hkv), _i32(Ncap), _i32(B), _i32(d), _i32(_dtype_code(q)), _ptr(ws), wsb, _stream())
    _check("saap_bucket_attention_mass", st)
    return mass, lse


def bucket_attention_mass_batch(q, Ks, off, ln, scale, out=None, lse=None, ws=None):
    """q [S,Hkv,R,d] bf16 (R queries per KV head); Ks [S,Hkv,Ncap,d] -> mass fp32 [S,Hkv,R,B], lse fp32 [S,Hkv,R]."""
    S, Hkv, R, d = q.shape
    Ncap = Ks.shape[2]
    B = ln.shape[2]
    dev = q.device
    mass = out if out is not None else torch.empty(S, Hkv, R, B, dtype=torch.float32, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hkv, R, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_BUCKET_ATTENTION_MASS_BATCH, dev, ws, S=S, Hkv=Hkv, N=R, B=B)
    st = load_library().saap_bucket_attention_mass_batch(
        _ptr(q), _ptr(Ks), _ptr(off), _ptr(ln), ctypes.c_float(scale), _ptr(mass), _ptr(lse), _i32(S), _i32(Hkv),
        _i32(R), _i32(Ncap), _i32(B), _i32(d), _i32(_dtype_code(q)), _ptr(ws), wsb, _stream())
    _check("saap_bucket_attention_mass_batch", st)
    return mass, lse


class _MlpF32(ctypes.Structure):
    _fields_ = [("W1", ctypes.c_void_p), ("b1", ctypes.c_void_p), ("W2", ctypes.c_void_p), ("b2", ctypes.c_void_p)]


def _mlp_struct(tensors):
    for t in tensors:
        if t.dtype != torch.float32:
            raise TypeError("the query model is trained in fp32")
    return _MlpF32(*(_ptr(t) for t in tensors))


def query_model_loss_grads(x, target, params, grads=None, loss=None, ws=None):
    """x [Hw,R,d] (bf16 or fp32), target fp32 [Hw,R,B], params = (W1 [Hw,hidden,d], b1 [Hw,hidden], W2 [Hw,B,hidden],
    b2 [Hw,B]) fp32 -> loss fp32 [Hw], grads (tuple shaped like params)."""
    Hw, R, d = x.shape
    W1, b1, W2, b2 = params
    hidden, B = W1.shape[1], W2.shape[1]
    if W1.shape != (Hw, hidden, d) or b1.shape != (Hw, hidden) or W2.shape != (Hw, B, hidden) or b2.shape != (Hw, B):
        raise ValueError("parameter shapes do not fit x")
    if target.shape != (Hw, R, B) or target.dtype != torch.float32:
        raise ValueError("target must be fp32 [Hw,R,B]")
    dev = x.device
    grads = grads if grads is not None else tuple(torch.empty_like(p) for p in params)
    loss = loss if loss is not None else torch.empty(Hw, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_QUERY_MODEL_LOSS_GRADS, dev, ws, Hkv=Hw, N=R, d=d, hidden=hidden, B=B)
    ps, gs = _mlp_struct(params), _mlp_struct(grads)
    st = load_library().saap_query_model_loss_grads(
        _ptr(x), _ptr(target), ctypes.byref(ps), ctypes.byref(gs), _ptr(loss), _i32(Hw), _i32(R), _i32(d), _i32(hidden),
        _i32(B), _i32(_dtype_code(x)), _ptr(ws), wsb, _stream())
    _check("saap_query_model_loss_grads", st)
    return loss, grads


class _BatchNormF32(ctypes.Structure):
    _fields_ = [("gamma", ctypes.c_void_p), ("beta", ctypes.c_void_p), ("grad_gamma", ctypes.c_void_p),
                ("grad_beta", ctypes.c_void_p), ("running_mean", ctypes.c_void_p), ("running_var", ctypes.c_void_p),
                ("momentum", ctypes.c_float), ("eps", ctypes.c_float)]


def query_model_bn_loss_grads(x, target, params, gamma, beta, running_mean=None, running_var=None, momentum=0.1, eps=1e-5,
                              grads=None, grad_gamma=None, grad_beta=None, loss=None, ws=None):
    """query_model_loss_grads for the model with batch normalisation of the hidden layer; gamma, beta [Hw,hidden]
    fp32; running_mean / running_var (both or neither) are updated in place.
    -> loss [Hw], grads (dW1, db1, dW2, db2), grad_gamma, grad_beta."""
    Hw, R, d = x.shape
    W1, b1, W2, b2 = params
    hidden, B = W1.shape[1], W2.shape[1]
    if W1.shape != (Hw, hidden, d) or b1.shape != (Hw, hidden) or W2.shape != (Hw, B, hidden) or b2.shape != (Hw, B):
        raise ValueError("parameter shapes do not fit x")
    if target.shape != (Hw, R, B) or target.dtype != torch.float32:
        raise ValueError("target must be fp32 [Hw,R,B]")
    for t in (gamma, beta, running_mean, running_var):
        if t is not None and (t.shape != (Hw, hidden) or t.dtype != torch.float32):
            raise ValueError("gamma, beta and the running statistics must be fp32 [Hw,hidden]")
    dev = x.device
    grads = grads if grads is not None else tuple(torch.empty_like(p) for p in params)
    grad_gamma = grad_gamma if grad_gamma is not None else torch.empty_like(gamma)
    grad_beta = grad_beta if grad_beta is not None else torch.empty_like(beta)
    loss = loss if loss is not None else torch.empty(Hw, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_QUERY_MODEL_LOSS_GRADS, dev, ws, Hkv=Hw, N=R, d=d, hidden=hidden, B=B)
    ps, gs = _mlp_struct(params), _mlp_struct(grads)
    bn = _BatchNormF32(_ptr(gamma), _ptr(beta), _ptr(grad_gamma), _ptr(grad_beta), _ptr(running_mean), _ptr(running_var),
                       momentum, eps)
    st = load_library().saap_query_model_bn_loss_grads(
        _ptr(x), _ptr(target), ctypes.byref(ps), ctypes.byref(gs), ctypes.byref(bn), _ptr(loss), _i32(Hw), _i32(R),
        _i32(d), _i32(hidden), _i32(B), _i32(_dtype_code(x)), _ptr(ws), wsb, _stream())
    _check("saap_query_model_bn_loss_grads", st)
    return loss, grads, grad_gamma, grad_beta


def fold_batch_norm(W1, b1, gamma, beta, running_mean, running_var, eps=1e-5, out_dtype=torch.bfloat16):
    """-> (W1' [Hw,hidden,d] out_dtype, b1' fp32): the inference form of the normalised first layer."""
    Hw, hidden, d = W1.shape
    for t in (W1, b1, gamma, beta, running_mean, running_var):
        if t.dtype != torch.float32:
            raise TypeError("fold_batch_norm takes fp32 tensors")
    W1o = torch.empty(Hw, hidden, d, dtype=out_dtype, device=W1.device)
    b1o = torch.empty(Hw, hidden, dtype=torch.float32, device=W1.device)
    st = load_library().saap_fold_batch_norm(_ptr(W1), _ptr(b1), _ptr(gamma), _ptr(beta), _ptr(running_mean),
                                             _ptr(running_var), ctypes.c_float(eps), _ptr(W1o), _ptr(b1o), _i32(Hw),
                                             _i32(hidden), _i32(d), _i32(_dtype_code(W1o)), _stream())
    _check("saap_fold_batch_norm", st)
    return W1o, b1o


def adam_update(param, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam step on one fp32 tensor, in place (param, m, v)."""
    for t in (param, grad, m, v):
        if t.dtype != torch.float32 or t.numel() != param.numel():
            raise TypeError("adam_update works on fp32 tensors of one size")
    st = load_library().saap_adam_update(_ptr(param), _ptr(grad), _ptr(m), _ptr(v), ctypes.c_size_t(param.numel()),
                                         _i32(step), ctypes.c_float(lr), ctypes.c_float(beta1), ctypes.c_float(beta2),
                                         ctypes.c_float(eps), _stream())
    _check("saap_adam_update", st)


def quantize_kv(Ks, Vs, ws=None):
    """Ks, Vs [S,Hkv,Ncap,d] (bucket-sorted) -> K8, V8 uint8 [S,Hkv,Ncap,d] (OCP FP8 E4M3 codes),
    kscale, vscale fp32 [S,Hkv] (one power of two per unit)."""
    S, Hkv, Ncap, d = Ks.shape
    dev = Ks.device
    K8 = torch.empty(S, Hkv, Ncap, d, dtype=torch.uint8, device=dev)
    V8 = torch.empty(S, Hkv, Ncap, d, dtype=torch.uint8, device=dev)
    ks = torch.empty(S, Hkv, dtype=torch.float32, device=dev)
    vs = torch.empty(S, Hkv, dtype=torch.float32, device=dev)
    if ws is None:
        ws = workspace(WS_HEADER_BYTES, dev)
    st = load_library().saap_quantize_kv(_ptr(Ks), _ptr(Vs), _ptr(K8), _ptr(V8), _ptr(ks), _ptr(vs), _i32(S), _i32(Hkv),
                                         _i32(Ncap), _i32(d), _i32(_dtype_code(Ks)), _ptr(ws),
                                         ctypes.c_size_t(ws.numel()), _stream())
    _check("saap_quantize_kv", st)
    return K8, V8, ks, vs


def sparse_decode_attention_fp8(q, K8, V8, kscale, vscale, off, ln, selected, scale, mode=GROUP_SUM,
                                out_dtype=torch.float32, out=None, lse=None, ws=None):
    """sparse_decode_attention on a cache written by quantize_kv; q bf16 [S,Hq,d]."""
    if q.dtype != torch.bfloat16 or K8.dtype != torch.uint8 or V8.dtype != torch.uint8:
        raise TypeError("q must be bf16, K8 and V8 uint8")
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = K8.shape
    B = ln.shape[2]
    nprobe = selected.shape[2]
    dev = q.device
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_SPARSE_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, mode=mode)
    st = load_library().saap_sparse_decode_attention_fp8(
        _ptr(q), _ptr(K8), _ptr(V8), _ptr(kscale), _ptr(vscale), _ptr(off), _ptr(ln),
        _ptr(selected) if nprobe > 0 else ctypes.c_void_p(0), _i32(nprobe), _i32(mode), ctypes.c_float(scale),
        _ptr(out), _i32(_dtype_code(out)), _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(Ncap), _i32(B), _i32(d),
        _ptr(ws), wsb, _stream())
    _check("saap_sparse_decode_attention_fp8", st)
    return out, lse


def select_attend(logits, q, Ks, Vs, off, ln, nprobe, scale, out_dtype=torch.float32, selected=None, out=None,
                  lse=None, ws=None, resident_run=-1):
    """select_buckets_from_logits + sparse_decode_attention in one call (one launch where the library can):
    logits fp32 [S,Hq,B] -> (selected int32 [S,Hkv,nprobe], out [S,Hq,d], lse fp32 [S,Hq]).  With
    resident_run = B (an index from build_windowed_index: off [S,Hkv,B+2], ln [S,Hkv,B+1]) the always-visited run
    is attended too, as by windowed_decode_attention."""
    if resident_run >= 0:
        return _select_attend_windowed(logits, q, Ks, Vs, off, ln, nprobe, resident_run, scale, out_dtype, selected, out,
                                       lse, ws)
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = Ks.shape
    B = ln.shape[2]
    dev = q.device
    selected = selected if selected is not None else torch.empty(S, Hkv, nprobe, dtype=torch.int32, device=dev)
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_SPARSE_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, mode=GROUP_SUM)
    st = load_library().saap_select_attend(
        _ptr(logits), _ptr(q), _ptr(Ks), _ptr(Vs), _ptr(off), _ptr(ln), _i32(nprobe), ctypes.c_float(scale),
        _ptr(selected) if nprobe > 0 else ctypes.c_void_p(0), _ptr(out), _i32(_dtype_code(out)), _ptr(lse), _i32(S),
        _i32(Hq), _i32(Hkv), _i32(Ncap), _i32(B), _i32(d), _i32(_dtype_code(q)), _ptr(ws), wsb, _stream())
    _check("saap_select_attend", st)
    return selected, out, lse


def _select_attend_windowed(logits, q, Ks, Vs, off, ln, nprobe, resident_run, scale, out_dtype, selected, out, lse, ws):
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = Ks.shape
    B = ln.shape[2] - 1
    dev = q.device
    selected = selected if selected is not None else torch.empty(S, Hkv, nprobe, dtype=torch.int32, device=dev)
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_SPARSE_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, mode=GROUP_SUM)
    st = load_library().saap_select_attend_windowed(
        _ptr(logits), _ptr(q), _ptr(Ks), _ptr(Vs), _ptr(off), _ptr(ln), _i32(nprobe), _i32(resident_run),
        ctypes.c_float(scale), _ptr(selected) if nprobe > 0 else ctypes.c_void_p(0), _ptr(out), _i32(_dtype_code(out)),
        _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(Ncap), _i32(B), _i32(d), _i32(_dtype_code(q)), _ptr(ws), wsb,
        _stream())
    _check("saap_select_attend_windowed", st)
    return selected, out, lse


def select_attend_fp8(logits, q, K8, V8, kscale, vscale, off, ln, nprobe, scale, out_dtype=torch.float32,
                      selected=None, out=None, lse=None, ws=None):
    """select_attend on a cache written by quantize_kv; q bf16 [S,Hq,d]."""
    if q.dtype != torch.bfloat16 or K8.dtype != torch.uint8 or V8.dtype != torch.uint8:
        raise TypeError("q must be bf16, K8 and V8 uint8")
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = K8.shape
    B = ln.shape[2]
    dev = q.device
    selected = selected if selected is not None else torch.empty(S, Hkv, nprobe, dtype=torch.int32, device=dev)
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_SPARSE_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, mode=GROUP_SUM)
    st = load_library().saap_select_attend_fp8(
        _ptr(logits), _ptr(q), _ptr(K8), _ptr(V8), _ptr(kscale), _ptr(vscale), _ptr(off), _ptr(ln), _i32(nprobe),
        ctypes.c_float(scale), _ptr(selected) if nprobe > 0 else ctypes.c_void_p(0), _ptr(out), _i32(_dtype_code(out)),
        _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(Ncap), _i32(B), _i32(d), _ptr(ws), wsb, _stream())
    _check("saap_select_attend_fp8", st)
    return selected, out, lse


def dense_decode_attention_fp8(q, K8, V8, kscale, vscale, scale, off=None, ln=None, out_dtype=torch.float32,
                               out=None, lse=None, ws=None):
    """dense_decode_attention on 8-bit K/V (packed, or a bucket-sorted cache with off/ln); q bf16."""
    if q.dtype != torch.bfloat16 or K8.dtype != torch.uint8 or V8.dtype != torch.uint8:
        raise TypeError("q must be bf16, K8 and V8 uint8")
    S, Hq, d = q.shape
    _, Hkv, N, _ = K8.shape
    B = ln.shape[2] if ln is not None else 0
    dev = q.device
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_DENSE_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv)
    st = load_library().saap_dense_decode_attention_fp8(
        _ptr(q), _ptr(K8), _ptr(V8), _ptr(kscale), _ptr(vscale), _ptr(off), _ptr(ln), _i32(B), ctypes.c_float(scale),
        _ptr(out), _i32(_dtype_code(out)), _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(N), _i32(d), _ptr(ws), wsb,
        _stream())
    _check("saap_dense_decode_attention_fp8", st)
    return out, lse


def build_windowed_index(bucket_ids, K, V, B, slack, n_sink, n_recent, ws=None):
    """Index with a resident run of W = n_sink + n_recent slots behind the B buckets.
    -> off [S,Hkv,B+2], len [S,Hkv,B+1], idx [S,Hkv,Ncap], Ksorted, Vsorted [S,Hkv,Ncap,d], resident_ids [S,Hkv,W]."""
    S, Hkv, N, d = K.shape
    W = n_sink + n_recent
    Ncap = max(N - W, 0) + B * slack + W
    dev = K.device
    off = torch.empty(S, Hkv, B + 2, dtype=torch.int32, device=dev)
    ln = torch.empty(S, Hkv, B + 1, dtype=torch.int32, device=dev)
    idx = torch.empty(S, Hkv, Ncap, dtype=torch.int32, device=dev)
    Ks = torch.zeros(S, Hkv, Ncap, d, dtype=K.dtype, device=dev)
    Vs = torch.zeros(S, Hkv, Ncap, d, dtype=K.dtype, device=dev)
    res = torch.empty(S, Hkv, max(W, 1), dtype=torch.int32, device=dev)[:, :, :W]
    ws, wsb = _ws(OP_BUILD_BUCKET_INDEX, dev, ws, S=S, Hkv=Hkv, N=N, B=B)
    st = load_library().saap_build_windowed_index(
        _ptr(bucket_ids), _ptr(K), _ptr(V), _ptr(off), _ptr(ln), _ptr(idx), _ptr(Ks), _ptr(Vs), _ptr(res), _i32(S),
        _i32(Hkv), _i32(N), _i32(Ncap), _i32(B), _i32(d), _i32(_dtype_code(K)), _i32(slack), _i32(n_sink),
        _i32(n_recent), _ptr(ws), wsb, _stream())
    _check("saap_build_windowed_index", st)
    return off, ln, idx, Ks, Vs, res


def window_push(x_new, k_new, v_new, pos_new, centroids, bias, off, ln, idx, Ks, Vs, resident_ids, n_sink, n_recent,
                overflow_flag=None, new_ids=None, ws=None):
    """In-place push of one key per (sequence, KV head) into the resident run; the displaced key moves
    to its bucket. -> (new_bucket_ids [S,Hkv], overflow_flag)."""
    S, Hkv, d = x_new.shape
    B = centroids.shape[1]
    Ncap = idx.shape[2]
    dev = x_new.device
    if new_ids is None:
        new_ids = torch.empty(S, Hkv, dtype=torch.int32, device=dev)
    if overflow_flag is None:
        overflow_flag = torch.zeros(4, dtype=torch.int32, device=dev)
    ws, wsb = _ws(OP_WINDOW_PUSH, dev, ws, S=S, Hkv=Hkv, B=B)
    st = load_library().saap_window_push(
        _ptr(x_new), _ptr(k_new), _ptr(v_new), _ptr(pos_new), _ptr(centroids), _ptr(bias), _ptr(off), _ptr(ln),
        _ptr(idx), _ptr(Ks), _ptr(Vs), _ptr(resident_ids), _ptr(new_ids), _ptr(overflow_flag), _i32(S), _i32(Hkv),
        _i32(Ncap), _i32(B), _i32(d), _i32(_dtype_code(x_new)), _i32(n_sink), _i32(n_recent), _ptr(ws), wsb, _stream())
    _check("saap_window_push", st)
    return new_ids, overflow_flag


def windowed_decode_attention(q, Ks, Vs, off, ln, selected, resident_run, scale, mode=GROUP_SUM,
                              out_dtype=torch.float32, out=None, lse=None, ws=None):
    """sparse_decode_attention over the selected buckets plus the always-visited run `resident_run`
    (-1 for none); off [S,Hkv,runs+1], ln [S,Hkv,runs]."""
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = Ks.shape
    runs = ln.shape[2]
    nprobe = selected.shape[2]
    dev = q.device
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_SPARSE_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, mode=mode)
    st = load_library().saap_windowed_decode_attention(
        _ptr(q), _ptr(Ks), _ptr(Vs), _ptr(off), _ptr(ln), _ptr(selected) if nprobe > 0 else ctypes.c_void_p(0),
        _i32(nprobe), _i32(mode), _i32(resident_run), ctypes.c_float(scale), _ptr(out), _i32(_dtype_code(out)),
        _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(Ncap), _i32(runs), _i32(d), _i32(_dtype_code(q)), _ptr(ws),
        wsb, _stream())
    _check("saap_windowed_decode_attention", st)
    return out, lse


def windowed_decode_attention_fp8(q, K8, V8, kscale, vscale, off, ln, selected, resident_run, scale, mode=GROUP_SUM,
                                  out_dtype=torch.float32, out=None, lse=None, ws=None):
    """windowed_decode_attention on a cache written by quantize_kv; q bf16 [S,Hq,d]."""
    if q.dtype != torch.bfloat16 or K8.dtype != torch.uint8 or V8.dtype != torch.uint8:
        raise TypeError("q must be bf16, K8 and V8 uint8")
    S, Hq, d = q.shape
    _, Hkv, Ncap, _ = K8.shape
    runs = ln.shape[2]
    nprobe = selected.shape[2]
    dev = q.device
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_SPARSE_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv, mode=mode)
    st = load_library().saap_windowed_decode_attention_fp8(
        _ptr(q), _ptr(K8), _ptr(V8), _ptr(kscale), _ptr(vscale), _ptr(off), _ptr(ln),
        _ptr(selected) if nprobe > 0 else ctypes.c_void_p(0), _i32(nprobe), _i32(mode), _i32(resident_run),
        ctypes.c_float(scale), _ptr(out), _i32(_dtype_code(out)), _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(Ncap),
        _i32(runs), _i32(d), _ptr(ws), wsb, _stream())
    _check("saap_windowed_decode_attention_fp8", st)
    return out, lse


def recompact_index(off, ln, idx, Ks, Vs, slack_new, Ncap_new, resident=False, overflow_flag=None):
    """Fresh slack behind every bucket without re-assignment. -> (off_new, idx_new, Ks_new, Vs_new, overflow_flag);
    ln stays valid."""
    S, Hkv, Ncap, d = Ks.shape
    runs = ln.shape[2]
    B = runs - (1 if resident else 0)
    dev = Ks.device
    off_new = torch.empty_like(off)
    idx_new = torch.empty(S, Hkv, Ncap_new, dtype=torch.int32, device=dev)
    Kn = torch.zeros(S, Hkv, Ncap_new, d, dtype=Ks.dtype, device=dev)
    Vn = torch.zeros(S, Hkv, Ncap_new, d, dtype=Ks.dtype, device=dev)
    if overflow_flag is None:
        overflow_flag = torch.zeros(4, dtype=torch.int32, device=dev)
    st = load_library().saap_recompact_index(_ptr(off), _ptr(ln), _ptr(idx), _ptr(Ks), _ptr(Vs), _ptr(off_new),
                                             _ptr(idx_new), _ptr(Kn), _ptr(Vn), _ptr(overflow_flag), _i32(S), _i32(Hkv),
                                             _i32(Ncap), _i32(Ncap_new), _i32(B), _i32(1 if resident else 0), _i32(d),
                                             _i32(_dtype_code(Ks)), _i32(slack_new), _stream())
    _check("saap_recompact_index", st)
    return off_new, idx_new, Kn, Vn, overflow_flag


def update_centroids(x_sorted, off, ln, centroids_old, normalize=True, out=None):
    """x_sorted [S,Hkv,Ncap,d] (features grouped by build_bucket_index), off, ln -> new centroids [Hkv,B,d]."""
    S, Hkv, Ncap, d = x_sorted.shape
    B = ln.shape[2]
    new = out if out is not None else torch.empty_like(centroids_old)
    st = load_library().saap_update_centroids(_ptr(x_sorted), _ptr(off), _ptr(ln), _ptr(centroids_old), _ptr(new),
                                              _i32(S), _i32(Hkv), _i32(Ncap), _i32(B), _i32(d),
                                              _i32(_dtype_code(x_sorted)), _i32(1 if normalize else 0), _stream())
    _check("saap_update_centroids", st)
    return new


def lloyd_iterations(x, centroids, iters, normalize=True):
    """`iters` iterations of (spherical) k-means on the device, composed of the library's calls: assign_keys,
    build_bucket_index on the features (grouping) and update_centroids.  x [S,Hkv,N,d], centroids [Hkv,B,d]
    (the initial ones; not modified) -> new centroids."""
    B = centroids.shape[1]
    c = centroids
    for _ in range(iters):
        ids = assign_keys(x, c)
        off, ln, _, xs, _ = build_bucket_index(ids, x, x, B, 0)
        c = update_centroids(xs, off, ln, c, normalize)
    return c


def dense_decode_attention(q, K, V, scale, off=None, ln=None, out_dtype=torch.float32, out=None, lse=None, ws=None):
    """q [S,Hq,d]; K,V [S,Hkv,N,d] (packed, or a bucket-sorted cache with off/ln) -> out, lse."""
    S, Hq, d = q.shape
    _, Hkv, N, _ = K.shape
    B = ln.shape[2] if ln is not None else 0
    dev = q.device
    out = out if out is not None else torch.empty(S, Hq, d, dtype=out_dtype, device=dev)
    lse = lse if lse is not None else torch.empty(S, Hq, dtype=torch.float32, device=dev)
    ws, wsb = _ws(OP_DENSE_DECODE_ATTENTION, dev, ws, S=S, Hq=Hq, Hkv=Hkv)
    st = load_library().saap_dense_decode_attention(
        _ptr(q), _ptr(K), _ptr(V), _ptr(off), _ptr(ln), _i32(B), ctypes.c_float(scale), _ptr(out),
        _i32(_dtype_code(out)), _ptr(lse), _i32(S), _i32(Hq), _i32(Hkv), _i32(N), _i32(d), _i32(_dtype_code(q)),
        _ptr(ws), wsb, _stream())
    _check("saap_dense_decode_attention", st)
    return out, lse
