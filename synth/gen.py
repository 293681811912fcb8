"""Seeded synthetic inputs for the SAAP hot path (shared by the GPU tests, the
oracle tests and bench.py).

This module only DRAWS INPUTS: keys, values, queries, centroids and classifier
weights with the shapes and the qualitative structure of the paper's workload
(Llama-3.1-8B head geometry, Section 6.1; a constant offset shared by all keys
of a head and a query distribution that differs from the key distribution,
Section 3; unbalanced buckets, Section 3).  None of the method's own steps
(assignment, index build, classifier, selection, attention) is implemented
here, and nothing here is used to compute an expected value.

Everything is generated with torch on the requested device from an explicit
torch.Generator, so a (config, seed, device type) triple names one set of
tensors.  The GPU library and the oracle always consume the SAME materialised
tensors (the oracle receives a host copy), so the generator itself is never
part of a parity comparison.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

ROPE_THETA = 500000.0


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    S: int            # sequences
    Hq: int           # query heads
    Hkv: int          # KV heads
    N: int            # keys per KV head
    B: int            # buckets per KV head
    hidden: int       # classifier hidden width
    nprobe: int
    dtype: str        # "f32" or "bf16"
    d: int = 128
    alpha: float | None = None   # Dirichlet concentration of the mixture weights (None = uniform)
    lloyd_on_keys: bool = False  # config 0: centroids are trained on the keys themselves
    n_queries: int = 1           # decode queries (time steps) drawn per head

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five workloads of the benchmark spec, in order, and one more for context.
CONFIGS = {
    "cfg0_tiny_f32": Workload("cfg0_tiny_f32", S=1, Hq=1, Hkv=1, N=4096, B=64, hidden=256, nprobe=8,
                              dtype="f32", lloyd_on_keys=True, n_queries=16),
    "cfg1_llama8b_128k": Workload("cfg1_llama8b_128k", S=1, Hq=32, Hkv=8, N=131072, B=1024, hidden=512,
                                  nprobe=51, dtype="bf16"),
    "cfg2_llama8b_500k_skew": Workload("cfg2_llama8b_500k_skew", S=1, Hq=32, Hkv=8, N=500000, B=4096,
                                       hidden=512, nprobe=205, dtype="bf16", alpha=0.3),
    "cfg3_batch8_128k": Workload("cfg3_batch8_128k", S=8, Hq=32, Hkv=8, N=131072, B=1024, hidden=512,
                                 nprobe=51, dtype="bf16"),
    "cfg4_layer_262k": Workload("cfg4_layer_262k", S=1, Hq=32, Hkv=8, N=262144, B=2048, hidden=512,
                                nprobe=102, dtype="bf16"),
    # Not in BASELINE.json: the shape of the paper's own timing (Section 6.2 "Timings": one KV head
    # with its 4 query heads, 171k keys, 32 of 1024 buckets visited), for context beside its figures.
    "paper_timing_1head_171k": Workload("paper_timing_1head_171k", S=1, Hq=4, Hkv=1, N=171000, B=1024,
                                        hidden=512, nprobe=32, dtype="bf16"),
    # Not in the benchmark spec: the batched-decode workload with 32 sequences, i.e. a launch large enough
    # (0.85 GB of visited K/V) to show the attention kernel's streaming rate without its fixed cost.
    "batch32_128k": Workload("batch32_128k", S=32, Hq=32, Hkv=8, N=131072, B=1024, hidden=512,
                             nprobe=51, dtype="bf16"),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _gen(device, *seed_parts: int) -> torch.Generator:
    seed = 0x9E3779B97F4A7C15
    for p in seed_parts:
        seed = (seed ^ (int(p) + 0x632BE59BD9B4E019)) * 0x100000001B3 % (1 << 63)
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def rope(x: torch.Tensor, pos: torch.Tensor, theta: float = ROPE_THETA) -> torch.Tensor:
    """Rotary embedding on interleaved pairs (x[2i], x[2i+1]), angle pos * theta^(-2i/d),
    evaluated in float64.  x [..., n, d], pos [n] (or broadcastable)."""
    d = x.shape[-1]
    xd = x.to(torch.float64)
    i = torch.arange(d // 2, device=x.device, dtype=torch.float64)
    inv = theta ** (-2.0 * i / d)
    ang = pos.to(torch.float64).unsqueeze(-1) * inv
    c, s = torch.cos(ang), torch.sin(ang)
    a, b = xd[..., 0::2], xd[..., 1::2]
    out = torch.empty_like(xd)
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


def _mixture_weights(J: int, alpha, seed_parts, device) -> torch.Tensor:
    """Mixture weights: uniform, or one draw of Dirichlet(alpha * 1_J) (numpy PCG64, host)."""
    if alpha is None:
        return torch.full((J,), 1.0 / J, device=device, dtype=torch.float64)
    rng = np.random.Generator(np.random.PCG64([int(p) & 0xFFFFFFFF for p in seed_parts]))
    w = rng.dirichlet(np.full(J, float(alpha)))
    return torch.from_numpy(w).to(device)


def head_mixture(cfg: Workload, seed: int, h: int, device):
    """Parameters of one KV head's key mixture: centres, weights, shared offset."""
    g = _gen(device, seed, 11, h)
    J, d = cfg.B, cfg.d
    centres = 2.0 * torch.randn(J, d, generator=g, device=device, dtype=torch.float32)
    weights = _mixture_weights(J, cfg.alpha, (seed, 17, h), device)
    direction = torch.randn(d, generator=g, device=device, dtype=torch.float32)
    offset = 20.0 * direction / direction.norm()
    return centres, weights, offset


def draw_keys_raw(cfg: Workload, seed: int, s: int, h: int, n: int, device, stream_id: int = 0):
    """n pre-RoPE key vectors of head h: centre of a random component + N(0,I) + shared offset."""
    centres, weights, offset = head_mixture(cfg, seed, h, device)
    g = _gen(device, seed, 23, s, h, stream_id)
    comp = torch.multinomial(weights.to(torch.float32), n, replacement=True, generator=g)
    x = centres[comp] + torch.randn(n, cfg.d, generator=g, device=device, dtype=torch.float32) + offset
    return x


def make_cache(cfg: Workload, seed: int, device):
    """-> dict with
         x_keys [S,Hkv,N,d]  assignment features (keys before RoPE), cfg dtype
         K, V   [S,Hkv,N,d]  cached keys (after RoPE at positions 0..N-1) and values, cfg dtype
    """
    dt = torch_dtype(cfg.dtype)
    S, Hkv, N, d = cfg.S, cfg.Hkv, cfg.N, cfg.d
    xk = torch.empty(S, Hkv, N, d, device=device, dtype=dt)
    K = torch.empty(S, Hkv, N, d, device=device, dtype=dt)
    V = torch.empty(S, Hkv, N, d, device=device, dtype=dt)
    pos = torch.arange(N, device=device)
    for s in range(S):
        for h in range(Hkv):
            raw = draw_keys_raw(cfg, seed, s, h, N, device)
            xk[s, h] = raw.to(dt)
            K[s, h] = rope(raw, pos).to(dt)
            g = _gen(device, seed, 31, s, h)
            V[s, h] = torch.randn(N, d, generator=g, device=device, dtype=torch.float32).to(dt)
            del raw
    return {"x_keys": xk, "K": K, "V": V}


def lloyd(samples: torch.Tensor, B: int, iters: int = 5) -> torch.Tensor:
    """Stand-in for the paper's offline k-means (Appendix A): spherical Lloyd iterations,
    initialised from the first B samples.  float64; an empty bucket keeps its centroid."""
    x = samples.to(torch.float64)
    c = x[:B].clone()
    c = c / c.norm(dim=1, keepdim=True).clamp_min(1e-30)
    for _ in range(iters):
        a = (x @ c.T).argmax(dim=1)
        sums = torch.zeros_like(c).index_add_(0, a, x)
        cnt = torch.bincount(a, minlength=B).to(torch.float64)
        mean = sums / cnt.clamp_min(1.0).unsqueeze(1)
        mean = mean / mean.norm(dim=1, keepdim=True).clamp_min(1e-30)
        c = torch.where((cnt > 0).unsqueeze(1), mean, c)
    return c


def make_centroids(cfg: Workload, seed: int, device, cache=None, n_train: int = 65536) -> torch.Tensor:
    """-> centroids [Hkv,B,d] in cfg dtype.  Trained on a fresh draw from each head's key mixture
    (configs 1-4) or on the head's own keys (config 0)."""
    dt = torch_dtype(cfg.dtype)
    out = torch.empty(cfg.Hkv, cfg.B, cfg.d, device=device, dtype=dt)
    for h in range(cfg.Hkv):
        if cfg.lloyd_on_keys:
            assert cache is not None
            samples = cache["x_keys"][0, h].to(torch.float32)
        else:
            samples = draw_keys_raw(cfg, seed, 0, h, max(n_train, cfg.B), device, stream_id=977)
        out[h] = lloyd(samples, cfg.B).to(dt)
    return out


def make_queries(cfg: Workload, seed: int, device, n_steps: int | None = None):
    """-> xq [T,S,Hq,d] classifier features (queries before RoPE) and q [T,S,Hq,d] attention
    queries (after RoPE at position N+t), cfg dtype.  Queries come from their own mixture,
    without the key offset."""
    dt = torch_dtype(cfg.dtype)
    T = n_steps if n_steps is not None else cfg.n_queries
    S, Hq, d, J = cfg.S, cfg.Hq, cfg.d, cfg.B
    xq = torch.empty(T, S, Hq, d, device=device, dtype=dt)
    q = torch.empty(T, S, Hq, d, device=device, dtype=dt)
    pos = cfg.N + torch.arange(T, device=device)
    for hq in range(Hq):
        g = _gen(device, seed, 41, hq)
        centres = 2.0 * torch.randn(J, d, generator=g, device=device, dtype=torch.float32)
        comp = torch.randint(0, J, (T * S,), generator=g, device=device)
        raw = centres[comp] + torch.randn(T * S, d, generator=g, device=device, dtype=torch.float32)
        raw = raw.view(T, S, d)
        xq[:, :, hq] = raw.to(dt)
        q[:, :, hq] = rope(raw.transpose(0, 1), pos).transpose(0, 1).to(dt)
    return xq, q


def make_classifier(cfg: Workload, seed: int, device, Hw: int | None = None):
    """Random-init two-layer perceptron d -> hidden -> B, N(0, 1/fan_in) weights, zero biases.
    -> W1 [Hw,hidden,d], b1 [Hw,hidden] fp32, W2 [Hw,B,hidden], b2 [Hw,B] fp32."""
    dt = torch_dtype(cfg.dtype)
    Hw = cfg.Hkv if Hw is None else Hw
    g = _gen(device, seed, 53)
    W1 = (torch.randn(Hw, cfg.hidden, cfg.d, generator=g, device=device) / math.sqrt(cfg.d)).to(dt)
    W2 = (torch.randn(Hw, cfg.B, cfg.hidden, generator=g, device=device) / math.sqrt(cfg.hidden)).to(dt)
    b1 = torch.zeros(Hw, cfg.hidden, device=device, dtype=torch.float32)
    b2 = torch.zeros(Hw, cfg.B, device=device, dtype=torch.float32)
    return W1, b1, W2, b2


def to_host_f32(t: torch.Tensor):
    """Host float32 numpy copy (exact for bf16 and fp32 tensors)."""
    return t.detach().to("cpu").to(torch.float32).numpy()
