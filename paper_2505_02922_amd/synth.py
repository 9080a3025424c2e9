"""Seeded synthetic inputs for the wave-index path (keys, values, queries).

This module only *generates inputs*: clusterable Gaussian-mixture keys, rotary
position encoding applied to them, Gaussian values, and queries aimed at a
mixture component.  It contains none of the method's arithmetic (no
clustering, no attention, no index layout) and is the one module that both the
CPU oracle's tests and the GPU path's tests / benchmark import.

The inputs stand in for the key/value activations of the long-context models
the paper evaluates (Llama-3-8B-1048K, Qwen2.5-7B; Evaluation, "Models"): keys
that cluster, coarse positional locality from rotary encoding (Wave Index,
"Lightweight Index Construction", footnote on RoPE), and a few dominant tokens
per query.

All randomness comes from `torch.Generator` objects seeded per (sequence, KV
head) unit, so a unit can be regenerated alone.  The random stream of a CPU
generator and of a GPU generator differ; a caller that needs the same numbers
on both sides generates once and copies.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Tuple

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and recipe of one synthetic workload (one transformer layer)."""
    name: str
    dtype: str                 # "f32" | "bf16" : storage type of q, K, V
    B: int                     # independent sequences
    Hq: int                    # query heads
    Hkv: int                   # key/value heads (Hq % Hkv == 0)
    d: int                     # head dimension
    N: int                     # context tokens
    n_sink: int
    n_local: int
    segment_len: int           # L
    clusters_per_segment: int  # k
    iters: int                 # T
    retrieve_frac: Optional[float]  # r = round(frac * m) ...
    retrieve_abs: Optional[int]     # ... or an absolute r
    n_components: int          # mixture components per KV head
    sigma: float               # per-token noise around the component mean
    rope_base: Optional[float]  # None: no rotary encoding
    outlier_token_frac: float = 0.0   # fraction of tokens scaled by outlier_token_scale
    outlier_token_scale: float = 1.0
    heavy_channels: int = 0    # channels with Student-t(3) heavy-tailed scales
    query_sigma: float = 0.5
    base_seed: int = 0

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def torch_dtype(self) -> torch.dtype:
        return {"f32": torch.float32, "bf16": torch.bfloat16}[self.dtype]

    def retrieve_count(self, m: int) -> int:
        """The workload's retrieval budget r for an index of m clusters per KV head: the
        absolute count if one is given, else the fraction of m rounded to the nearest integer
        (the paper's 150 of 8192 clusters = 1.8 %)."""
        if self.retrieve_abs is not None:
            return self.retrieve_abs
        return int(math.floor(self.retrieve_frac * m + 0.5))


def _wl(**kw) -> Workload:
    return Workload(**kw)


# The five workloads of the benchmark definition.  Average cluster size 16
# ("one centroid per 16 tokens", 8K-token segments, 10 iterations: Evaluation,
# "Parameters") gives k = L / 16.
WORKLOADS = {
    "tiny_f32": _wl(name="tiny_f32", dtype="f32", B=1, Hq=1, Hkv=1, d=64, N=4096,
                    n_sink=4, n_local=64, segment_len=2048, clusters_per_segment=128,
                    iters=10, retrieve_frac=None, retrieve_abs=16, n_components=128,
                    sigma=0.3, rope_base=None, outlier_token_frac=0.02,
                    outlier_token_scale=4.0),
    "llama8b_32k": _wl(name="llama8b_32k", dtype="bf16", B=1, Hq=32, Hkv=8, d=128, N=32768,
                       n_sink=4, n_local=1024, segment_len=8192, clusters_per_segment=512,
                       iters=10, retrieve_frac=0.018, retrieve_abs=None, n_components=2048,
                       sigma=0.25, rope_base=500000.0),
    "llama8b_120k_b16": _wl(name="llama8b_120k_b16", dtype="bf16", B=16, Hq=32, Hkv=8, d=128,
                            N=122880, n_sink=4, n_local=1024, segment_len=8192,
                            clusters_per_segment=512, iters=10, retrieve_frac=0.018,
                            retrieve_abs=None, n_components=2048, sigma=0.25,
                            rope_base=500000.0),
    "llama8b_1m": _wl(name="llama8b_1m", dtype="bf16", B=1, Hq=32, Hkv=8, d=128, N=1048576,
                      n_sink=4, n_local=1024, segment_len=8192, clusters_per_segment=512,
                      iters=10, retrieve_frac=0.01, retrieve_abs=None, n_components=65536,
                      sigma=0.25, rope_base=500000.0),
    "qwen7b_64k_b64": _wl(name="qwen7b_64k_b64", dtype="bf16", B=64, Hq=28, Hkv=4, d=128,
                          N=65536, n_sink=4, n_local=1024, segment_len=8192,
                          clusters_per_segment=512, iters=20, retrieve_frac=0.02,
                          retrieve_abs=None, n_components=2048, sigma=0.25,
                          rope_base=1000000.0, heavy_channels=4),
}


def unit_seed(wl: Workload, b: int, h_kv: int, stream: int = 0) -> int:
    """Seed of the generator for one (sequence, KV head) unit.  `stream`
    separates the key/value stream (0) from query streams (1 + query set)."""
    return (wl.base_seed * 1000003 + b * 1009 + h_kv) * 4099 + stream


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def rope(x: torch.Tensor, positions: torch.Tensor, base: float) -> torch.Tensor:
    """Rotary position encoding, half-split pairing: channel i is paired with
    channel i + d/2 and the pair is rotated by positions * base**(-2i/d)."""
    d = x.shape[-1]
    half = d // 2
    inv_freq = base ** (-torch.arange(half, device=x.device, dtype=torch.float64) * 2.0 / d)
    ang = positions.to(torch.float64)[:, None] * inv_freq[None, :]
    cos, sin = torch.cos(ang).to(x.dtype), torch.sin(ang).to(x.dtype)
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * cos - x2 * sin, x1 * sin + x2 * cos], dim=-1)


def _component_means(wl: Workload, b: int, h_kv: int, device) -> Tuple[torch.Tensor, torch.Tensor]:
    """Mixture means [n_components, d] and per-channel scales [d] of a unit."""
    g = _gen(unit_seed(wl, b, h_kv, 0), device)
    means = torch.randn(wl.n_components, wl.d, generator=g, device=device, dtype=torch.float32)
    scales = torch.ones(wl.d, device=device, dtype=torch.float32)
    if wl.heavy_channels > 0:
        # Student-t(3) = normal / sqrt(chi2_3 / 3); scale = max(1, 8 |t|) on a few channels.
        ch = torch.randperm(wl.d, generator=g, device=device)[: wl.heavy_channels]
        z = torch.randn(wl.heavy_channels, generator=g, device=device)
        chi = (torch.randn(wl.heavy_channels, 3, generator=g, device=device) ** 2).sum(-1)
        t = z / torch.sqrt(chi / 3.0)
        scales[ch] = torch.clamp(8.0 * t.abs(), min=1.0)
    return means, scales


def make_kv_unit(wl: Workload, b: int, h_kv: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Keys and values [N, d] of one (sequence, KV head) unit in the storage dtype."""
    means, scales = _component_means(wl, b, h_kv, device)
    g = _gen(unit_seed(wl, b, h_kv, 0) + 1, device)
    comp = torch.randint(0, wl.n_components, (wl.N,), generator=g, device=device)
    K = means[comp]
    K += wl.sigma * torch.randn(wl.N, wl.d, generator=g, device=device, dtype=torch.float32)
    if wl.outlier_token_frac > 0.0:
        u = torch.rand(wl.N, generator=g, device=device)
        K = torch.where((u < wl.outlier_token_frac)[:, None], K * wl.outlier_token_scale, K)
    K = K * scales[None, :]
    if wl.rope_base is not None:
        K = rope(K, torch.arange(wl.N, device=device), wl.rope_base)
    V = torch.randn(wl.N, wl.d, generator=g, device=device, dtype=torch.float32)
    dt = wl.torch_dtype()
    return K.to(dt), V.to(dt)


def make_kv(wl: Workload, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Keys and values [B, Hkv, N, d] in the storage dtype, filled unit by unit."""
    dt = wl.torch_dtype()
    K = torch.empty(wl.B, wl.Hkv, wl.N, wl.d, dtype=dt, device=device)
    V = torch.empty_like(K)
    for b in range(wl.B):
        for h in range(wl.Hkv):
            K[b, h], V[b, h] = make_kv_unit(wl, b, h, device)
    return K, V


def make_queries(wl: Workload, query_set: int = 0, device="cpu") -> torch.Tensor:
    """Queries [B, Hq, d]: each query head aims at one mixture component of its
    KV head (component mean + Gaussian noise), rotary-encoded at position N."""
    q = torch.empty(wl.B, wl.Hq, wl.d, dtype=torch.float32, device=device)
    for b in range(wl.B):
        for h in range(wl.Hkv):
            means, _ = _component_means(wl, b, h, device)
            g = _gen(unit_seed(wl, b, h, 1 + query_set), device)
            comp = torch.randint(0, wl.n_components, (wl.G,), generator=g, device=device)
            qq = means[comp] + wl.query_sigma * torch.randn(wl.G, wl.d, generator=g, device=device)
            if wl.rope_base is not None:
                qq = rope(qq, torch.full((wl.G,), wl.N, device=device), wl.rope_base)
            q[b, h * wl.G:(h + 1) * wl.G] = qq
    return q.to(wl.torch_dtype())


def scaled(wl: Workload, **changes) -> Workload:
    """A copy of `wl` with some fields replaced (smaller N, other G, ...)."""
    return dataclasses.replace(wl, **changes)
