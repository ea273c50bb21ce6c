"""Seeded synthetic inputs for the KV-cache context-switch path.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic and imports neither the GPU binding nor any checker, so the
same tensors can be handed to both.  The inputs stand in for the paper's
workloads (Llama2-7B / OPT-6.7B contexts built from its datasets, Sec. 4): only
the cache shapes, sizes and the presence of a few large-magnitude channels
(Sec. 5.2 notes extreme outliers in the KV cache) are reproduced.
"""
from __future__ import annotations

import math
from typing import NamedTuple

import torch


class Geometry(NamedTuple):
    """[L][2][Hkv][N][D] fp16 cache, chunks of T tokens, quantisation groups of G."""
    L: int
    Hkv: int
    Hq: int
    D: int
    N: int
    T: int
    G: int

    @property
    def n_chunks(self) -> int:
        return self.N // self.T

    @property
    def elements(self) -> int:
        return self.L * 2 * self.Hkv * self.N * self.D


class Workload(NamedTuple):
    name: str
    geom: Geometry
    seed: int
    n_queries: int          # 0 = no scoring in this workload
    outlier_channels: int   # per (layer, K|V, kv-head)
    outlier_scale: float
    bits_rule: str          # "uniform" | "scores-25-50-25" | "score-terciles"
    n_contexts: int = 1
    select_frac: float = 1.0


def _n_out(D: int) -> int:
    return max(1, round(0.01 * D))


# The five benchmark configurations (index = position in the configs list).
WORKLOADS = (
    Workload("tiny", Geometry(2, 4, 4, 64, 512, 16, 64), 0, 0, 4, 8.0, "uniform"),
    Workload("gemma2b-4k", Geometry(18, 1, 8, 256, 4096, 16, 64), 1, 0, _n_out(256), 10.0,
             "scores-25-50-25"),
    Workload("llama2-7b-4k", Geometry(32, 32, 32, 128, 4096, 16, 64), 2, 32, _n_out(128), 10.0,
             "score-terciles"),
    Workload("llama7b-2k-pool", Geometry(32, 32, 32, 128, 2048, 16, 64), 3, 0, _n_out(128), 10.0,
             "uniform", n_contexts=64, select_frac=0.4),
    Workload("llama3-8b-32k", Geometry(32, 8, 32, 128, 32768, 32, 128), 4, 64, _n_out(128), 10.0,
             "score-terciles"),
)

(_STREAM_KV, _STREAM_OUTLIER, _STREAM_Q, _STREAM_BITS, _STREAM_SUBSET, _STREAM_SCORES,
 _STREAM_KV_I8, _STREAM_WEIGHTS, _STREAM_HIDDEN) = range(9)


def _gen(seed: int, stream: int, device="cpu", context: int = 0) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 4096 + context) * 16 + stream)
    return g


def outlier_multiplier(geom: Geometry, seed: int, n_channels: int, scale: float,
                       context: int = 0) -> torch.Tensor:
    """fp32 [L][2][Hkv][1][D]: `scale` on n_channels seeded channels per slab row, 1 elsewhere."""
    g = _gen(seed, _STREAM_OUTLIER, "cpu", context)
    mult = torch.ones((geom.L, 2, geom.Hkv, 1, geom.D), dtype=torch.float32)
    for l in range(geom.L):
        for kv in range(2):
            for h in range(geom.Hkv):
                ch = torch.randperm(geom.D, generator=g)[:n_channels]
                mult[l, kv, h, 0, ch] = scale
    return mult


def make_kv(geom: Geometry, seed: int, device="cpu", outlier_channels: int = 0,
            outlier_scale: float = 1.0, context: int = 0) -> torch.Tensor:
    """fp16 cache [L][2][Hkv][N][D]: N(0,1) with a few channels per head scaled up."""
    dev = torch.device(device)
    g = _gen(seed, _STREAM_KV, dev, context)
    mult = outlier_multiplier(geom, seed, outlier_channels, outlier_scale, context).to(dev)
    kv = torch.empty((geom.L, 2, geom.Hkv, geom.N, geom.D), dtype=torch.float16, device=dev)
    for l in range(geom.L):   # layer by layer keeps the fp32 staging small
        x = torch.randn((2, geom.Hkv, geom.N, geom.D), generator=g, device=dev,
                        dtype=torch.float32)
        x.mul_(mult[l])
        kv[l].copy_(x)
    return kv


def make_kv_i8(geom: Geometry, seed: int, device="cpu", context: int = 0) -> torch.Tensor:
    """int8 cache [L][2][Hkv][N][D] as an engine with static per-channel 8-bit scales holds it
    (Sec. 4: the prototype keeps its KV cache in INT8): after such scaling every channel spans
    a similar integer range, so values are round(N(0,1) * 32) clipped to [-128, 127]."""
    dev = torch.device(device)
    g = _gen(seed, _STREAM_KV_I8, dev, context)
    kv = torch.empty((geom.L, 2, geom.Hkv, geom.N, geom.D), dtype=torch.int8, device=dev)
    for l in range(geom.L):
        x = torch.randn((2, geom.Hkv, geom.N, geom.D), generator=g, device=dev,
                        dtype=torch.float32)
        kv[l].copy_(x.mul_(32.0).round_().clamp_(-128, 127))
    return kv


def make_q(geom: Geometry, seed: int, n_queries: int, device="cpu") -> torch.Tensor:
    """fp16 queries [L][Hq][R][D] ~ N(0, std = 1/sqrt(D))."""
    dev = torch.device(device)
    g = _gen(seed, _STREAM_Q, dev)
    q = torch.randn((geom.L, geom.Hq, n_queries, geom.D), generator=g, device=dev,
                    dtype=torch.float32)
    q.mul_(1.0 / math.sqrt(geom.D))
    return q.to(torch.float16)


def draw_bits_uniform(n_chunks: int, seed: int, context: int = 0,
                      widths=(8, 4, 2)) -> torch.Tensor:
    """uint8 [n_chunks], each drawn uniformly from `widths`."""
    g = _gen(seed, _STREAM_BITS, "cpu", context)
    pick = torch.randint(0, len(widths), (n_chunks,), generator=g)
    return torch.tensor(widths, dtype=torch.uint8)[pick]


def draw_scores(n_chunks: int, seed: int) -> torch.Tensor:
    """fp32 [n_chunks] ~ U(0,1): stand-in tolerance scores where a workload has no query rows."""
    g = _gen(seed, _STREAM_SCORES, "cpu")
    return torch.rand((n_chunks,), generator=g, dtype=torch.float32)


def draw_subset(n_chunks: int, k: int, seed: int, draw: int = 0) -> torch.Tensor:
    """int32 [k]: k distinct chunk indices, ascending."""
    g = _gen(seed, _STREAM_SUBSET, "cpu", draw)
    return torch.randperm(n_chunks, generator=g)[:k].sort().values.to(torch.int32)


LAYER_WEIGHTS = ("w_norm1", "wq", "wk", "wv", "wo", "w_norm2", "w_gate", "w_up", "w_down")


def make_layer_weights(d_model: int, n_q_heads: int, n_kv_heads: int, head_dim: int, d_ff: int,
                       seed: int, device="cpu", layer: int = 0) -> dict:
    """Seeded random weights of one Llama-style block, fp16, stored [in][out]: projections
    ~ N(0, 1/sqrt(in)), norm gains ~ 1 + 0.1 N(0,1).  They stand in for trained weights, which
    are not available; only the shapes are those of the paper's models."""
    dev = torch.device(device)
    g = _gen(seed, _STREAM_WEIGHTS, dev, layer)
    shapes = {"w_norm1": (d_model,), "wq": (d_model, n_q_heads * head_dim),
              "wk": (d_model, n_kv_heads * head_dim), "wv": (d_model, n_kv_heads * head_dim),
              "wo": (n_q_heads * head_dim, d_model), "w_norm2": (d_model,),
              "w_gate": (d_model, d_ff), "w_up": (d_model, d_ff), "w_down": (d_ff, d_model)}
    out = {}
    for name in LAYER_WEIGHTS:
        shp = shapes[name]
        x = torch.randn(shp, generator=g, device=dev, dtype=torch.float32)
        if len(shp) == 1:
            x.mul_(0.1).add_(1.0)
        else:
            x.mul_(1.0 / math.sqrt(shp[0]))
        out[name] = x.to(torch.float16)
    return out


def make_hidden(n_tokens: int, d_model: int, seed: int, device="cpu") -> torch.Tensor:
    """fp16 hidden states [n_tokens][d_model] ~ N(0,1): the layer inputs of a token sequence."""
    dev = torch.device(device)
    g = _gen(seed, _STREAM_HIDDEN, dev)
    return torch.randn((n_tokens, d_model), generator=g, device=dev, dtype=torch.float32).to(torch.float16)
