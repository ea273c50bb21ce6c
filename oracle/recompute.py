"""CPU oracle for the recompute of interleaved chunks (arXiv 2403.11805, Sec. 3.3,
"Making interleaved chunks recomputable" and its six-token example).

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain numpy in float64 on
the exact values of the fp16 inputs.  The layer is a Llama-style block (the
paper's example uses a Llama2-7B layer): RMSNorm, q/k/v projections, rotary
position encoding on q and k (pairs (i, i + D/2), angle pos * base^(-2i/D)),
causal attention with grouped query heads, output projection and residual,
RMSNorm, SwiGLU feed-forward and residual.  Weights are [in][out].

Two independent routes to the same numbers:
  layer_full        the block applied to a whole sequence, written as dense
                    matrix algebra with an explicit mask matrix;
  recompute_layer   the paper's procedure in its order: the tokens of the missing
                    chunks only, encoded with their GLOBAL positions; their K/V
                    inserted between the resident K/V; attention of the recomputed
                    queries over the recovered K/V under a causal mask by global
                    position; the tokens handed to the next layer.
K and V live in the fp16 cache, so both routes round them to fp16 before the
attention reads them: that rounding belongs to the data flow, not to an
implementation.  Nothing else is rounded.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class LayerDims:
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5


WEIGHT_NAMES = ("w_norm1", "wq", "wk", "wv", "wo", "w_norm2", "w_gate", "w_up", "w_down")


def _f64(a) -> np.ndarray:
    return np.asarray(a).astype(np.float64)


def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """Each row divided by the root of its mean square (+ eps), times the gain."""
    x = _f64(x)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * _f64(w)


def rope(u: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary encoding of u [tokens][heads][D] at integer positions pos [tokens]: the pair
    (u[i], u[i + D/2]) is rotated by the angle pos * base^(-2i/D)."""
    u = _f64(u)
    D = u.shape[-1]
    half = D // 2
    out = np.empty_like(u)
    for i in range(half):
        ang = _f64(pos) * (base ** (-2.0 * i / D))
        c, s = np.cos(ang)[:, None], np.sin(ang)[:, None]
        a, b = u[:, :, i], u[:, :, i + half]
        out[:, :, i] = a * c - b * s
        out[:, :, i + half] = b * c + a * s
    return out


def to_cache(a: np.ndarray) -> np.ndarray:
    """Values as the fp16 cache holds them."""
    return np.asarray(a, dtype=np.float64).astype(np.float16)


def _project(x, w, dims: LayerDims):
    xn = rmsnorm(x, w["w_norm1"], dims.rms_eps)
    M = xn.shape[0]
    q = (xn @ _f64(w["wq"])).reshape(M, dims.n_q_heads, dims.head_dim)
    k = (xn @ _f64(w["wk"])).reshape(M, dims.n_kv_heads, dims.head_dim)
    v = (xn @ _f64(w["wv"])).reshape(M, dims.n_kv_heads, dims.head_dim)
    return q, k, v


def _feed_forward(x1, w, dims: LayerDims):
    xn = rmsnorm(x1, w["w_norm2"], dims.rms_eps)
    g = xn @ _f64(w["w_gate"])
    u = xn @ _f64(w["w_up"])
    return x1 + ((g / (1.0 + np.exp(-g))) * u) @ _f64(w["w_down"])


def visible(pos_query: int, pos_key: int) -> bool:
    """Causal mask by global position: a token sees itself and every token before it."""
    return pos_key <= pos_query


def layer_full(x: np.ndarray, w: dict, dims: LayerDims):
    """The block on a whole sequence x [N][d_model] (token n at position n).
    -> (k_cache fp16 [Hkv][N][D], v_cache fp16 [Hkv][N][D], y float64 [N][d_model])."""
    N = x.shape[0]
    pos = np.arange(N)
    q, k, v = _project(x, w, dims)
    q = rope(q, pos, dims.rope_base)
    k = rope(k, pos, dims.rope_base)
    k16, v16 = to_cache(k), to_cache(v)
    kf, vf = _f64(k16), _f64(v16)
    mask = np.array([[visible(r, c) for c in range(N)] for r in range(N)])
    per = dims.n_q_heads // dims.n_kv_heads
    o = np.zeros((N, dims.n_q_heads, dims.head_dim))
    for h in range(dims.n_q_heads):
        g = h // per
        s = q[:, h, :] @ kf[:, g, :].T / np.sqrt(dims.head_dim)
        s = np.where(mask, s, -np.inf)
        a = np.exp(s - s.max(axis=1, keepdims=True))
        a /= a.sum(axis=1, keepdims=True)
        o[:, h, :] = a @ vf[:, g, :]
    x1 = _f64(x) + o.reshape(N, -1) @ _f64(w["wo"])
    y = _feed_forward(x1, w, dims)
    return (np.ascontiguousarray(k16.transpose(1, 0, 2)), np.ascontiguousarray(v16.transpose(1, 0, 2)), y)


def recompute_layer(x_missing: np.ndarray, chunk_idx, chunk_tokens: int, k_cache: np.ndarray,
                    v_cache: np.ndarray, w: dict, dims: LayerDims) -> np.ndarray:
    """Sec. 3.3, step by step.  x_missing [M][d_model]: the layer inputs of the tokens of the
    missing chunks (chunk_idx ascending, chunk_tokens tokens each).  k_cache / v_cache: fp16
    [Hkv][N][D] of this layer with the resident chunks in place; the missing chunks' entries
    are overwritten here.  -> y float64 [M][d_model], the tokens handed to the next layer."""
    T = chunk_tokens
    pos = np.concatenate([np.arange(c * T, (c + 1) * T) for c in chunk_idx])     # global positions
    M = len(pos)
    assert x_missing.shape[0] == M
    # recompute the missing tokens' q, k, v; encode q and k with the GLOBAL positions
    q, k, v = _project(x_missing, w, dims)
    q = rope(q, pos, dims.rope_base)
    k = rope(k, pos, dims.rope_base)
    # insert the recomputed K/V between the resident ones: the layer's K/V is whole again
    for m in range(M):
        k_cache[:, pos[m], :] = to_cache(k[m])
        v_cache[:, pos[m], :] = to_cache(v[m])
    # attention of the recomputed queries over the recovered K/V; a token keeps the tokens before it
    per = dims.n_q_heads // dims.n_kv_heads
    o = np.zeros((M, dims.n_q_heads, dims.head_dim))
    for m in range(M):
        p = int(pos[m])
        keep = [c for c in range(k_cache.shape[1]) if visible(p, c)]
        for h in range(dims.n_q_heads):
            g = h // per
            s = _f64(k_cache[g, keep, :]) @ q[m, h, :] / np.sqrt(dims.head_dim)
            a = np.exp(s - s.max())
            a /= a.sum()
            o[m, h, :] = a @ _f64(v_cache[g, keep, :])
    x1 = _f64(x_missing) + o.reshape(M, -1) @ _f64(w["wo"])
    return _feed_forward(x1, w, dims)
