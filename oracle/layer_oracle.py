"""CPU oracle for the attention half of a LLaMA-style layer (the models of Table 2, Section 4.1.1).

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this file; the product path never does, and this
file imports nothing from the product package.

A layer of these models computes, for a sequence of S tokens,
    a  = rmsnorm(x) * w_attn                        (the input of the q, k, v projections)
    q, k, v = a Wq^T, a Wk^T, a Wv^T                split into heads of width d
    q, k <- rotary embedding by position
    o_in = causal softmax(q k^T / sqrt(d)) v         per head; key / value heads shared by groups of query heads
    x1 = x + o_in Wo^T                              (o_in is the input of the o projection)
    m  = rmsnorm(x1) * w_mlp                         (the input of gate and up)
    y  = x1 + (silu(m Wg^T) * (m Wu^T)) Wd^T
so that the four activation tensors the pruning statistics are taken from come out of one forward pass.
The paper does not restate these formulas; they are the published architecture it prunes.  Readings: rmsnorm
divides by sqrt(mean(x^2) + eps); the rotary embedding pairs dimension i with i + d/2 and turns the pair by the
angle position * base^(-2i/d), base 10000; softmax in float64.  Plain NumPy, no blocking.

Parity status:
  rmsnorm            pinned (hand example, scale invariance)
  rotary             pinned (position 0 is the identity, norms preserved, relative-position property of the scores)
  causal_attention   pinned (brute-force loops, first token attends only to itself, uniform values give the mean,
                     grouped key / value heads equal repeated heads)
  layer_forward      pinned (composition of the pinned pieces and of the feed-forward oracle; identity cases:
                     zero o and down weights leave the residual stream unchanged)
"""
from __future__ import annotations

import numpy as np


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


def rmsnorm(x, weight, eps: float = 1e-5) -> np.ndarray:
    x = _f64(x)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * _f64(weight)


def rotary(x, positions, base: float = 10000.0) -> np.ndarray:
    """x [tokens, heads, d]; dimension i < d/2 is paired with i + d/2 and the pair (a, b) becomes
    (a cos - b sin, b cos + a sin) with angle positions[t] * base^(-2i/d)."""
    x = _f64(x)
    d = x.shape[-1]
    half = d // 2
    inv = base ** (-2.0 * np.arange(half) / d)
    ang = _f64(positions)[:, None, None] * inv[None, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * np.cos(ang) - b * np.sin(ang), b * np.cos(ang) + a * np.sin(ang)], axis=-1)


def causal_attention(q, k, v) -> np.ndarray:
    """q [S, H, d], k, v [S, Hkv, d] for one sequence; query head h uses key / value head h // (H // Hkv).
    out[s, h] = sum_{t <= s} softmax_t(q[s, h] . k[t, g] / sqrt(d)) v[t, g]."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    s_len, heads, d = q.shape
    group = heads // k.shape[1]
    out = np.zeros_like(q)
    mask = np.tril(np.ones((s_len, s_len), dtype=bool))
    for h in range(heads):
        g = h // group
        scores = q[:, h] @ k[:, g].T / np.sqrt(d)
        scores = np.where(mask, scores, -np.inf)
        scores -= scores.max(axis=1, keepdims=True)
        p = np.exp(scores)
        p /= p.sum(axis=1, keepdims=True)
        out[:, h] = p @ v[:, g]
    return out


def layer_forward(x, w, n_seqs: int, seq_len: int, heads: int, kv_heads: int, head_dim: int, eps: float = 1e-5,
                  base: float = 10000.0):
    """One layer on x [n_seqs * seq_len, hidden]; w maps names (attn_norm, q, k, v, o, mlp_norm, gate, up, down) to
    weights.  Returns the four activation tensors the projections' statistics are taken from and the layer output."""
    x = _f64(x)
    tokens = n_seqs * seq_len
    pos = np.tile(np.arange(seq_len), n_seqs)
    attn_in = rmsnorm(x, w["attn_norm"], eps)
    q = rotary((attn_in @ _f64(w["q"]).T).reshape(tokens, heads, head_dim), pos, base)
    k = rotary((attn_in @ _f64(w["k"]).T).reshape(tokens, kv_heads, head_dim), pos, base)
    v = (attn_in @ _f64(w["v"]).T).reshape(tokens, kv_heads, head_dim)
    o_in = np.concatenate([causal_attention(q[b * seq_len:(b + 1) * seq_len], k[b * seq_len:(b + 1) * seq_len],
                                            v[b * seq_len:(b + 1) * seq_len]) for b in range(n_seqs)])
    o_in = o_in.reshape(tokens, heads * head_dim)
    x1 = x + o_in @ _f64(w["o"]).T
    mlp_in = rmsnorm(x1, w["mlp_norm"], eps)
    a = mlp_in @ _f64(w["gate"]).T
    down_in = a / (1.0 + np.exp(-a)) * (mlp_in @ _f64(w["up"]).T)
    y = x1 + down_in @ _f64(w["down"]).T
    return {"attn_in": attn_in, "o_in": o_in, "mlp_in": mlp_in, "down_in": down_in, "out": y}
