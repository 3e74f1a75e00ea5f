"""Decoder-only transformer forward: full recomputation and a KV-cached path.

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper fixes only "Llama backbones" (Sec. V-A, "LLM Backbones") and the
sequence shape (Sec. V-A, "Hyperparameters").  The architecture written out
here is the pre-norm Llama decoder: RMSNorm, rotary position embedding with
half-split pairing, causal softmax attention with grouped KV heads, SwiGLU MLP,
no biases, untied LM head.

Two routines are written separately on purpose:
  * `forward_full`  - the definition: run the network over a whole sequence.
  * `CachedDecoder` - keys/values kept per layer, new tokens attend to the cache.
Tests require them to agree.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence

import torch


def _f(t: torch.Tensor, dtype: torch.dtype) -> torch.Tensor:
    return t.detach().to(device="cpu").to(dtype)


def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    """y = x / sqrt(mean(x^2) + eps) * gain, per row (last dimension)."""
    ms = (x * x).sum(dim=-1, keepdim=True) / x.shape[-1]
    return x / torch.sqrt(ms + eps) * gain


def rope(x: torch.Tensor, positions: torch.Tensor, theta: float) -> torch.Tensor:
    """Rotary embedding, half-split pairing.

    x: [n, H, h]; positions: [n] integers.  For i < h/2 the pair (x_i, x_{i+h/2})
    is rotated by the angle pos * theta^(-2i/h).  Angles are formed in float64.
    """
    n, H, h = x.shape
    half = h // 2
    i = torch.arange(half, dtype=torch.float64)
    inv_freq = theta ** (-2.0 * i / h)                                 # [half]
    ang = positions.to(torch.float64)[:, None] * inv_freq[None, :]     # [n, half]
    c = torch.cos(ang).to(x.dtype)[:, None, :]
    s = torch.sin(ang).to(x.dtype)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return torch.cat([lo * c - hi * s, hi * c + lo * s], dim=-1)


def softmax_rows(z: torch.Tensor) -> torch.Tensor:
    """Max-subtracted softmax over the last dimension (-inf entries give 0)."""
    m = z.max(dim=-1, keepdim=True).values
    e = torch.exp(z - m)
    return e / e.sum(dim=-1, keepdim=True)


def silu(z: torch.Tensor) -> torch.Tensor:
    return z / (1.0 + torch.exp(-z))


def _split_qkv(qkv: torch.Tensor, shape) -> tuple:
    n = qkv.shape[0]
    Hq, Hkv, h = shape.n_heads, shape.n_kv_heads, shape.head_dim
    q = qkv[:, : Hq * h].reshape(n, Hq, h)
    k = qkv[:, Hq * h: (Hq + Hkv) * h].reshape(n, Hkv, h)
    v = qkv[:, (Hq + Hkv) * h:].reshape(n, Hkv, h)
    return q, k, v


def _mlp(x: torch.Tensor, lw: dict, shape, dtype) -> torch.Tensor:
    y = rmsnorm(x, _f(lw["ffn_norm"], dtype), shape.rms_eps)
    gu = y @ _f(lw["w_gate_up"], dtype).T
    F = shape.d_ffn
    act = silu(gu[:, :F]) * gu[:, F:]
    return x + act @ _f(lw["w_down"], dtype).T


def forward_full(w: dict, shape, tokens: Sequence[int], dtype=torch.float64,
                 logits_at: Optional[Sequence[int]] = None,
                 position_offset: int = 0) -> torch.Tensor:
    """Logits of one sequence by full recomputation.

    tokens: the n token ids s_0..s_{n-1}; s_i sits at position i + position_offset.
    Returns logits [len(logits_at), V] (default: every position).  Row r is the
    next-token distribution after reading tokens[0 .. logits_at[r]].
    """
    n = len(tokens)
    ids = torch.as_tensor(list(tokens), dtype=torch.long)
    pos = torch.arange(n, dtype=torch.long) + position_offset
    Hq, Hkv, h = shape.n_heads, shape.n_kv_heads, shape.head_dim
    group = Hq // Hkv
    x = _f(w["tok_emb"], dtype)[ids]                                   # [n, d]
    causal = torch.tril(torch.ones(n, n, dtype=torch.bool))            # key m visible to query i iff m <= i
    for lw in w["layers"]:
        y = rmsnorm(x, _f(lw["attn_norm"], dtype), shape.rms_eps)
        q, k, v = _split_qkv(y @ _f(lw["wqkv"], dtype).T, shape)
        q = rope(q, pos, shape.rope_theta)
        k = rope(k, pos, shape.rope_theta)
        heads = []
        for j in range(Hq):
            kv = j // group                                            # contiguous groups of query heads
            scores = (q[:, j, :] @ k[:, kv, :].T) / math.sqrt(h)        # [n, n]
            scores = scores.masked_fill(~causal, float("-inf"))
            heads.append(softmax_rows(scores) @ v[:, kv, :])            # [n, h]
        a = torch.cat(heads, dim=-1)                                    # [n, Hq*h]
        x = x + a @ _f(lw["wo"], dtype).T
        x = _mlp(x, lw, shape, dtype)
    if logits_at is None:
        logits_at = range(n)
    xs = x[torch.as_tensor(list(logits_at), dtype=torch.long)]
    return rmsnorm(xs, _f(w["final_norm"], dtype), shape.rms_eps) @ _f(w["lm_head"], dtype).T


class CachedDecoder:
    """Incremental forward of ONE sequence with per-layer key/value caches.

    `extend(tokens)` feeds any number of new tokens (a whole query, or a single
    decode token) and returns the logits after the last of them.
    """

    def __init__(self, w: dict, shape, dtype=torch.float64):
        self.w, self.shape, self.dtype = w, shape, dtype
        self.keys: List[Optional[torch.Tensor]] = [None] * shape.n_layers     # each [L, Hkv, h], post-RoPE
        self.values: List[Optional[torch.Tensor]] = [None] * shape.n_layers
        self.length = 0

    def extend(self, tokens: Sequence[int]) -> torch.Tensor:
        s, dt = self.shape, self.dtype
        m = len(tokens)
        ids = torch.as_tensor(list(tokens), dtype=torch.long)
        pos = torch.arange(self.length, self.length + m, dtype=torch.long)
        Hq, Hkv, h = s.n_heads, s.n_kv_heads, s.head_dim
        group = Hq // Hkv
        x = _f(self.w["tok_emb"], dt)[ids]
        for li, lw in enumerate(self.w["layers"]):
            y = rmsnorm(x, _f(lw["attn_norm"], dt), s.rms_eps)
            q, k, v = _split_qkv(y @ _f(lw["wqkv"], dt).T, s)
            q = rope(q, pos, s.rope_theta)
            k = rope(k, pos, s.rope_theta)
            if self.keys[li] is None:
                self.keys[li], self.values[li] = k, v
            else:
                self.keys[li] = torch.cat([self.keys[li], k], dim=0)
                self.values[li] = torch.cat([self.values[li], v], dim=0)
            K, V = self.keys[li], self.values[li]
            a = torch.empty(m, Hq * h, dtype=dt)
            for r in range(m):
                visible = self.length + r + 1                           # cached tokens + new ones up to itself
                for j in range(Hq):
                    kv = j // group
                    sc = (K[:visible, kv, :] @ q[r, j, :]) / math.sqrt(h)
                    a[r, j * h:(j + 1) * h] = softmax_rows(sc[None, :])[0] @ V[:visible, kv, :]
            x = x + a @ _f(lw["wo"], dt).T
            x = _mlp(x, lw, s, dt)
        self.length += m
        last = rmsnorm(x[-1:], _f(self.w["final_norm"], dt), s.rms_eps)
        return (last @ _f(self.w["lm_head"], dt).T)[0]
