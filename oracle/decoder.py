"""Oracle of the decoder forward pass (test infrastructure; see package docstring).

The paper only says that every generated token costs a full forward pass of
the active model (Section "Preliminary": p_t = f(y_{1:t-1})) and that each
model keeps its own KV cache, prefilling only the tokens it has not seen when
it is switched to ("KV Cache management").  The layer itself is the public
Qwen2-style decoder block: pre-RMSNorm, grouped-query attention with rotary
position embedding (rotate-half pairing), SwiGLU MLP, residual connections,
final RMSNorm and a linear LM head (tied to the embedding or not).  No biases.

Arithmetic: fp64 everywhere.  The weights are bf16 values (inputs).  With
``contract=True`` the rotated key and the value are rounded to bf16 (via fp32,
round to nearest even) when they are stored in the KV cache, which is the one
place where the pipeline keeps an activation in bf16; every other activation
(residual stream, normalised inputs, queries, attention probabilities and
outputs, MLP activations, logits) stays unrounded.  With ``contract=False``
nothing is rounded, which makes the function the textbook decoder and lets a
test compare it with an independent library implementation.

Why no other rounding point: rounding an activation to bf16 turns a relative
difference delta between two otherwise equivalent computations (fp32 versus
fp64 accumulation, a different summation order) into sqrt(delta * 2^-8), and a
chain of such roundings drives it up to the bf16 step itself within a couple of
layers; logits of two correct implementations would then differ by ~1e-2 and
no entropy or argmax tolerance finer than that could be met by anyone.
"""

from __future__ import annotations

import math
from typing import List, Optional, Sequence

import torch

F64 = torch.float64


def round_bf16(x: torch.Tensor) -> torch.Tensor:
    """Round fp64 values to the nearest bf16 (through fp32) and return fp64."""
    return x.to(torch.float32).to(torch.bfloat16).to(F64)


def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    """x / sqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = (x * x).mean(dim=-1, keepdim=True)
    return x / torch.sqrt(ms + eps) * gain


def rope_angles(pos: int, head_dim: int, theta: float) -> torch.Tensor:
    """pos * theta^(-2i/head_dim) for i = 0 .. head_dim/2 - 1."""
    i = torch.arange(head_dim // 2, dtype=F64)
    return pos * torch.pow(torch.tensor(theta, dtype=F64), -2.0 * i / head_dim)


def rope(x: torch.Tensor, pos: int, theta: float) -> torch.Tensor:
    """Rotate the pairs (i, i + head_dim/2) of every head vector by the angle
    pos * theta^(-2i/head_dim).  x: [..., head_dim]."""
    hd = x.shape[-1]
    half = hd // 2
    ang = rope_angles(pos, hd, theta)
    c, s = torch.cos(ang), torch.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return torch.cat([a * c - b * s, b * c + a * s], dim=-1)


def attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor) -> torch.Tensor:
    """softmax(q k^T / sqrt(head_dim)) v for one query vector per head.

    q: [Hq, hd]; k, v: [Hkv, n, hd]; query head j reads kv head j // (Hq/Hkv).
    Returns [Hq, hd].
    """
    hq, hd = q.shape
    hkv, n, _ = k.shape
    g = hq // hkv
    out = torch.empty(hq, hd, dtype=F64)
    for j in range(hq):
        h = j // g
        s = (k[h] @ q[j]) / math.sqrt(hd)          # [n]
        p = torch.exp(s - s.max())
        p = p / p.sum()
        out[j] = p @ v[h]
    return out


def silu(z: torch.Tensor) -> torch.Tensor:
    return z / (1.0 + torch.exp(-z))


class OracleModel:
    """One decoder with its own KV cache (one cache per sequence slot)."""

    def __init__(self, weights, max_ctx: int, n_slots: int = 1, contract: bool = True,
                 keep_fp64_weights: bool = True):
        self.w = weights
        self.s = weights.shape
        self.max_ctx = max_ctx
        self.contract = contract
        self.keep = keep_fp64_weights
        self._w64 = {}
        s = self.s
        self.k_cache = torch.zeros(s.n_layers, n_slots, s.n_kv_heads, max_ctx, s.head_dim, dtype=F64)
        self.v_cache = torch.zeros_like(self.k_cache)

    # -- helpers ------------------------------------------------------------
    def _f64(self, key, t: torch.Tensor) -> torch.Tensor:
        if not self.keep:
            return t.to(F64)
        if key not in self._w64:
            self._w64[key] = t.to(F64)
        return self._w64[key]

    def _r(self, x: torch.Tensor) -> torch.Tensor:
        return round_bf16(x) if self.contract else x

    # -- one invocation -----------------------------------------------------
    def forward(self, tokens: Sequence[int], pos0: int, slot: int = 0,
                logit_scale: float = 1.0, want_hidden: bool = False) -> dict:
        """Run the model over ``tokens`` placed at positions pos0, pos0+1, ...

        Writes their K and V rows into the cache of ``slot``; row i attends to
        cache positions 0 .. pos0+i.  Returns the logits of the LAST row times
        ``logit_scale`` (fp64 [V]).
        """
        s = self.s
        n = len(tokens)
        if n < 1 or pos0 < 0 or pos0 + n > self.max_ctx:
            raise ValueError("span does not fit the cache")
        hq, hkv, hd = s.n_q_heads, s.n_kv_heads, s.head_dim
        h = self._f64("embed", self.w.embed)[list(tokens)].clone()          # [n, d]
        for l, lw in enumerate(self.w.layers):
            x = rmsnorm(h, self._f64((l, "an"), lw.attn_norm), s.rms_eps)
            qkv = x @ self._f64((l, "qkv"), lw.w_qkv).T                         # [n, (Hq+2Hkv) hd]
            q = qkv[:, :hq * hd].reshape(n, hq, hd)
            k = qkv[:, hq * hd:(hq + hkv) * hd].reshape(n, hkv, hd)
            v = qkv[:, (hq + hkv) * hd:].reshape(n, hkv, hd)
            for i in range(n):
                self.k_cache[l, slot, :, pos0 + i] = self._r(rope(k[i], pos0 + i, s.rope_theta))
                self.v_cache[l, slot, :, pos0 + i] = self._r(v[i])
            o = torch.empty(n, hq * hd, dtype=F64)
            for i in range(n):
                qi = rope(q[i], pos0 + i, s.rope_theta)
                ctx = pos0 + i + 1
                o[i] = attention(qi, self.k_cache[l, slot, :, :ctx], self.v_cache[l, slot, :, :ctx]).reshape(-1)
            h = h + o @ self._f64((l, "o"), lw.w_o).T
            x = rmsnorm(h, self._f64((l, "mn"), lw.mlp_norm), s.rms_eps)
            gu = x @ self._f64((l, "gu"), lw.w_gate_up).T                       # [n, 2 ffn]
            a = silu(gu[:, :s.d_ffn]) * gu[:, s.d_ffn:]
            h = h + a @ self._f64((l, "dn"), lw.w_down).T
        x_last = rmsnorm(h[-1], self._f64("fn", self.w.final_norm), s.rms_eps)
        lm = self._f64("embed", self.w.embed) if s.tied_lm_head else self._f64("lm", self.w.lm_head)
        logits = (lm @ x_last) * float(logit_scale)
        out = dict(logits=logits)
        if want_hidden:
            out["hidden"] = h
            out["x_last"] = x_last
        return out
