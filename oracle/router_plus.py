"""Oracle of the learned router of R-Stitch+ (test infrastructure; see package docstring).

Section "RL-based Routing with Latency-aware Reward": at a step whose entropy exceeds tau the hidden
state of the current model goes through a light router that decides whether to stay on the small
model or switch to the large one; low-entropy tokens always go to the small model.  Algorithm 1 (the
R-Stitch+ branch) takes the arg max of the router's two outputs and uses it only while the small
model is active; a large model above tau keeps going whatever the router says.
Section "Architecture and Overhead of Router": six feed-forward blocks with GELU and residual
connections on a vector of the small model's hidden size, then a normalisation, then a linear layer
with two outputs; 0.17 M parameters in all.

The paper gives no widths.  Reading used here: block i is x <- x + W2_i gelu(W1_i x + b1_i) + b2_i
with a bottleneck of r channels (W1_i: [r, d], W2_i: [d, r]); GELU is the exact (erf) form; the
normalisation is a LayerNorm with gain and bias over the d channels (eps 1e-5); the head is
[2, d] with bias, output 0 = stay on the small model, output 1 = switch to the large model; a tie
stays.  With d = 1536 and r = 8 that is 162 866 parameters (the paper's 0.17 M; its "3584" for the
input width is the hidden size of its 7B model and cannot be met with 0.17 M parameters and r >= 4).
All arithmetic fp64; weights are bf16 values (inputs).
"""

from __future__ import annotations

import math
import torch

F64 = torch.float64
N_BLOCKS = 6
LN_EPS = 1e-5


# Weights: any object with the fields w1, b1, w2, b2 (lists of six tensors: [r, d], [r], [d, r], [d]),
# ln_gain, ln_bias ([d]), w_head ([2, d]) and b_head ([2]); workloads.make_router_weights draws one.


def gelu(x: torch.Tensor) -> torch.Tensor:
    """x * Phi(x) with the normal distribution function written through erf."""
    return 0.5 * x * (1.0 + torch.erf(x / math.sqrt(2.0)))


def layernorm(x: torch.Tensor, gain: torch.Tensor, bias: torch.Tensor, eps: float = LN_EPS) -> torch.Tensor:
    mu = x.mean(dim=-1, keepdim=True)
    var = ((x - mu) ** 2).mean(dim=-1, keepdim=True)
    return (x - mu) / torch.sqrt(var + eps) * gain + bias


def router_logits(w, hidden: torch.Tensor) -> torch.Tensor:
    """hidden: [d] (or [n, d]) -> the two outputs (stay, switch), fp64."""
    x = hidden.to(F64)
    for i in range(N_BLOCKS):
        t = gelu(x @ w.w1[i].to(F64).T + w.b1[i].to(F64))
        x = x + t @ w.w2[i].to(F64).T + w.b2[i].to(F64)
    x = layernorm(x, w.ln_gain.to(F64), w.ln_bias.to(F64))
    return x @ w.w_head.to(F64).T + w.b_head.to(F64)


def wants_llm(w, hidden: torch.Tensor) -> bool:
    """Algorithm 1, R-Stitch+ branch: switch iff the arg max of the two outputs is the large model."""
    out = router_logits(w, hidden)
    return bool(out[1] > out[0])


def switch_plus(h_norm: float, tau: float, active: int, router_says_llm: bool):
    """Eq. 2 with the router in the loop (Algorithm 1): returns (hi, accept, next_active).

    hi = entropy above tau.  On the small model the hand-over happens iff hi and the router says
    so; otherwise its token is kept and it goes on.  The large model ignores the router: it keeps
    going while hi and hands back when not hi; its token is always kept."""
    hi = h_norm > tau
    if active == 0:
        go = hi and router_says_llm
        return hi, not go, (1 if go else 0)
    return hi, True, (1 if hi else 0)
