"""Oracle of the entropy router (test infrastructure; see package docstring).

Eq. 1: the uncertainty of a step is the Shannon entropy of the next-token
distribution divided by log V, a number in [0, 1].
Eq. 2: the small model hands over when its normalised entropy is strictly
above tau; the large model hands back when its own is at or below tau.

All arithmetic is fp64.  The entropy is the definition written out: softmax,
then minus the sum of p log p with 0 log 0 taken as 0.
"""

from __future__ import annotations

import math

import torch

SLM, LLM = 0, 1

FLAG_HI = 1          # normalised entropy strictly above tau
FLAG_ACCEPT = 2      # the token of this step is kept
FLAG_NEXT_LLM = 4    # the model that runs the next step is the large one
FLAG_NONFINITE = 8   # some logit was NaN or infinite; the step is treated as uncertain


def softmax(logits: torch.Tensor) -> torch.Tensor:
    x = logits.to(torch.float64)
    e = torch.exp(x - x.max())
    return e / e.sum()


def entropy_nats(logits: torch.Tensor) -> float:
    """-sum_i p_i ln p_i of p = softmax(logits), natural log."""
    p = softmax(logits)
    plogp = torch.where(p > 0, p * torch.log(torch.where(p > 0, p, torch.ones_like(p))),
                        torch.zeros_like(p))
    return float(-plogp.sum())


def normalised_entropy(logits: torch.Tensor) -> float:
    """Eq. 1: entropy divided by log V."""
    return entropy_nats(logits) / math.log(logits.numel())


def greedy_token(logits: torch.Tensor) -> int:
    """Index of the largest logit; the lowest index among equals."""
    x = logits.to(torch.float64)
    return int(torch.nonzero(x == x.max())[0, 0])


def switch(h_norm: float, tau: float, active: int):
    """Eq. 2 together with the accept/discard rule of Algorithm 1.

    Returns (hi, accept, next_active): a small-model token is discarded exactly
    when hi; a large-model token is always kept; the next step runs on the large
    model exactly when hi.
    """
    hi = h_norm > tau
    accept = not (active == SLM and hi)
    return hi, accept, (LLM if hi else SLM)


def route(logits: torch.Tensor, tau: float, active: int) -> dict:
    """Everything the router reports for one step from its (scaled) logits."""
    x = logits.to(torch.float64)
    v = x.numel()
    if not bool(torch.isfinite(x).all()):
        flags = FLAG_NONFINITE | FLAG_HI | FLAG_NEXT_LLM | (FLAG_ACCEPT if active == LLM else 0)
        return dict(token=-1, flags=flags, h_nats=float("nan"), h_norm=float("nan"),
                    max_logit=float("nan"), log_z=float("nan"))
    h = entropy_nats(x)
    hn = h / math.log(v)
    hi, accept, nxt = switch(hn, tau, active)
    flags = (FLAG_HI if hi else 0) | (FLAG_ACCEPT if accept else 0) | (FLAG_NEXT_LLM if nxt == LLM else 0)
    m = float(x.max())
    return dict(token=greedy_token(x), flags=flags, h_nats=h, h_norm=hn, max_logit=m,
                log_z=m + float(torch.log(torch.exp(x - m).sum())))


def sample_token(logits: torch.Tensor, uniforms: torch.Tensor) -> int:
    """A token drawn from softmax(logits) (Section "Preliminary": the next token is sampled from the
    distribution the active model outputs), by the Gumbel-max construction: with u_i independent
    uniforms in (0, 1), argmax_i (logit_i - ln(-ln u_i)) is distributed as softmax(logits).  The
    uniforms are inputs (one per vocabulary entry, drawn by the caller per position); the lowest
    index wins among equal maxima."""
    x = logits.to(torch.float64) - torch.log(-torch.log(uniforms.to(torch.float64)))
    return int(torch.nonzero(x == x.max())[0, 0])
