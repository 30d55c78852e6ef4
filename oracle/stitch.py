"""Oracle of the stitched inference loop (test infrastructure; see package docstring).

Algorithm 1 ("Inference procedure"): decoding starts on the small model; the
active model first brings its own KV cache up to date with whatever part of
prompt + output it has not processed (a prefill over that suffix; a plain
decode step when the suffix is one token), which yields a next-token
distribution and a token; the entropy of the distribution is compared with tau
(Eq. 2); a small-model token with entropy above tau is thrown away and the same
position is redone by the large model; a large-model token is always kept and
control returns to the small model as soon as the large model's entropy is at
or below tau.

Position-explicit form used here: ``n_kv[m]`` is the number of tokens of
prompt + output whose K/V rows model m holds.  The paper's cache-size counter
L also counts the token just sampled, so L = n_kv + 1 after an accepted step,
and its "rollback" of the small model's cache on a discard only drops that
sampled token: the K/V rows written during the discarded step belong to
tokens that were already accepted and stay valid.
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

SLM, LLM = 0, 1


@dataclass
class Invocation:
    model: int            # which model ran
    pos0: int             # position of the first token of the span
    span: List[int]       # tokens fed in (the suffix the model had not seen)
    token: int            # token it produced
    h_norm: float         # normalised entropy of its distribution
    hi: bool              # h_norm > tau
    accept: bool          # token appended to the output


@dataclass
class StitchResult:
    output: List[int] = field(default_factory=list)
    trace: List[Invocation] = field(default_factory=list)

    @property
    def n_llm_tokens(self) -> int:
        return sum(1 for r in self.trace if r.accept and r.model == LLM)

    @property
    def n_rejected(self) -> int:
        return sum(1 for r in self.trace if not r.accept)


Forward = Callable[[int, List[int], int], Tuple[int, float]]


def generate(prompt: Sequence[int], forward: Forward, tau: float, n_tokens: int,
             eos: Optional[int] = None, max_invocations: Optional[int] = None) -> StitchResult:
    """Run Algorithm 1 until ``n_tokens`` tokens have been accepted.

    ``forward(model, span, pos0)`` runs model ``model`` over ``span`` placed at
    positions pos0.., updating that model's cache, and returns the token it
    proposes for position pos0+len(span) and the normalised entropy (Eq. 1) of
    the distribution it was drawn from.
    """
    seq = list(prompt)
    n_kv = [0, 0]
    active = SLM
    res = StitchResult()
    while len(res.output) < n_tokens:
        if max_invocations is not None and len(res.trace) >= max_invocations:
            break
        pos0 = n_kv[active]
        span = seq[pos0:]
        token, h = forward(active, span, pos0)
        n_kv[active] = len(seq)
        hi = h > tau
        if active == SLM and hi:
            res.trace.append(Invocation(active, pos0, span, token, h, True, False))
            active = LLM                      # token discarded; the large model redoes this position
            continue
        res.trace.append(Invocation(active, pos0, span, token, h, hi, True))
        if active == LLM and not hi:
            active = SLM                      # token kept; hand back
        seq.append(token)
        res.output.append(token)
        if eos is not None and token == eos:
            break
    return res


def decoder_forward(models, scale_of_pos: Callable[[int], float], log: Optional[list] = None,
                    uniforms_of_pos: Optional[Callable[[int], object]] = None) -> Forward:
    """Bind two ``oracle.decoder.OracleModel`` objects (index SLM, LLM) into the
    ``forward`` callable of :func:`generate`.  ``scale_of_pos(p)`` is the logit
    scale used when predicting the token at absolute position p.  When ``log``
    is a list, the scaled logits of every invocation are appended to it.
    ``uniforms_of_pos(p)``: when given, the token at position p is SAMPLED from
    the distribution with these uniforms (one per vocabulary entry) instead of
    taken greedily."""
    from . import router

    def forward(model: int, span: List[int], pos0: int) -> Tuple[int, float]:
        out = models[model].forward(span, pos0, logit_scale=scale_of_pos(pos0 + len(span)))
        logits = out["logits"]
        if log is not None:
            log.append(logits)
        if uniforms_of_pos is not None:
            token = router.sample_token(logits, uniforms_of_pos(pos0 + len(span)))
        else:
            token = router.greedy_token(logits)
        return token, router.normalised_entropy(logits)

    return forward


def generate_plus(prompt: Sequence[int], forward_state, router_says_llm: Callable[[object], bool], tau: float,
                  n_tokens: int, max_invocations: Optional[int] = None) -> StitchResult:
    """Algorithm 1 with its R-Stitch+ branch: as :func:`generate`, but a small-model step whose
    entropy exceeds tau hands over only if the router, given that step's hidden state, picks the
    large model; otherwise the token is kept and the small model goes on.

    ``forward_state(model, span, pos0)`` returns (token, normalised entropy, state);
    ``router_says_llm(state)`` is consulted only for small-model steps above tau.
    """
    seq = list(prompt)
    n_kv = [0, 0]
    active = SLM
    res = StitchResult()
    while len(res.output) < n_tokens:
        if max_invocations is not None and len(res.trace) >= max_invocations:
            break
        pos0 = n_kv[active]
        span = seq[pos0:]
        token, h, state = forward_state(active, span, pos0)
        n_kv[active] = len(seq)
        hi = h > tau
        if active == SLM and hi and router_says_llm(state):
            res.trace.append(Invocation(active, pos0, span, token, h, True, False))
            active = LLM
            continue
        res.trace.append(Invocation(active, pos0, span, token, h, hi, True))
        if active == LLM and not hi:
            active = SLM
        seq.append(token)
        res.output.append(token)
    return res


def generate_random(prompt: Sequence[int], forward: Forward, p_slm: float, u_of_pos: Callable[[int], float],
                    n_tokens: int) -> StitchResult:
    """Random-routing baseline (Section "Experiments", paragraph "Latency-accuracy trade-off"): every
    token is assigned to the small model with a fixed probability p_slm and to the large model
    otherwise, whatever the distributions look like.  The token at absolute position t goes to the
    small model iff u_of_pos(t) < p_slm (u uniform in (0, 1), drawn per position); the assigned model
    first catches up with the tokens it has not seen (same cache bookkeeping as Algorithm 1) and its
    token is always kept: nothing is discarded, since the assignment does not look at the step.
    """
    seq = list(prompt)
    n_kv = [0, 0]
    res = StitchResult()
    while len(res.output) < n_tokens:
        model = SLM if u_of_pos(len(seq)) < p_slm else LLM
        pos0 = n_kv[model]
        span = seq[pos0:]
        token, h = forward(model, span, pos0)
        n_kv[model] = len(seq)
        res.trace.append(Invocation(model, pos0, span, token, h, False, True))
        seq.append(token)
        res.output.append(token)
    return res
