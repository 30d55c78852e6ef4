"""Pins for oracle/stitch.py: hand-worked runs of Algorithm 1 and the special
cases its switching rule (Eq. 2) implies."""
import math

import torch

import workloads as W
from oracle import decoder, router, stitch
from oracle.stitch import SLM, LLM


class Script:
    """A scripted pair of models: invocation i returns (tokens[i], entropies[i])
    and records which model ran, on which span, at which position."""

    def __init__(self, tokens, entropies):
        self.tokens, self.entropies, self.calls = tokens, entropies, []

    def __call__(self, model, span, pos0):
        i = len(self.calls)
        self.calls.append((model, list(span), pos0))
        return self.tokens[i], self.entropies[i]


def test_hand_worked_trace():
    # prompt of 3 tokens, tau = 0.5.  Worked by hand from Algorithm 1:
    #  1 SLM first runs over the whole prompt (3 tokens), H .2 -> keep 100
    #  2 SLM decodes from [100], H .4 -> keep 101
    #  3 SLM decodes from [101], H .9 -> token 999 discarded, switch to LLM
    #  4 LLM's first participation: full prefill of prompt+output (5 tokens), H .8 -> keep 200, LLM continues
    #  5 LLM decodes from [200], H .5 == tau -> keep 201, hand back (<= tau)
    #  6 SLM has seen 5 tokens, sequence has 7: partial prefill of the 2 LLM tokens, H .1 -> keep 102
    #  7 SLM decodes from [102], H .7 -> token 998 discarded, switch to LLM
    #  8 LLM has seen 6 of 8: partial prefill of [201, 102], H .3 -> keep 202, hand back
    #  9 SLM decodes from [202], H .0 -> keep 103
    sc = Script([100, 101, 999, 200, 201, 102, 998, 202, 103],
                [0.2, 0.4, 0.9, 0.8, 0.5, 0.1, 0.7, 0.3, 0.0])
    r = stitch.generate([10, 11, 12], sc, tau=0.5, n_tokens=7)
    assert r.output == [100, 101, 200, 201, 102, 202, 103]
    assert sc.calls == [
        (SLM, [10, 11, 12], 0),
        (SLM, [100], 3),
        (SLM, [101], 4),
        (LLM, [10, 11, 12, 100, 101], 0),
        (LLM, [200], 5),
        (SLM, [200, 201], 5),
        (SLM, [102], 7),
        (LLM, [201, 102], 6),
        (SLM, [202], 8),
    ]
    assert [t.accept for t in r.trace] == [True, True, False, True, True, True, False, True, True]
    assert [t.hi for t in r.trace] == [False, False, True, True, False, False, True, False, False]
    assert r.n_llm_tokens == 3 and r.n_rejected == 2


def test_llm_run_lengths_and_span_bookkeeping():
    # After the SLM accepted j tokens since the hand-back, the LLM's catch-up span is j + 1;
    # after the LLM produced k tokens, the SLM's catch-up span is k.
    ent = [0.9,            # SLM rejects at once
           0.9, 0.9, 0.1,  # LLM keeps 3 tokens, hands back after the third
           0.1, 0.1, 0.1, 0.9,  # SLM: span 3, then two decodes, then reject (j = 3 accepted)
           0.1]            # LLM: span j + 1 = 4
    sc = Script(list(range(50, 59)), ent)
    r = stitch.generate([1, 2], sc, tau=0.5, n_tokens=7)
    spans = [(m, len(s), p) for m, s, p in sc.calls]
    assert spans == [(SLM, 2, 0), (LLM, 2, 0), (LLM, 1, 2), (LLM, 1, 3), (SLM, 3, 2), (SLM, 1, 5), (SLM, 1, 6),
                     (SLM, 1, 7), (LLM, 4, 4)]
    assert r.output == [51, 52, 53, 54, 55, 56, 58]


def test_budget_counts_accepted_tokens_and_invocation_cap_counts_calls():
    sc = Script(list(range(100)), [0.9, 0.1] * 50)     # every SLM call rejected, every LLM call hands back
    r = stitch.generate([7], sc, tau=0.5, n_tokens=5)
    assert len(r.output) == 5 and len(r.trace) == 10
    sc = Script(list(range(100)), [0.9, 0.1] * 50)
    r = stitch.generate([7], sc, tau=0.5, n_tokens=5, max_invocations=7)
    assert len(r.trace) == 7 and len(r.output) == 3


def test_eos_stops_after_append():
    sc = Script([5, 6, 2, 9], [0.0] * 4)
    r = stitch.generate([1], sc, tau=0.5, n_tokens=10, eos=2)
    assert r.output == [5, 6, 2]


def _pair(seed=3):
    wl = W.WORKLOADS["cfg1_tiny_pair"]
    ws, wlg = W.make_weights(wl.slm, seed, 0), W.make_weights(wl.llm, seed, 1)
    prompt = W.make_prompt(wl).tolist()[:12]
    scales = W.logit_scale(wl, 0, 64)
    mk = lambda: [decoder.OracleModel(ws, 64), decoder.OracleModel(wlg, 64)]  # noqa: E731
    return wl, prompt, scales, mk


def _single_model_greedy(model, prompt, scales, n):
    seq = list(prompt)
    lg = model.forward(seq, 0, logit_scale=float(scales[len(seq)]))["logits"]
    out = []
    for _ in range(n):
        t = router.greedy_token(lg)
        out.append(t)
        seq.append(t)
        lg = model.forward([t], len(seq) - 1, logit_scale=float(scales[len(seq)]))["logits"]
    return out


def test_tau_at_least_one_is_small_model_greedy_decoding():
    wl, prompt, scales, mk = _pair()
    models = mk()
    r = stitch.generate(prompt, stitch.decoder_forward(models, lambda p: float(scales[p])), tau=1.0, n_tokens=20)
    assert all(t.model == SLM and t.accept for t in r.trace)
    assert r.output == _single_model_greedy(mk()[SLM], prompt, scales, 20)


def test_negative_tau_is_large_model_greedy_decoding_after_one_small_call():
    wl, prompt, scales, mk = _pair()
    r = stitch.generate(prompt, stitch.decoder_forward(mk(), lambda p: float(scales[p])), tau=-1.0, n_tokens=20)
    assert [t.model for t in r.trace] == [SLM] + [LLM] * 20
    assert not r.trace[0].accept and all(t.accept for t in r.trace[1:])
    assert len(r.trace[1].span) == len(prompt)                  # first participation: full prefill
    assert r.output == _single_model_greedy(mk()[LLM], prompt, scales, 20)


def test_stitched_run_is_independent_of_how_catchup_spans_are_fed():
    # Feeding every catch-up span token by token instead of as one prefill must not change the run.
    wl, prompt, scales, mk = _pair()
    hs = [t.h_norm for t in stitch.generate(prompt, stitch.decoder_forward(mk(), lambda p: float(scales[p])),
                                            tau=2.0, n_tokens=30).trace]
    tau = W.pick_tau(hs, 60.0, 4e-3 / math.log(1024))
    ref = stitch.generate(prompt, stitch.decoder_forward(mk(), lambda p: float(scales[p])), tau=tau, n_tokens=30)
    assert 0 < ref.n_llm_tokens < 30 and any(len(t.span) > 1 and t.pos0 > 0 for t in ref.trace)
    models = mk()

    def one_by_one(model, span, pos0):
        for i, t in enumerate(span):
            lg = models[model].forward([t], pos0 + i, logit_scale=float(scales[pos0 + len(span)]))["logits"]
        return router.greedy_token(lg), router.normalised_entropy(lg)

    alt = stitch.generate(prompt, one_by_one, tau=tau, n_tokens=30)
    assert alt.output == ref.output
    assert [(t.model, t.accept) for t in alt.trace] == [(t.model, t.accept) for t in ref.trace]
    assert max(abs(a.h_norm - b.h_norm) for a, b in zip(alt.trace, ref.trace)) < 1e-9


def test_random_routing_assigns_each_token_by_its_own_draw():
    # u per absolute position; p = 0.5: positions 3, 4 -> small, 5, 6 -> large, 7 -> small.  By hand:
    #  t=3 SLM over the prompt [10,11,12]          -> 100
    #  t=4 SLM decodes [100]                       -> 101
    #  t=5 LLM first participation, 5 tokens       -> 200
    #  t=6 LLM decodes [200]                       -> 201
    #  t=7 SLM catches up with [101?]...: it has seen 4 tokens (0..3), the sequence has 7 -> span [101, 200, 201]
    u = {3: 0.1, 4: 0.4, 5: 0.9, 6: 0.5, 7: 0.49}
    sc = Script([100, 101, 200, 201, 102], [0.9, 0.9, 0.1, 0.1, 0.9])          # entropies are ignored
    r = stitch.generate_random([10, 11, 12], sc, 0.5, lambda t: u[t], 5)
    assert r.output == [100, 101, 200, 201, 102] and r.n_rejected == 0
    assert sc.calls == [(SLM, [10, 11, 12], 0), (SLM, [100], 3), (LLM, [10, 11, 12, 100, 101], 0), (LLM, [200], 5),
                        (SLM, [101, 200, 201], 4)]


def test_random_routing_special_cases_and_share():
    toks = list(range(500, 900))
    ent = [0.5] * 400
    all_slm = Script(toks, ent)
    a = stitch.generate_random([1, 2], all_slm, 1.0, lambda t: 0.999999, 50)
    assert all(m == SLM for m, _, _ in all_slm.calls) and a.output == toks[:50]
    all_llm = Script(toks, ent)
    stitch.generate_random([1, 2], all_llm, 0.0, lambda t: 1e-9, 50)
    assert all(m == LLM for m, _, _ in all_llm.calls)
    # the share of small-model tokens follows p
    us = W.uniform01(3, 77, 0, 402).tolist()
    sc = Script(toks, ent)
    r = stitch.generate_random([1, 2], sc, 0.3, lambda t: us[t], 400)
    share = sum(1 for t in r.trace if t.model == SLM) / 400
    assert abs(share - 0.3) < 0.07
    # every token of prompt + output is seen exactly once by each model that ran at or after it
    seen = {SLM: 0, LLM: 0}
    for m, span, pos0 in sc.calls:
        assert pos0 == seen[m]
        seen[m] += len(span)
