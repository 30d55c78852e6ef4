"""Pins for oracle/router_plus.py (the R-Stitch+ router) and the R-Stitch+ branch of Algorithm 1 in oracle/stitch.py."""
import math

import pytest
import torch
import torch.nn as nn
import torch.nn.functional as F

import workloads as W
from oracle import router, router_plus as rp, stitch
from oracle.stitch import SLM, LLM
from workloads.recipes import misc_normal

F64 = torch.float64


def test_gelu_closed_forms_and_library():
    x = torch.tensor([0.0, 1.0, -1.0, 8.0, -8.0], dtype=F64)
    y = rp.gelu(x)
    phi1 = 0.5 * (1.0 + math.erf(1.0 / math.sqrt(2.0)))          # normal distribution function at 1
    assert y[0] == 0.0 and float(y[1]) == pytest.approx(phi1, rel=1e-14) and float(y[2]) == pytest.approx(-(1 - phi1), rel=1e-13)
    assert float(y[3]) == pytest.approx(8.0, abs=1e-13) and abs(float(y[4])) < 1e-13
    z = misc_normal(5, 1, 1000) * 3
    assert torch.allclose(rp.gelu(z), F.gelu(z), rtol=1e-12, atol=1e-14)        # the erf form, not the tanh approximation
    assert not torch.allclose(rp.gelu(z), F.gelu(z, approximate="tanh"), rtol=1e-6, atol=1e-8)


def test_layernorm_closed_forms_and_library():
    g, b = misc_normal(5, 2, 64), misc_normal(5, 3, 64)
    const = torch.full((64,), 3.5, dtype=F64)
    assert torch.allclose(rp.layernorm(const, g, b), b, atol=1e-12)             # a constant vector has zero deviation
    x = misc_normal(5, 4, 7 * 64).view(7, 64)
    assert torch.allclose(rp.layernorm(x, g, b), F.layer_norm(x, (64,), g, b, 1e-5), rtol=1e-12, atol=1e-13)
    y = rp.layernorm(x, torch.ones(64, dtype=F64), torch.zeros(64, dtype=F64), eps=0.0)
    assert torch.allclose(y.mean(-1), torch.zeros(7, dtype=F64), atol=1e-13) and torch.allclose((y * y).mean(-1), torch.ones(7, dtype=F64), rtol=1e-12)


def test_parameter_count_of_the_reading():
    w = W.make_router_weights(1536, 8, seed=1)
    assert w.n_params() == 6 * (8 * 1536 + 8 + 1536 * 8 + 1536) + 2 * 1536 + 2 * 1536 + 2 == 162866    # the paper: 0.17 M


def test_zero_up_projections_leave_only_norm_and_head():
    w = W.make_router_weights(96, 4, seed=2)
    for i in range(6):
        w.w2[i] = torch.zeros_like(w.w2[i])
        w.b2[i] = torch.zeros_like(w.b2[i])
    x = misc_normal(5, 5, 96)
    want = F.linear(F.layer_norm(x, (96,), w.ln_gain.double(), w.ln_bias.double(), 1e-5), w.w_head.double(), w.b_head.double())
    assert torch.allclose(rp.router_logits(w, x), want, rtol=1e-12, atol=1e-13)


def test_whole_router_against_library_modules():
    d, r = 128, 8
    w = W.make_router_weights(d, r, seed=3)
    blocks = []
    for i in range(6):
        a, b = nn.Linear(d, r, dtype=F64), nn.Linear(r, d, dtype=F64)
        with torch.no_grad():
            a.weight.copy_(w.w1[i].double()); a.bias.copy_(w.b1[i].double())
            b.weight.copy_(w.w2[i].double()); b.bias.copy_(w.b2[i].double())
        blocks.append(nn.Sequential(a, nn.GELU(), b))
    ln, head = nn.LayerNorm(d, eps=1e-5, dtype=F64), nn.Linear(d, 2, dtype=F64)
    with torch.no_grad():
        ln.weight.copy_(w.ln_gain.double()); ln.bias.copy_(w.ln_bias.double())
        head.weight.copy_(w.w_head.double()); head.bias.copy_(w.b_head.double())
    x = misc_normal(5, 6, 3 * d).view(3, d)
    y = x.clone()
    with torch.no_grad():
        for blk in blocks:
            y = y + blk(y)
        want = head(ln(y))
    got = rp.router_logits(w, x)
    assert torch.allclose(got, want, rtol=1e-11, atol=1e-12)
    assert [rp.wants_llm(w, x[i]) for i in range(3)] == [bool(want[i, 1] > want[i, 0]) for i in range(3)]


def test_switch_plus_truth_table():
    # (entropy, tau, active, router says large) -> (hi, accept, next)
    rows = [
        (0.9, 0.5, SLM, True, (True, False, LLM)),     # uncertain and the router agrees: discard, hand over
        (0.9, 0.5, SLM, False, (True, True, SLM)),     # uncertain but the router keeps the small model: token kept
        (0.2, 0.5, SLM, True, (False, True, SLM)),     # low entropy always stays (the router is not even asked)
        (0.5, 0.5, SLM, True, (False, True, SLM)),     # equality is "not above"
        (0.9, 0.5, LLM, False, (True, True, LLM)),     # the large model ignores the router
        (0.2, 0.5, LLM, True, (False, True, SLM)),
    ]
    for h, tau, active, says, want in rows:
        assert rp.switch_plus(h, tau, active, says) == want
    # with a router that always says "large" the rule is Eq. 2 itself
    for h in (0.1, 0.5, 0.7):
        for active in (SLM, LLM):
            assert rp.switch_plus(h, 0.5, active, True) == router.switch(h, 0.5, active)


class Script:
    def __init__(self, tokens, entropies):
        self.tokens, self.entropies, self.calls = tokens, entropies, []

    def __call__(self, model, span, pos0):
        i = len(self.calls)
        self.calls.append((model, list(span), pos0))
        return self.tokens[i], self.entropies[i], i            # the "state" handed to the router is the call index


def test_generate_plus_hand_worked_trace():
    # tau .5; router says "large" only for the states listed.  By hand from Algorithm 1 (R-Stitch+ branch):
    #  0 SLM over the prompt, H .9, router(0) = stay   -> keep 100 although uncertain
    #  1 SLM [100], H .8, router(1) = large            -> 999 discarded, hand over
    #  2 LLM first participation over 4 tokens, H .7   -> keep 200, stays (above tau; the router is not asked)
    #  3 LLM [200], H .2                               -> keep 201, hand back
    #  4 SLM catches up with [200, 201], H .3          -> keep 101
    #  5 SLM [101], H .6, router(5) = stay             -> keep 102
    sc = Script([100, 999, 200, 201, 101, 102], [0.9, 0.8, 0.7, 0.2, 0.3, 0.6])
    asked = []

    def says_llm(state):
        asked.append(state)
        return state in (1,)

    r = stitch.generate_plus([10, 11, 12], sc, says_llm, tau=0.5, n_tokens=5)
    assert r.output == [100, 200, 201, 101, 102]
    assert sc.calls == [(SLM, [10, 11, 12], 0), (SLM, [100], 3), (LLM, [10, 11, 12, 100], 0), (LLM, [200], 4),
                        (SLM, [200, 201], 4), (SLM, [101], 6)]
    assert asked == [0, 1, 5]                                   # only small-model steps above tau
    assert [t.accept for t in r.trace] == [True, False, True, True, True, True]


def test_generate_plus_special_cases():
    tokens, ent = list(range(100, 120)), [0.9, 0.1, 0.8, 0.7, 0.2, 0.95, 0.3, 0.6, 0.1, 0.9, 0.4, 0.5, 0.6, 0.2, 0.8, 0.1, 0.3, 0.7, 0.2, 0.6]
    # a router that always picks the large model: Algorithm 1 without the branch
    a = stitch.generate_plus([1, 2], Script(tokens, ent), lambda s: True, 0.5, 8)
    fwd = Script(tokens, ent)
    b = stitch.generate([1, 2], lambda m, sp, p: fwd(m, sp, p)[:2], 0.5, 8)
    assert a.output == b.output and [(t.model, t.pos0, t.span, t.accept) for t in a.trace] == [(t.model, t.pos0, t.span, t.accept) for t in b.trace]
    # a router that never does: the large model is never invoked and every token is kept
    sc = Script(tokens, ent)
    c = stitch.generate_plus([1, 2], sc, lambda s: False, 0.5, 8)
    assert all(m == SLM for m, _, _ in sc.calls) and c.output == tokens[:8] and c.n_rejected == 0
