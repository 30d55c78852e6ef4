"""Pins for oracle/router.py: closed forms, brute force, a library routine.

Each test is chosen so that a plausible slip in the oracle (a dropped term, the
wrong log base or normaliser, a sign, > versus >=) fails it.
"""
import math

import pytest
import torch

from oracle import router
from workloads.recipes import misc_normal

VOCABS = [2, 3, 1024, 152064]


@pytest.mark.parametrize("v", VOCABS)
def test_uniform_distribution_has_entropy_log_v(v):
    # Eq. 1: the normaliser log V is the entropy of the uniform distribution.
    x = torch.full((v,), 3.25, dtype=torch.float64)
    assert router.entropy_nats(x) == pytest.approx(math.log(v), rel=1e-12)
    assert router.normalised_entropy(x) == pytest.approx(1.0, rel=1e-12)


@pytest.mark.parametrize("v", VOCABS)
def test_one_hot_distribution_has_entropy_zero(v):
    x = torch.zeros(v, dtype=torch.float64)
    x[v // 2] = 800.0          # every other probability underflows to exactly 0: exercises 0 log 0 = 0
    assert router.entropy_nats(x) == 0.0
    assert router.greedy_token(x) == v // 2


@pytest.mark.parametrize("v", [2, 7, 1024, 152064])
@pytest.mark.parametrize("a", [-3.0, 0.5, 4.0, 12.0])
def test_two_level_closed_form(v, a):
    # logits {a, 0, ..., 0}: p1 = e^a / (e^a + V - 1), the rest share 1 - p1 equally.
    x = torch.zeros(v, dtype=torch.float64)
    x[0] = a
    p1 = math.exp(a) / (math.exp(a) + v - 1)
    rest = (1 - p1) / (v - 1)
    h = -p1 * math.log(p1) - (v - 1) * rest * math.log(rest)
    assert router.entropy_nats(x) == pytest.approx(h, rel=1e-10, abs=1e-13)
    assert router.normalised_entropy(x) == pytest.approx(h / math.log(v), rel=1e-10, abs=1e-13)


def test_brute_force_python_loops_tiny_vocab():
    for v, tag in [(2, 1), (5, 2), (17, 3), (64, 4)]:
        x = (misc_normal(11, tag, v) * 3.0)
        xs = [float(t) for t in x]
        z = sum(math.exp(t) for t in xs)
        ps = [math.exp(t) / z for t in xs]
        h = -sum(p * math.log(p) for p in ps)
        assert router.entropy_nats(x) == pytest.approx(h, rel=1e-12)
        assert router.greedy_token(x) == max(range(v), key=lambda i: xs[i])


def test_matches_library_categorical_entropy():
    x = misc_normal(12, 1, 4096) * 2.5
    lib = float(torch.distributions.Categorical(logits=x).entropy())
    assert router.entropy_nats(x) == pytest.approx(lib, rel=1e-10)
    from scipy.stats import entropy as sp_entropy
    from scipy.special import softmax as sp_softmax
    assert router.entropy_nats(x) == pytest.approx(float(sp_entropy(sp_softmax(x.numpy()))), rel=1e-10)


def test_shift_invariance_and_bounds():
    x = misc_normal(13, 1, 1000) * 4.0
    h = router.entropy_nats(x)
    assert router.entropy_nats(x + 123.456) == pytest.approx(h, rel=1e-9)
    assert router.entropy_nats(x - 9000.0) == pytest.approx(h, rel=1e-9)
    assert 0.0 <= h <= math.log(1000)
    assert 0.0 <= router.normalised_entropy(x) <= 1.0


def test_scaling_logits_up_lowers_entropy():
    x = misc_normal(14, 1, 512)
    hs = [router.entropy_nats(x * s) for s in (0.5, 1.0, 2.0, 4.0, 8.0)]
    assert all(a > b for a, b in zip(hs, hs[1:]))


def test_argmax_lowest_index_among_equals():
    x = torch.tensor([0.0, 5.0, 5.0, -1.0, 5.0], dtype=torch.float64)
    assert router.greedy_token(x) == 1


def test_switch_rule_table():
    # Eq. 2 and Algorithm 1: strict > for the small model handing over, <= for handing back.
    S, L = router.SLM, router.LLM
    assert router.switch(0.30, 0.25, S) == (True, False, L)    # small model uncertain: discard, go to large
    assert router.switch(0.20, 0.25, S) == (False, True, S)    # small model certain: keep, stay
    assert router.switch(0.25, 0.25, S) == (False, True, S)    # equality is NOT above tau
    assert router.switch(0.30, 0.25, L) == (True, True, L)     # large model uncertain: keep, stay on large
    assert router.switch(0.20, 0.25, L) == (False, True, S)    # large model certain: keep, hand back
    assert router.switch(0.25, 0.25, L) == (False, True, S)    # equality hands back


def test_route_record_and_flags():
    x = torch.zeros(8, dtype=torch.float64)
    x[3] = 2.0
    r = router.route(x, tau=0.5, active=router.SLM)
    p1 = math.exp(2.0) / (math.exp(2.0) + 7)
    h = -p1 * math.log(p1) - (1 - p1) * math.log((1 - p1) / 7)
    assert r["token"] == 3
    assert r["h_nats"] == pytest.approx(h, rel=1e-12)
    assert r["h_norm"] == pytest.approx(h / math.log(8), rel=1e-12)
    assert r["max_logit"] == 2.0
    assert r["log_z"] == pytest.approx(math.log(math.exp(2.0) + 7), rel=1e-12)
    hi = h / math.log(8) > 0.5
    assert bool(r["flags"] & router.FLAG_HI) == hi
    assert bool(r["flags"] & router.FLAG_ACCEPT) == (not hi)
    assert bool(r["flags"] & router.FLAG_NEXT_LLM) == hi
    r2 = router.route(x, tau=0.5, active=router.LLM)
    assert r2["flags"] & router.FLAG_ACCEPT


def test_nonfinite_logits_are_flagged_uncertain():
    x = torch.zeros(8, dtype=torch.float64)
    x[1] = float("nan")
    r = router.route(x, tau=0.9, active=router.SLM)
    assert r["flags"] & router.FLAG_NONFINITE and r["flags"] & router.FLAG_HI
    assert not (r["flags"] & router.FLAG_ACCEPT)


def test_sample_token_follows_the_softmax_distribution():
    """Gumbel-max draws against the probabilities themselves, and against the same draws made another way: the
    exponential race (the index with the smallest -ln(u_i) / p_i wins), which is the same event written without
    logarithms of logarithms."""
    import workloads as W
    logits = torch.tensor([2.0, 0.5, -1.0, 1.2, 0.0], dtype=torch.float64)
    p = router.softmax(logits)
    n = 40000
    key = W.stream_key(7, 99)
    u = W.uniform23(key, 0, n * 5).view(n, 5)
    counts = torch.zeros(5)
    for t in range(n):
        tok = router.sample_token(logits, u[t])
        if t < 2000:
            race = int(torch.argmin(-torch.log(u[t]) / p))
            assert tok == race
        counts[tok] += 1
    freq = counts / n
    sigma = torch.sqrt(p * (1 - p) / n)
    assert bool(((freq - p).abs() <= 4.5 * sigma).all()), (freq, p)


def test_sample_token_special_cases():
    import workloads as W
    u = W.uniform23(W.stream_key(1, 2), 0, 64)
    peaked = torch.zeros(64, dtype=torch.float64)
    peaked[17] = 200.0
    assert router.sample_token(peaked, u) == 17                       # a certain token is always drawn
    flat = torch.zeros(64, dtype=torch.float64)
    assert router.sample_token(flat, u) == int(torch.argmax(u))       # equal logits: the largest uniform wins
    same = torch.full((64,), 0.5, dtype=torch.float64)
    assert router.sample_token(flat, same) == 0                       # all equal: the lowest index
    assert float(u.min()) > 0 and float(u.max()) < 1
    assert torch.equal(u.to(torch.float32).double(), u)               # an fp32 holds these uniforms exactly
