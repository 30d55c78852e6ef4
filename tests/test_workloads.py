"""The synthetic-input recipes: determinism, slice-addressability, statistics,
and the shape arithmetic against the paper's memory table."""
import math

import pytest
import torch

import workloads as W
from workloads import rng, shapes


def test_counter_rng_is_slice_addressable_and_deterministic():
    a = rng.uniform01(3, 7, 0, 1000)
    b = torch.cat([rng.uniform01(3, 7, 0, 123), rng.uniform01(3, 7, 123, 877)])
    assert torch.equal(a, b)
    assert not torch.equal(a, rng.uniform01(4, 7, 0, 1000))
    assert not torch.equal(a, rng.uniform01(3, 8, 0, 1000))
    n1 = rng.normal(3, 7, 0, 512)
    assert torch.equal(n1[100:200], rng.normal(3, 7, 100, 100))


def test_rng_statistics():
    u = rng.uniform01(1, 1, 0, 200000)
    assert 0 < float(u.min()) and float(u.max()) < 1
    assert abs(float(u.mean()) - 0.5) < 5e-3 and abs(float(u.var()) - 1 / 12) < 2e-3
    z = rng.normal(1, 2, 0, 200000)
    assert abs(float(z.mean())) < 1e-2 and abs(float(z.std()) - 1) < 1e-2
    assert abs(float((z ** 4).mean()) - 3) < 0.1
    r = rng.randint(1, 3, 0, 100000, 1024)
    assert int(r.min()) >= 0 and int(r.max()) <= 1023 and len(torch.unique(r)) == 1024


def test_weights_recipe():
    w = W.make_weights(W.TINY_L, 0, 1)
    s = W.TINY_L
    assert w.embed.shape == (1024, 256) and w.lm_head is not w.embed
    assert w.layers[0].w_qkv.shape == ((8 + 4) * 32, 256) and w.layers[0].w_gate_up.shape == (2 * 768, 256)
    assert w.layers[3].w_down.shape == (256, 768) and w.layers[0].w_o.shape == (256, 256)
    assert all(t.dtype == torch.bfloat16 for t in (w.embed, w.layers[0].w_qkv, w.final_norm))
    assert torch.all(w.final_norm == 1) and torch.all(w.layers[1].attn_norm == 1)
    assert abs(float(w.layers[2].w_gate_up.float().std()) - 0.02) < 5e-4
    assert not torch.equal(w.layers[0].w_qkv, w.layers[1].w_qkv)
    tied = W.make_weights(W.TINY_S, 0, 0)
    assert tied.lm_head is tied.embed
    again = W.make_weights(W.TINY_L, 0, 1)
    assert torch.equal(again.layers[2].w_down, w.layers[2].w_down)


def test_prompts_and_scale_schedule():
    wl = W.WORKLOADS["cfg1_tiny_pair"]
    p = W.make_prompt(wl)
    assert p.shape == (32,) and int(p.min()) >= 0 and int(p.max()) < 1024
    s = W.logit_scale(wl, 0, 5000)
    assert s.dtype == torch.float32 and float(s.min()) >= 0.5 and float(s.max()) <= 8.0
    assert abs(float(s.mean()) - 4.25) < 0.1
    assert torch.equal(W.logit_scale(wl, 100, 10), s[100:110])
    w5 = W.WORKLOADS["cfg5_s15_m32_b8"]
    lens = [W.recipes.prompt_length(w5, i) for i in range(8)]
    assert all(512 <= n <= 2048 for n in lens) and len(set(lens)) > 1
    assert W.WORKLOADS["cfg3_s15_m7"].max_ctx == 4608 and w5.max_ctx == 10240


def test_pick_tau_sits_in_a_gap_at_the_percentile():
    h = [i / 100 for i in range(100)]
    tau = W.pick_tau(h, 70.0, 1e-3)
    assert sum(x > tau for x in h) == 30 and all(abs(x - tau) > 4e-3 for x in h)
    # a too-narrow gap at the rank is skipped upward
    h2 = [0.0, 0.1, 0.2, 0.2000001, 0.5, 0.9]
    assert W.pick_tau(h2, 50.0, 1e-3) == pytest.approx(0.35)


def test_shape_arithmetic_against_the_papers_memory_table():
    # Table "Memory usage ... under BF16": per-token KV cache 0.028 / 0.055 / 0.189 / 0.253 MB and
    # weights 3036 / 15640 / 29275 / 63890 MB for the 1.5B / 7B / 14B / 32B models.  The table is
    # measured inside a serving framework, so agreement is to a few per cent, in MiB.
    import os
    mib = 2.0 ** 20
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "memory_table.txt"))
            if l.strip() and not l.startswith("#")]
    table = {r[0]: [float(v) for v in r[1:]] for r in rows}
    for s, key in [(W.S15, "1.5B"), (W.M7, "7B"), (W.M14, "14B"), (W.M32, "32B")]:
        kv_mb, w_mb, at8k, at16k = table[key]
        assert shapes.kv_bytes_per_token(s) / mib == pytest.approx(kv_mb, rel=0.04)
        assert shapes.weight_bytes_resident(s) / mib == pytest.approx(w_mb, rel=0.08)
        # the table's own totals are weights + context * KV per token
        assert at16k - at8k == pytest.approx(8192 * kv_mb, rel=0.02)
        assert (shapes.weight_bytes_resident(s) + 16384 * shapes.kv_bytes_per_token(s)) / mib == pytest.approx(at16k, rel=0.08)
    assert [shapes.kv_bytes_per_token(s) for s in (W.S15, W.M7, W.M14, W.M32)] == [28672, 57344, 196608, 262144]
    # bytes one decode step must read
    assert shapes.weight_bytes_read_per_step(W.S15) == pytest.approx(3087.7e6, rel=1e-4)
    assert shapes.weight_bytes_read_per_step(W.M7) == pytest.approx(14141.0e6, rel=1e-4)
    assert shapes.step_bytes(W.S15, [2560]) == shapes.weight_bytes_read_per_step(W.S15) + 28672 * 2561
