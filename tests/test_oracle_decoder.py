"""Pins for oracle/decoder.py.

Module-level closed forms and library routines, then the whole forward pass
(rounding switched off) against the transformers library's own Qwen2 decoder
built with the same synthetic weights - an implementation that shares nothing
with the oracle.
"""
import math

import pytest
import torch
import torch.nn.functional as F

import workloads as W
from oracle import decoder
from workloads.recipes import misc_normal

F64 = torch.float64


def rnd(seed, tag, *shape):
    n = 1
    for s in shape:
        n *= s
    return misc_normal(seed, tag, n).view(*shape)


# ---------------------------------------------------------------- rounding
def test_round_bf16_ties_to_even():
    x = torch.tensor([1 + 2 ** -8, 1 + 2 ** -8 + 2 ** -20, 1 + 3 * 2 ** -8, -(1 + 2 ** -8), 0.02], dtype=F64)
    r = decoder.round_bf16(x)
    assert r[0] == 1.0 and r[1] == 1 + 2 ** -7 and r[2] == 1 + 2 ** -6 and r[3] == -1.0
    assert abs(float(r[4]) - 0.02) <= 0.02 * 2 ** -8 and float(r[4]) != 0.02


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_constant_vector_closed_form():
    c, eps = 3.0, 1e-6
    x = torch.full((5, 64), c, dtype=F64)
    g = torch.full((64,), 2.0, dtype=F64)
    y = decoder.rmsnorm(x, g, eps)
    assert torch.allclose(y, torch.full_like(x, 2.0 * c / math.sqrt(c * c + eps)), rtol=1e-14)


def test_rmsnorm_matches_library():
    x, g = rnd(1, 1, 7, 96), rnd(1, 2, 96)
    assert torch.allclose(decoder.rmsnorm(x, g, 1e-6), F.rms_norm(x, (96,), g, 1e-6), rtol=1e-12, atol=1e-14)


def test_rmsnorm_eps_is_inside_the_root():
    x = torch.zeros(4, dtype=F64)
    x[0] = 1e-3
    y = decoder.rmsnorm(x, torch.ones(4, dtype=F64), 1e-6)
    assert float(y[0]) == pytest.approx(1e-3 / math.sqrt(1e-6 / 4 + 1e-6), rel=1e-12)


# ---------------------------------------------------------------- RoPE
def test_rope_position_zero_is_identity_and_norm_is_preserved():
    x = rnd(2, 1, 6, 128)
    assert torch.equal(decoder.rope(x, 0, 1e6), x)
    for pos in (1, 17, 4607, 10239):
        y = decoder.rope(x, pos, 1e6)
        assert torch.allclose(y.norm(dim=-1), x.norm(dim=-1), rtol=1e-13)
        # every rotated pair keeps its own length too
        assert torch.allclose(y[..., :64] ** 2 + y[..., 64:] ** 2, x[..., :64] ** 2 + x[..., 64:] ** 2, rtol=1e-12)


def test_rope_two_dimensional_case_is_a_plain_rotation():
    # head_dim 2: one pair, frequency theta^0 = 1, so the angle is the position itself.
    y = decoder.rope(torch.tensor([1.0, 0.0], dtype=F64), 3, 1e6)
    assert torch.allclose(y, torch.tensor([math.cos(3.0), math.sin(3.0)], dtype=F64), rtol=1e-14)


def test_rope_frequencies():
    a = decoder.rope_angles(5, 8, 1e6)
    want = [5 * 1e6 ** (-2 * i / 8) for i in range(4)]
    assert torch.allclose(a, torch.tensor(want, dtype=F64), rtol=1e-13)


def test_rope_inner_product_depends_on_relative_position_only():
    q, k = rnd(3, 1, 128), rnd(3, 2, 128)
    ref = decoder.rope(q, 9, 1e6) @ decoder.rope(k, 4, 1e6)
    for shift in (1, 100, 4000):
        assert float(decoder.rope(q, 9 + shift, 1e6) @ decoder.rope(k, 4 + shift, 1e6)) == pytest.approx(float(ref), rel=1e-9)


# ---------------------------------------------------------------- attention
def test_attention_over_single_token_returns_its_value_row():
    q, k, v = rnd(4, 1, 12, 128), rnd(4, 2, 2, 1, 128), rnd(4, 3, 2, 1, 128)
    o = decoder.attention(q, k, v)
    for j in range(12):
        assert torch.allclose(o[j], v[j // 6, 0], rtol=1e-14)


def test_attention_with_equal_keys_averages_values():
    q, v = rnd(5, 1, 4, 32), rnd(5, 2, 2, 9, 32)
    k = rnd(5, 3, 2, 1, 32).expand(2, 9, 32).contiguous()
    o = decoder.attention(q, k, v)
    for j in range(4):
        assert torch.allclose(o[j], v[j // 2].mean(dim=0), rtol=1e-12)


@pytest.mark.parametrize("hq,hkv,hd,n", [(4, 2, 32, 37), (12, 2, 128, 70), (8, 8, 32, 5), (28, 4, 128, 33)])
def test_attention_matches_library_sdpa(hq, hkv, hd, n):
    q, k, v = rnd(6, 1, hq, hd), rnd(6, 2, hkv, n, hd), rnd(6, 3, hkv, n, hd)
    ref = F.scaled_dot_product_attention(q.view(1, hq, 1, hd), k.view(1, hkv, n, hd), v.view(1, hkv, n, hd),
                                         enable_gqa=(hq != hkv)).view(hq, hd)
    assert torch.allclose(decoder.attention(q, k, v), ref, rtol=1e-10, atol=1e-13)


def test_attention_peaked_query_selects_one_row():
    hd, n = 32, 50
    k = torch.zeros(1, n, hd, dtype=F64)
    v = rnd(7, 1, 1, n, hd)
    k[0, 31, 0] = 1.0
    q = torch.zeros(1, hd, dtype=F64)
    q[0, 0] = 1e4
    assert torch.allclose(decoder.attention(q, k, v)[0], v[0, 31], rtol=1e-12)


# ---------------------------------------------------------------- MLP pieces
def test_silu():
    z = rnd(8, 1, 100) * 4
    assert float(decoder.silu(torch.zeros(1, dtype=F64))) == 0.0
    assert torch.allclose(decoder.silu(z), F.silu(z), rtol=1e-13, atol=1e-15)
    assert float(decoder.silu(torch.tensor(1.0, dtype=F64))) == pytest.approx(1 / (1 + math.exp(-1.0)), rel=1e-14)


# ---------------------------------------------------------------- whole model vs an independent library decoder
def hf_model(w):
    from transformers import Qwen2Config, Qwen2ForCausalLM
    s = w.shape
    cfg = Qwen2Config(vocab_size=s.vocab, hidden_size=s.d_model, intermediate_size=s.d_ffn,
                      num_hidden_layers=s.n_layers, num_attention_heads=s.n_q_heads,
                      num_key_value_heads=s.n_kv_heads, max_position_embeddings=4096,
                      rms_norm_eps=s.rms_eps, rope_theta=s.rope_theta,
                      tie_word_embeddings=s.tied_lm_head, attn_implementation="eager",
                      use_sliding_window=False)
    assert cfg.head_dim == s.head_dim if hasattr(cfg, "head_dim") else True
    m = Qwen2ForCausalLM(cfg).double().eval()
    hq, hkv, hd = s.n_q_heads, s.n_kv_heads, s.head_dim
    sd = {"model.embed_tokens.weight": w.embed.double(), "model.norm.weight": w.final_norm.double(),
          "lm_head.weight": w.lm_head.double()}
    for l, lw in enumerate(w.layers):
        p = f"model.layers.{l}."
        qkv = lw.w_qkv.double()
        sd[p + "self_attn.q_proj.weight"] = qkv[:hq * hd]
        sd[p + "self_attn.k_proj.weight"] = qkv[hq * hd:(hq + hkv) * hd]
        sd[p + "self_attn.v_proj.weight"] = qkv[(hq + hkv) * hd:]
        sd[p + "self_attn.q_proj.bias"] = torch.zeros(hq * hd, dtype=F64)
        sd[p + "self_attn.k_proj.bias"] = torch.zeros(hkv * hd, dtype=F64)
        sd[p + "self_attn.v_proj.bias"] = torch.zeros(hkv * hd, dtype=F64)
        sd[p + "self_attn.o_proj.weight"] = lw.w_o.double()
        gu = lw.w_gate_up.double()
        sd[p + "mlp.gate_proj.weight"] = gu[:s.d_ffn]
        sd[p + "mlp.up_proj.weight"] = gu[s.d_ffn:]
        sd[p + "mlp.down_proj.weight"] = lw.w_down.double()
        sd[p + "input_layernorm.weight"] = lw.attn_norm.double()
        sd[p + "post_attention_layernorm.weight"] = lw.mlp_norm.double()
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in k or "lm_head" in k for k in missing), (missing, unexpected)
    return m


@pytest.mark.parametrize("shape,role", [(W.TINY_S, 0), (W.TINY_L, 1)])
def test_forward_without_rounding_matches_transformers_qwen2(shape, role):
    # std 0.1 instead of 0.02 so that attention and the MLP actually shape the logits
    w = W.make_weights(shape, seed=5, role=role, std=0.1)
    toks = W.rng.randint(5, 99, 0, 40, shape.vocab).tolist()
    hf = hf_model(w)
    with torch.no_grad():
        ref = hf(torch.tensor([toks])).logits[0]                  # [40, V], causal
    # one invocation over the whole span.  The library evaluates its rotary
    # cos/sin table in fp32 whatever the model dtype, so agreement stops near
    # 1e-6 on logits of magnitude ~3; a structural slip would show as O(1).
    tol = dict(rtol=0, atol=2e-5)
    m = decoder.OracleModel(w, max_ctx=64, contract=False)
    out = m.forward(toks, 0)["logits"]
    assert torch.allclose(out, ref[-1], **tol)
    # the same sequence fed as prefill(17) + catch-up(5) + decode steps: every
    # invocation must reproduce the causal logits at its last position
    m2 = decoder.OracleModel(w, max_ctx=64, contract=False)
    cuts = [(0, 17), (17, 22)] + [(i, i + 1) for i in range(22, 40)]
    for a, b in cuts:
        lg = m2.forward(toks[a:b], a)["logits"]
        assert torch.allclose(lg, ref[b - 1], **tol), (a, b)
    assert torch.allclose(m.k_cache, m2.k_cache, rtol=1e-10, atol=1e-12)
    assert float(ref[-1].std()) > 0.5      # the comparison is not between two near-zero vectors


def test_logit_scale_multiplies_logits():
    w = W.make_weights(W.TINY_S, seed=6, role=0)
    toks = [3, 1, 4, 1, 5]
    a = decoder.OracleModel(w, 16).forward(toks, 0)["logits"]
    b = decoder.OracleModel(w, 16).forward(toks, 0, logit_scale=4.5)["logits"]
    assert torch.allclose(b, a * 4.5, rtol=1e-14)


def test_rounding_contract_stays_close_to_exact_arithmetic_and_is_applied():
    w = W.make_weights(W.TINY_L, seed=7, role=1, std=0.05)
    toks = W.rng.randint(7, 99, 0, 24, 1024).tolist()
    exact = decoder.OracleModel(w, 32, contract=False).forward(toks, 0)["logits"]
    m = decoder.OracleModel(w, 32, contract=True)
    rounded = m.forward(toks, 0)["logits"]
    err = float((exact - rounded).abs().max())
    assert 0 < err < 0.005 * float(exact.abs().max())
    # what is stored in the cache is representable in bf16
    assert torch.equal(m.k_cache, decoder.round_bf16(m.k_cache))
    assert torch.equal(m.v_cache, decoder.round_bf16(m.v_cache))


def test_catchup_equals_sequential_decode_under_the_contract():
    w = W.make_weights(W.TINY_S, seed=8, role=0)
    toks = W.rng.randint(8, 99, 0, 20, 1024).tolist()
    a = decoder.OracleModel(w, 32)
    a.forward(toks[:9], 0)
    la = a.forward(toks[9:], 9)["logits"]
    b = decoder.OracleModel(w, 32)
    for i, t in enumerate(toks):
        lb = b.forward([t], i)["logits"]
    assert torch.allclose(la, lb, rtol=1e-9, atol=1e-11)
    assert torch.allclose(a.k_cache, b.k_cache, rtol=0, atol=1e-12)


def test_identity_lm_head_returns_the_normalised_hidden_state():
    # vocab == d_model and an identity LM head: logits are the final normalised hidden state
    s = W.ModelShape("id", 1, 64, 2, 1, 32, 96, 64, False)
    w = W.make_weights(s, seed=9, role=0)
    w.lm_head = torch.eye(64, dtype=torch.bfloat16)
    m = decoder.OracleModel(w, 8)
    out = m.forward([5, 6, 7], 0, want_hidden=True)
    assert torch.equal(out["logits"], out["x_last"])
    h = out["hidden"][-1]
    assert torch.allclose(out["x_last"], h / torch.sqrt((h * h).mean() + 1e-6), rtol=1e-14, atol=0)


def test_span_must_fit_cache():
    w = W.make_weights(W.TINY_S, seed=8, role=0)
    with pytest.raises(ValueError):
        decoder.OracleModel(w, 8).forward([1, 2, 3], 6)
