"""Why the oracle rounds only the K/V rows to bf16 and no other activation.

The workload description fixes bf16 weights, fp32 accumulation and a bf16 KV cache; it says nothing about
rounding the inputs of the other matrix products.  A first reading rounded every one of them to bf16.  This
test shows, on the oracle alone (no GPU code involved), that under that reading two EQUIVALENT computations -
here the same model with its embedding perturbed by one part in 10^7 (10^6 for a 4-layer model), the size of
the difference between fp32 and fp64 accumulation - end up with logits that differ by 1e-2 .. 3e-2, the whole
2e-2 tolerance the benchmark spec states, so no implementation could be compared with any other; with only the K/V rows
rounded the same computations stay 10 to 100 times closer (at most 2e-4 at 28 layers).  A bf16 rounding turns a relative difference delta into roughly sqrt(delta * 2^-8) (a few
elements flip by a whole bf16 step), and a chain of roundings drives it to the bf16 step itself.
"""
import torch

import workloads as W
from oracle import decoder

F64 = torch.float64


class RoundsEveryMatmulInput(decoder.OracleModel):
    """The oracle's forward pass with the first reading's extra rounding points: the normalised inputs of the
    QKV, gate/up and LM-head products, the rotated query, the attention output and the SwiGLU output are
    rounded to bf16 as well (K/V rows as in the oracle)."""

    def forward(self, tokens, pos0, slot=0, logit_scale=1.0, want_hidden=False):
        s, r = self.s, decoder.round_bf16
        n = len(tokens)
        hq, hkv, hd = s.n_q_heads, s.n_kv_heads, s.head_dim
        h = self._f64("embed", self.w.embed)[list(tokens)].clone()
        for l, lw in enumerate(self.w.layers):
            x = r(decoder.rmsnorm(h, self._f64((l, "an"), lw.attn_norm), s.rms_eps))
            qkv = x @ self._f64((l, "qkv"), lw.w_qkv).T
            q = qkv[:, :hq * hd].reshape(n, hq, hd)
            k = qkv[:, hq * hd:(hq + hkv) * hd].reshape(n, hkv, hd)
            v = qkv[:, (hq + hkv) * hd:].reshape(n, hkv, hd)
            for i in range(n):
                self.k_cache[l, slot, :, pos0 + i] = r(decoder.rope(k[i], pos0 + i, s.rope_theta))
                self.v_cache[l, slot, :, pos0 + i] = r(v[i])
            o = torch.empty(n, hq * hd, dtype=F64)
            for i in range(n):
                qi = r(decoder.rope(q[i], pos0 + i, s.rope_theta))
                ctx = pos0 + i + 1
                o[i] = decoder.attention(qi, self.k_cache[l, slot, :, :ctx], self.v_cache[l, slot, :, :ctx]).reshape(-1)
            h = h + r(o) @ self._f64((l, "o"), lw.w_o).T
            x = r(decoder.rmsnorm(h, self._f64((l, "mn"), lw.mlp_norm), s.rms_eps))
            gu = x @ self._f64((l, "gu"), lw.w_gate_up).T
            a = r(decoder.silu(gu[:, :s.d_ffn]) * gu[:, s.d_ffn:])
            h = h + a @ self._f64((l, "dn"), lw.w_down).T
        x_last = r(decoder.rmsnorm(h[-1], self._f64("fn", self.w.final_norm), s.rms_eps))
        lm = self._f64("embed", self.w.embed) if s.tied_lm_head else self._f64("lm", self.w.lm_head)
        return dict(logits=(lm @ x_last) * float(logit_scale))


def logits_of(cls, shape, draw, eps):
    """Logits of the last of 100 prompt tokens (logit scale 8); draw = None: the model as drawn; otherwise its
    embedding is multiplied by (1 + eps * N(0,1)) with noise stream `draw`."""
    w = W.make_weights(shape, 3, 1)
    m = cls(w, 128)
    if draw is not None:
        noise = W.rng.normal(3, 4242 + draw, 0, w.embed.numel()).view(w.embed.shape)
        m._w64["embed"] = w.embed.double() * (1.0 + eps * noise)
    toks = W.rng.randint(3, 5, 0, 100, shape.vocab).tolist()
    return m.forward(toks, 0, logit_scale=8.0)["logits"]


def divergences(cls, n_layers, eps, draws=4):
    """Largest logit difference between the model and each of `draws` perturbed copies of it."""
    shape = W.ModelShape("rounding_probe", n_layers, 256, 8, 2, 32, 768, 1024, False)
    base = logits_of(cls, shape, None, eps)
    return [float((base - logits_of(cls, shape, t, eps)).abs().max()) for t in range(draws)]


def test_without_rounding_points_the_subclass_is_the_oracle():
    """The subclass differs from the oracle by its rounding points only: with rounding made the identity the
    two forward passes agree to fp64 rounding."""
    shape = W.ModelShape("rounding_probe", 2, 256, 8, 2, 32, 768, 1024, False)
    w = W.make_weights(shape, 3, 1)
    toks = W.rng.randint(3, 6, 0, 12, shape.vocab).tolist()
    saved = decoder.round_bf16
    try:
        decoder.round_bf16 = lambda x: x
        a = RoundsEveryMatmulInput(w, 32).forward(toks, 0, logit_scale=3.0)["logits"]
        b = decoder.OracleModel(w, 32, contract=False).forward(toks, 0, logit_scale=3.0)["logits"]
    finally:
        decoder.round_bf16 = saved
    assert float((a - b).abs().max()) < 1e-12


# (layers, relative perturbation): 28 layers at 1e-7; 4 layers need 1e-6 before an element reliably flips
CASES = [(28, 1e-7), (4, 1e-6)]


def test_rounding_every_matmul_input_makes_equivalent_runs_diverge_beyond_the_tolerance():
    for n_layers, eps in CASES:
        d = divergences(RoundsEveryMatmulInput, n_layers, eps)
        assert min(d) >= 1e-2, f"{n_layers} layers: {d}"           # measured 1.3e-2 .. 3.4e-2


def test_kv_rounding_alone_amplifies_fp32_sized_differences_past_a_millinat():
    """The rounding the workload does prescribe (bf16 K/V rows) is itself an amplifier: two oracle runs of a 28-layer
    model whose inputs differ by 3 parts in 10^6 - what fp32 accumulation over a few thousand terms leaves - end up
    with logits 5e-4 .. 4.4e-3 apart.  A call that prefills many rows at once on a deep model therefore cannot be
    compared with another implementation's to 1e-3 nats as a whole; the GPU parity tests compare the rows written
    and the last row's distribution given those rows instead."""
    d = divergences(decoder.OracleModel, 28, 3e-6)
    assert max(d) >= 1e-3 and max(d) <= 2e-2, d


def test_rounding_only_the_kv_rows_keeps_equivalent_runs_an_order_of_magnitude_closer():
    for (n_layers, eps), cap in zip(CASES, (5e-4, 2e-3)):
        d = divergences(decoder.OracleModel, n_layers, eps)
        assert max(d) <= cap, f"{n_layers} layers: {d}"             # measured 2.5e-7 .. 1.7e-4 and 2.1e-4 .. 1.3e-3
