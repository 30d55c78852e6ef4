"""The five synthetic workloads: weights, prompts, logit-scale schedule, tau.

They stand in for the paper's math benchmarks and real checkpoints (Section
"Experiments"), none of which exist offline: model sizes, batch size 1 (and 8),
context budgets and the share of tokens routed to the large model follow the
paper; the numbers inside the tensors are seeded noise.

Recipe (all seeded through ``workloads.rng``):
  * weights: bf16( 0.02 * N(0,1) ), one stream per (role, layer, tensor);
    RMSNorm gains are exactly 1.0; the fused tensors ``w_qkv`` (rows: all query
    heads, then key heads, then value heads) and ``w_gate_up`` (rows: gate,
    then up) are drawn directly in fused form;
  * prompt ids: uniform in [0, vocab);
  * logit scale: ``s_p = 0.5 + 7.5 * u(p)`` keyed on the absolute position p of
    the token being predicted, the same for both models, so the schedule does
    not depend on the routing path;
  * tau: a percentile of the small model's normalised entropies over a
    small-model-only run, placed in the middle of a gap between two samples.
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

from . import rng
from .shapes import ModelShape, TINY_S, TINY_L, S15, M7, M14, M32

# stream ids -----------------------------------------------------------------
_K_EMBED, _K_LMHEAD, _K_QKV, _K_O, _K_GATEUP, _K_DOWN = 1, 2, 3, 4, 5, 6
_STREAM_PROMPT = (1 << 20)               # + sequence index
_STREAM_SCALE = (1 << 20) + 1 * 4096     # + sequence index
_STREAM_PROMPT_LEN = (1 << 20) + 2 * 4096
_STREAM_MISC = (1 << 20) + 3 * 4096      # + caller's tag
_STREAM_ROUTER = (1 << 20) + 4 * 4096    # + tensor index


def _stream(role: int, layer: int, kind: int) -> int:
    return (role * 512 + (layer + 1)) * 16 + kind


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    slm: ModelShape
    llm: Optional[ModelShape]
    prompt_len: int            # per sequence; for n_seqs > 1 see prompt_len_range
    n_decode: int              # accepted tokens per sequence
    tau_percentile: Optional[float]
    n_seqs: int = 1
    prompt_len_range: Optional[tuple] = None
    max_span: int = 64

    @property
    def max_ctx(self) -> int:
        longest = self.prompt_len_range[1] if self.prompt_len_range else self.prompt_len
        return longest + self.n_decode


WORKLOADS = {
    "cfg1_tiny_pair": Workload("cfg1_tiny_pair", 0, TINY_S, TINY_L, 32, 64, 70.0),
    "cfg2_s15_decode": Workload("cfg2_s15_decode", 1, S15, None, 2048, 512, None),
    "cfg3_s15_m7": Workload("cfg3_s15_m7", 2, S15, M7, 512, 4096, 70.0),
    "cfg4_s15_m14": Workload("cfg4_s15_m14", 3, S15, M14, 1024, 8192, 80.0),
    "cfg5_s15_m32_b8": Workload("cfg5_s15_m32_b8", 4, S15, M32, 2048, 8192, 70.0,
                                n_seqs=8, prompt_len_range=(512, 2048)),
}


@dataclass
class LayerWeights:
    attn_norm: torch.Tensor    # [d] bf16
    w_qkv: torch.Tensor        # [(Hq+2Hkv)*hd, d] bf16
    w_o: torch.Tensor          # [d, Hq*hd] bf16
    mlp_norm: torch.Tensor     # [d] bf16
    w_gate_up: torch.Tensor    # [2*ffn, d] bf16
    w_down: torch.Tensor       # [d, ffn] bf16


@dataclass
class ModelWeights:
    shape: ModelShape
    embed: torch.Tensor        # [V, d] bf16
    lm_head: torch.Tensor      # [V, d] bf16 (the same tensor as embed when tied)
    final_norm: torch.Tensor   # [d] bf16
    layers: List[LayerWeights] = field(default_factory=list)

    def to(self, device) -> "ModelWeights":
        emb = self.embed.to(device)
        lm = emb if self.shape.tied_lm_head else self.lm_head.to(device)
        return ModelWeights(
            self.shape, emb, lm, self.final_norm.to(device),
            [LayerWeights(*(getattr(l, f).to(device) for f in
                            ("attn_norm", "w_qkv", "w_o", "mlp_norm", "w_gate_up", "w_down")))
             for l in self.layers])


def _normal_bf16(seed: int, stream: int, rows: int, cols: int, std: float, device,
                 chunk: int = 1 << 24) -> torch.Tensor:
    out = torch.empty(rows * cols, dtype=torch.bfloat16, device=device)
    n = rows * cols
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        z = rng.normal(seed, stream, s, c, device)
        out[s:s + c] = (z * std).to(torch.float32).to(torch.bfloat16)
    return out.view(rows, cols)


def make_weights(shape: ModelShape, seed: int, role: int, device="cpu",
                 std: float = 0.02) -> ModelWeights:
    """role: 0 = small model, 1 = large model of the pair."""
    d = shape.d_model
    ones = lambda: torch.ones(d, dtype=torch.bfloat16, device=device)  # noqa: E731
    embed = _normal_bf16(seed, _stream(role, -1, _K_EMBED), shape.vocab, d, std, device)
    lm_head = embed if shape.tied_lm_head else _normal_bf16(
        seed, _stream(role, -1, _K_LMHEAD), shape.vocab, d, std, device)
    w = ModelWeights(shape, embed, lm_head, ones())
    for l in range(shape.n_layers):
        w.layers.append(LayerWeights(
            ones(),
            _normal_bf16(seed, _stream(role, l, _K_QKV), shape.qkv_rows, d, std, device),
            _normal_bf16(seed, _stream(role, l, _K_O), d, shape.q_dim, std, device),
            ones(),
            _normal_bf16(seed, _stream(role, l, _K_GATEUP), 2 * shape.d_ffn, d, std, device),
            _normal_bf16(seed, _stream(role, l, _K_DOWN), d, shape.d_ffn, std, device),
        ))
    return w


def prompt_length(wl: Workload, seq: int = 0) -> int:
    if wl.prompt_len_range is None:
        return wl.prompt_len
    lo, hi = wl.prompt_len_range
    return lo + int(rng.randint(wl.seed, _STREAM_PROMPT_LEN, seq, 1, hi - lo + 1)[0])


def make_prompt(wl: Workload, seq: int = 0, length: Optional[int] = None) -> torch.Tensor:
    """int64 token ids of sequence ``seq`` (CPU tensor)."""
    n = prompt_length(wl, seq) if length is None else length
    return rng.randint(wl.seed, _STREAM_PROMPT + seq, 0, n, wl.slm.vocab)


def logit_scale(wl: Workload, pos_start: int, count: int, seq: int = 0) -> torch.Tensor:
    """fp32 scale for predicting the tokens at absolute positions
    pos_start .. pos_start+count-1 of sequence ``seq`` (CPU tensor)."""
    u = rng.uniform01(wl.seed, _STREAM_SCALE + seq, pos_start, count)
    return (0.5 + 7.5 * u).to(torch.float32)


def misc_normal(seed: int, tag: int, count: int) -> torch.Tensor:
    """fp64 standard normals for ad-hoc test inputs (module-level parity cases)."""
    return rng.normal(seed, _STREAM_MISC + tag, 0, count)


def misc_uniform(seed: int, tag: int, count: int) -> torch.Tensor:
    return rng.uniform01(seed, _STREAM_MISC + tag, 0, count)


def pick_tau(h_norm: Sequence[float], percentile: float, min_gap: float) -> float:
    """Threshold at the given percentile of the samples, placed mid-way between
    two neighbouring sorted samples at least ``min_gap`` apart (searching upward
    from the nearest-rank position), so that no sample sits on the threshold."""
    v = sorted(float(x) for x in h_norm)
    n = len(v)
    if n < 2:
        raise ValueError("need at least two entropy samples")
    k = min(max(int(-(-percentile * n // 100)) - 1, 0), n - 2)   # nearest rank, 0-based
    for j in list(range(k, n - 1)) + list(range(k - 1, -1, -1)):
        if v[j + 1] - v[j] >= min_gap:
            return 0.5 * (v[j] + v[j + 1])
    return 0.5 * (v[k] + v[k + 1])


@dataclass
class RouterWeights:
    """Weights of the R-Stitch+ router (Section "Architecture and Overhead of Router": six residual feed-forward
    blocks, a normalisation, a two-output linear layer).  All bf16.  Data holder only."""
    w1: List[torch.Tensor]     # 6 x [r, d]
    b1: List[torch.Tensor]     # 6 x [r]
    w2: List[torch.Tensor]     # 6 x [d, r]
    b2: List[torch.Tensor]     # 6 x [d]
    ln_gain: torch.Tensor      # [d]
    ln_bias: torch.Tensor      # [d]
    w_head: torch.Tensor       # [2, d]
    b_head: torch.Tensor       # [2]

    def tensors(self) -> List[torch.Tensor]:
        return self.w1 + self.b1 + self.w2 + self.b2 + [self.ln_gain, self.ln_bias, self.w_head, self.b_head]

    def n_params(self) -> int:
        return sum(t.numel() for t in self.tensors())

    def to(self, device) -> "RouterWeights":
        mv = lambda ts: [t.to(device) for t in ts]  # noqa: E731
        return RouterWeights(mv(self.w1), mv(self.b1), mv(self.w2), mv(self.b2), self.ln_gain.to(device),
                             self.ln_bias.to(device), self.w_head.to(device), self.b_head.to(device))


def make_router_weights(d: int, r: int, seed: int, device="cpu") -> RouterWeights:
    """Seeded synthetic router (the trained one of the paper does not exist offline): matrices N(0, 0.05), block
    biases N(0, 0.002) (small beside a hidden state of a random N(0, 0.02) model, so that the outputs depend on the
    state), head bias N(0, 0.05), LayerNorm gain 1 + N(0, 0.1) and bias N(0, 0.1), all rounded to bf16."""
    def draw(idx, count, std, shift=0.0):
        z = rng.normal(seed, _STREAM_ROUTER + idx, 0, count, device)
        return (shift + std * z).to(torch.float32).to(torch.bfloat16)
    w = RouterWeights([], [], [], [], draw(60, d, 0.1, 1.0), draw(61, d, 0.1), draw(62, 2 * d, 0.05).view(2, d), draw(63, 2, 0.05))
    for i in range(6):
        w.w1.append(draw(4 * i, r * d, 0.05).view(r, d))
        w.b1.append(draw(4 * i + 1, r, 0.002))
        w.w2.append(draw(4 * i + 2, d * r, 0.05).view(d, r))
        w.b2.append(draw(4 * i + 3, d, 0.002))
    return w
