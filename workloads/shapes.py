"""Decoder shapes of the stitched pairs and their byte accounting.

The paper names the model families (a 1.5B small model paired with 7B, 14B and
32B large models, Section "Experiments", implementation details) and prints
their bf16 footprint (Table "Memory usage of SLM/LLM models and their KV
caches"); the layer dimensions below are the public Qwen2-family shapes of
those sizes plus two tiny shapes a CPU can run in seconds.
"""

from __future__ import annotations

from dataclasses import dataclass


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    tied_lm_head: bool
    rms_eps: float = 1e-6
    rope_theta: float = 1e6

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def params_per_layer(self) -> int:
        d, f = self.d_model, self.d_ffn
        return self.qkv_rows * d + self.q_dim * d + 3 * d * f + 2 * d


TINY_S = ModelShape("tiny_s", 2, 128, 4, 2, 32, 384, 1024, True)
TINY_L = ModelShape("tiny_l", 4, 256, 8, 2, 32, 768, 1024, False)
S15 = ModelShape("s15", 28, 1536, 12, 2, 128, 8960, 152064, True)
M7 = ModelShape("m7", 28, 3584, 28, 4, 128, 18944, 152064, False)
M14 = ModelShape("m14", 48, 5120, 40, 8, 128, 13824, 152064, False)
M32 = ModelShape("m32", 64, 5120, 40, 8, 128, 27648, 152064, False)

SHAPES = {s.name: s for s in (TINY_S, TINY_L, S15, M7, M14, M32)}

BF16 = 2


def kv_bytes_per_token(s: ModelShape) -> int:
    """K and V rows of one token over all layers, bf16."""
    return 2 * s.n_layers * s.n_kv_heads * s.head_dim * BF16


def weight_bytes_read_per_step(s: ModelShape) -> int:
    """Bytes of weights one forward pass must read: every layer, the LM head,
    the final-norm gains and one embedding row (per input token row: here 1)."""
    n = s.n_layers * s.params_per_layer + s.vocab * s.d_model + s.d_model + s.d_model
    return n * BF16


def weight_bytes_resident(s: ModelShape) -> int:
    n = s.n_layers * s.params_per_layer + s.vocab * s.d_model + s.d_model
    if not s.tied_lm_head:
        n += s.vocab * s.d_model
    return n * BF16


def step_bytes(s: ModelShape, ctx_lens, n_rows: int | None = None) -> int:
    """Algorithmic HBM bytes of one forward invocation.

    ``ctx_lens``: for every sequence in the call, the number of cached tokens
    its attention reads (position of its last row + 1).  Weights are read once
    per call whatever the number of rows; each row writes one token of KV.
    """
    ctx_lens = list(ctx_lens)
    rows = n_rows if n_rows is not None else len(ctx_lens)
    kvb = kv_bytes_per_token(s)
    return weight_bytes_read_per_step(s) + kvb * (sum(ctx_lens) + rows)
