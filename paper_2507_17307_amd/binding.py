"""ctypes binding of librstitch.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/rstitch.h).
Torch tensors are used as device buffers; what crosses the boundary is their
``data_ptr()`` and the raw handle of torch's current HIP stream.  ``Model`` is a
convenience holder that keeps the borrowed buffers alive for the lifetime of the
C handle; it adds no arithmetic.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

RS_SLM, RS_LLM = 0, 1
FLAG_HI, FLAG_ACCEPT, FLAG_NEXT_LLM, FLAG_NONFINITE, FLAG_BADARG, FLAG_ABORTED, FLAG_ROUTER_STAY = 1, 2, 4, 8, 16, 32, 64

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path() -> str:
    return os.path.join(_HERE, "librstitch.so")


class RsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"rstitch status {status}: {message}")
        self.status = status


class RsConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab",
        "tied_lm_head", "max_ctx", "max_seqs", "max_rows")] + [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class _RsWeights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + [
        (n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "w_qkv", "w_o", "mlp_norm", "w_gate_up", "w_down")]


class _RsRouterWeights(C.Structure):
    _fields_ = [("d", C.c_int32), ("r", C.c_int32), ("ln_eps", C.c_float)] + [
        (n, C.POINTER(C.c_void_p)) for n in ("w1", "b1", "w2", "b2")] + [
        (n, C.c_void_p) for n in ("ln_gain", "ln_bias", "w_head", "b_head")]


def _load() -> C.CDLL:
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
            "or python paper_2507_17307_amd/build.py). There is no fallback path.")
    lib = C.CDLL(path)
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    lib.rs_last_error.restype = C.c_char_p
    lib.rs_last_error.argtypes = []
    lib.rs_abi_version.restype = i32
    lib.rs_abi_version.argtypes = []
    lib.rs_workspace_bytes.restype = sz
    lib.rs_workspace_bytes.argtypes = [C.POINTER(RsConfig)]
    lib.rs_kv_bytes.restype = sz
    lib.rs_kv_bytes.argtypes = [C.POINTER(RsConfig)]
    lib.rs_create_model.restype = i32
    lib.rs_create_model.argtypes = [C.POINTER(RsConfig), C.POINTER(_RsWeights), vp, vp, vp, sz, C.POINTER(vp)]
    lib.rs_destroy_model.restype = i32
    lib.rs_destroy_model.argtypes = [vp]
    lib.rs_decode_step.restype = i32
    lib.rs_decode_step.argtypes = [vp, i32, vp, vp, vp, vp, f32, i32, vp, vp, vp]
    lib.rs_catchup_prefill.restype = i32
    lib.rs_catchup_prefill.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, f32, i32, vp, vp, vp]
    lib.rs_route_scratch_bytes.restype = sz
    lib.rs_route_scratch_bytes.argtypes = [i32, i32]
    lib.rs_route.restype = i32
    lib.rs_route.argtypes = [vp, i32, i32, vp, f32, i32, vp, vp, sz, vp]
    lib.rs_set_sampling.restype = i32
    lib.rs_set_sampling.argtypes = [vp, i32, C.c_uint64]
    lib.rs_route_plus.restype = i32
    lib.rs_route_plus.argtypes = [vp, vp, i32, C.POINTER(_RsRouterWeights), i32, vp, vp, vp]
    lib.rs_route_static.restype = i32
    lib.rs_route_static.argtypes = [vp, i32, i32, vp, f32, i32, vp, vp]
    lib.rs_stitch_generate.restype = i32
    lib.rs_stitch_generate.argtypes = [vp, vp, i32, vp, i32, i32, i32, i32, vp, f32, i32, vp, i32, vp, vp]
    lib.rs_set_spin_limit.restype = i32
    lib.rs_set_spin_limit.argtypes = [vp, C.c_uint32]
    lib.rs_set_phase_timer.restype = i32
    lib.rs_set_phase_timer.argtypes = [vp, i32, i32, vp, vp]
    return lib


lib = _load()


def _check(status: int) -> None:
    if status != 0:
        raise RsError(status, rs_last_error())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


# ------------------------------------------------------------------ plain entry points
def rs_last_error() -> str:
    return lib.rs_last_error().decode()


def rs_abi_version() -> int:
    return lib.rs_abi_version()


def rs_workspace_bytes(cfg: RsConfig) -> int:
    return lib.rs_workspace_bytes(C.byref(cfg))


def rs_kv_bytes(cfg: RsConfig) -> int:
    return lib.rs_kv_bytes(C.byref(cfg))


def rs_create_model(cfg: RsConfig, weights, kv_k: torch.Tensor, kv_v: torch.Tensor,
                    workspace: torch.Tensor) -> int:
    """weights: object with embed, lm_head, final_norm and layers[*].{attn_norm,w_qkv,w_o,mlp_norm,
    w_gate_up,w_down} as contiguous bf16 device tensors.  Returns the opaque handle."""
    n = cfg.n_layers
    arrs = {}
    for name in ("attn_norm", "w_qkv", "w_o", "mlp_norm", "w_gate_up", "w_down"):
        arrs[name] = (C.c_void_p * n)(*[getattr(l, name).data_ptr() for l in weights.layers])
    w = _RsWeights(weights.embed.data_ptr(), weights.lm_head.data_ptr(), weights.final_norm.data_ptr(),
                   *[C.cast(arrs[k], C.POINTER(C.c_void_p)) for k in
                     ("attn_norm", "w_qkv", "w_o", "mlp_norm", "w_gate_up", "w_down")])
    handle = C.c_void_p()
    _check(lib.rs_create_model(C.byref(cfg), C.byref(w), kv_k.data_ptr(), kv_v.data_ptr(), workspace.data_ptr(),
                               workspace.numel() * workspace.element_size(), C.byref(handle)))
    return handle.value


def rs_destroy_model(handle: int) -> None:
    _check(lib.rs_destroy_model(handle))


def rs_decode_step(handle: int, n_seqs: int, d_seq_slot, d_token, d_pos, d_logit_scale, tau: float, active: int,
                   d_out, d_logits=None, stream=None) -> None:
    _check(lib.rs_decode_step(handle, n_seqs, _ptr(d_seq_slot), _ptr(d_token), _ptr(d_pos), _ptr(d_logit_scale),
                              tau, active, _ptr(d_out), _ptr(d_logits), _stream(stream)))


def rs_catchup_prefill(handle: int, n_seqs: int, n_rows: int, d_seq_slot, d_tokens, d_span_offset, d_pos0,
                       d_logit_scale, tau: float, active: int, d_out, d_logits=None, stream=None) -> None:
    _check(lib.rs_catchup_prefill(handle, n_seqs, n_rows, _ptr(d_seq_slot), _ptr(d_tokens), _ptr(d_span_offset),
                                  _ptr(d_pos0), _ptr(d_logit_scale), tau, active, _ptr(d_out), _ptr(d_logits),
                                  _stream(stream)))


def rs_route_scratch_bytes(n: int, vocab: int) -> int:
    return lib.rs_route_scratch_bytes(n, vocab)


def rs_route(d_logits, n: int, vocab: int, d_logit_scale, tau: float, active: int, d_out, d_scratch,
             stream=None) -> None:
    _check(lib.rs_route(_ptr(d_logits), n, vocab, _ptr(d_logit_scale), tau, active, _ptr(d_out), _ptr(d_scratch),
                        0 if d_scratch is None else d_scratch.numel() * d_scratch.element_size(), _stream(stream)))


def rs_route_static(d_logits, n: int, vocab: int, d_logit_scale, tau: float, active: int, d_out, stream=None) -> None:
    _check(lib.rs_route_static(_ptr(d_logits), n, vocab, _ptr(d_logit_scale), tau, active, _ptr(d_out), _stream(stream)))


class RouterPlus:
    """Marshalled rs_router_weights: keeps the device tensors and the pointer arrays alive.
    weights: object with w1, b1, w2, b2 (lists of six bf16 device tensors), ln_gain, ln_bias, w_head, b_head."""

    def __init__(self, weights, ln_eps: float = 1e-5):
        self.weights = weights
        self._arrs = {n: (C.c_void_p * 6)(*[t.data_ptr() for t in getattr(weights, n)]) for n in ("w1", "b1", "w2", "b2")}
        r, d = weights.w1[0].shape
        self.struct = _RsRouterWeights(d, r, ln_eps, *[C.cast(self._arrs[n], C.POINTER(C.c_void_p)) for n in ("w1", "b1", "w2", "b2")],
                                       weights.ln_gain.data_ptr(), weights.ln_bias.data_ptr(), weights.w_head.data_ptr(),
                                       weights.b_head.data_ptr())


def rs_route_plus(handle: Optional[int], d_hidden, n_seqs: int, router: RouterPlus, active: int, d_out,
                  d_router_logits=None, stream=None) -> None:
    """d_out: tensor or raw address of the records to update."""
    out = d_out if isinstance(d_out, int) else _ptr(d_out)
    _check(lib.rs_route_plus(handle, _ptr(d_hidden), n_seqs, C.byref(router.struct), active, out,
                             _ptr(d_router_logits), _stream(stream)))


STITCH_RUNNING, STITCH_DONE, STITCH_TRACE_FULL, STITCH_FLAGGED, STITCH_ABORTED = range(5)
STITCH_RECORD_INTS = 10     # rs_stitch_record: model, pos0, n_rows, reserved, then the 6 words of rs_route_out
STITCH_RESULT_INTS = 8      # rs_stitch_result: status, n_tokens, n_records, seen_slm, seen_llm, active, n_target, reserved


def rs_stitch_generate(slm: int, llm: int, seq_slot: int, d_seq, n_prompt: int, n_new: int, seen_slm: int,
                       seen_llm: int, d_logit_scale, tau: float, eos: int, d_trace, max_records: int, d_result,
                       stream=None) -> None:
    """d_seq: int32 tensor [n_prompt + n_new]; d_trace: int32 tensor [max_records, 10]; d_result: int32 tensor [8]."""
    _check(lib.rs_stitch_generate(slm, llm, seq_slot, _ptr(d_seq), n_prompt, n_new, seen_slm, seen_llm,
                                  _ptr(d_logit_scale), tau, eos, _ptr(d_trace), max_records, _ptr(d_result),
                                  _stream(stream)))


def rs_set_sampling(handle: int, enabled: bool, key: int = 0) -> None:
    _check(lib.rs_set_sampling(handle, int(bool(enabled)), key & 0xFFFFFFFFFFFFFFFF))


PHASE_QKV, PHASE_OPROJ, PHASE_GATEUP, PHASE_DOWN, PHASE_LMHEAD, PHASE_ATTN = range(6)


def rs_set_spin_limit(handle: int, polls: int) -> None:
    _check(lib.rs_set_spin_limit(handle, polls))


def rs_set_phase_timer(handle: int, phase: int, layer: int = 0, start_event: int = 0, stop_event: int = 0) -> None:
    """start_event / stop_event: raw hipEvent_t handles (integers); phase < 0 disarms."""
    _check(lib.rs_set_phase_timer(handle, phase, layer, start_event or None, stop_event or None))


# ------------------------------------------------------------------ records
@dataclass
class RouteOut:
    token: int
    flags: int
    h_nats: float
    h_norm: float
    max_logit: float
    log_z: float

    @property
    def hi(self) -> bool:
        return bool(self.flags & FLAG_HI)

    @property
    def accept(self) -> bool:
        return bool(self.flags & FLAG_ACCEPT)


def new_route_out(n: int, device="cuda") -> torch.Tensor:
    """Device buffer for n rs_route_out records (6 x 32-bit words each)."""
    return torch.zeros(n, 6, dtype=torch.int32, device=device)


def read_route_out(buf: torch.Tensor) -> List[RouteOut]:
    host = buf.cpu()
    ints, floats = host, host.view(torch.float32)
    return [RouteOut(int(ints[i, 0]), int(ints[i, 1]) & 0xFFFFFFFF, float(floats[i, 2]), float(floats[i, 3]),
                     float(floats[i, 4]), float(floats[i, 5])) for i in range(host.shape[0])]


# ------------------------------------------------------------------ buffer holder
def make_config(shape, max_ctx: int, max_seqs: int = 1, max_rows: int = 64) -> RsConfig:
    return RsConfig(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                    shape.vocab, int(shape.tied_lm_head), max_ctx, max_seqs, max_rows, shape.rms_eps, shape.rope_theta)


class Model:
    """Owns the device buffers a C handle borrows (weights, KV caches, workspace) and small
    staging tensors for the per-call arrays."""

    def __init__(self, weights, max_ctx: int, max_seqs: int = 1, max_rows: int = 64, device="cuda"):
        self.shape = weights.shape
        self.weights = weights                      # bf16 tensors already on `device`
        max_ctx = (max_ctx + 7) // 8 * 8            # the library wants a multiple of 8
        self.cfg = make_config(self.shape, max_ctx, max_seqs, max_rows)
        kvb, wsb = rs_kv_bytes(self.cfg), rs_workspace_bytes(self.cfg)
        if kvb == 0 or wsb == 0:
            raise RsError(-1, rs_last_error())
        self.kv_k = torch.zeros(kvb // 2, dtype=torch.bfloat16, device=device)
        self.kv_v = torch.zeros(kvb // 2, dtype=torch.bfloat16, device=device)
        self.workspace = torch.zeros(wsb, dtype=torch.uint8, device=device)
        self.device = device
        self.handle = rs_create_model(self.cfg, weights, self.kv_k, self.kv_v, self.workspace)

    def close(self) -> None:
        if self.handle:
            rs_destroy_model(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def kv_view(self, which: str) -> torch.Tensor:
        """[layer, slot, kv_head, position, head_dim] view of a cache (V is stored transposed)."""
        c = self.cfg
        if which == "k":
            return self.kv_k.view(c.n_layers, c.max_seqs, c.n_kv_heads, c.max_ctx, c.head_dim)
        return self.kv_v.view(c.n_layers, c.max_seqs, c.n_kv_heads, c.head_dim, c.max_ctx).transpose(3, 4)

    def _i32(self, values: Sequence[int]) -> torch.Tensor:
        return torch.tensor(list(values), dtype=torch.int32, device=self.device)

    def decode_step(self, tokens: Sequence[int], positions: Sequence[int], tau: float, active: int,
                    scales: Optional[Sequence[float]] = None, slots: Optional[Sequence[int]] = None,
                    want_logits: bool = False):
        n = len(tokens)
        slots = list(range(n)) if slots is None else slots
        out = new_route_out(n, self.device)
        logits = torch.empty(n, self.cfg.vocab, dtype=torch.float32, device=self.device) if want_logits else None
        sc = None if scales is None else torch.tensor(list(scales), dtype=torch.float32, device=self.device)
        rs_decode_step(self.handle, n, self._i32(slots), self._i32(tokens), self._i32(positions), sc, tau, active,
                       out, logits)
        return (read_route_out(out), logits) if want_logits else read_route_out(out)

    def catchup_prefill(self, spans: Sequence[Sequence[int]], pos0: Sequence[int], tau: float, active: int,
                        scales: Optional[Sequence[float]] = None, slots: Optional[Sequence[int]] = None,
                        want_logits: bool = False):
        n = len(spans)
        slots = list(range(n)) if slots is None else slots
        off = [0]
        flat: List[int] = []
        for s in spans:
            flat.extend(s)
            off.append(len(flat))
        out = new_route_out(n, self.device)
        logits = torch.empty(n, self.cfg.vocab, dtype=torch.float32, device=self.device) if want_logits else None
        sc = None if scales is None else torch.tensor(list(scales), dtype=torch.float32, device=self.device)
        rs_catchup_prefill(self.handle, n, len(flat), self._i32(slots), self._i32(flat), self._i32(off),
                           self._i32(pos0), sc, tau, active, out, logits)
        return (read_route_out(out), logits) if want_logits else read_route_out(out)

    def forward_span(self, tokens: Sequence[int], pos0: int, tau: float, active: int, scale: float = 1.0,
                     slot: int = 0, want_logits: bool = False):
        """One sequence, any span length: chunks of max_rows through rs_catchup_prefill (a single
        token goes through rs_decode_step).  Returns the router record of the last chunk."""
        tokens = list(tokens)
        res = None
        mr = self.cfg.max_rows
        for s in range(0, len(tokens), mr):
            chunk = tokens[s:s + mr]
            if len(chunk) == 1:
                res = self.decode_step(chunk, [pos0 + s], tau, active, [scale], [slot], want_logits)
            else:
                res = self.catchup_prefill([chunk], [pos0 + s], tau, active, [scale], [slot], want_logits)
        return res
