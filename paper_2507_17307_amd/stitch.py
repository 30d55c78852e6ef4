"""Host driver of the stitched inference loop on top of the C ABI.

Algorithm 1 ("Inference procedure"): the active model processes the suffix of
prompt + output it has not seen (rs_catchup_prefill; rs_decode_step when that is
one token), the library returns the proposed token and the routing flags of
Eq. 2, and this loop applies them: a rejected small-model token is dropped and
the large model takes over at the same position; the large model hands back as
soon as its entropy is at or below tau.  The loop is position-explicit: the
number of tokens each model has cached is all the state there is, so the
"rollback" of a rejected step is simply not advancing it.

Per invocation the host does one library call, one stream synchronisation and
reads one 24-byte record.  Tokens and the record live in pinned host memory that
the GPU addresses directly; positions, scales and span offsets are pointers
into small device tables, so no per-step buffers are created or copied.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B

SLM, LLM = B.RS_SLM, B.RS_LLM


@dataclass
class Invocation:
    model: int
    pos0: int
    n_rows: int
    token: int
    h_norm: float
    flags: int

    @property
    def accept(self) -> bool:
        return bool(self.flags & B.FLAG_ACCEPT)


@dataclass
class StitchRun:
    output: List[int] = field(default_factory=list)
    trace: List[Invocation] = field(default_factory=list)


class StitchedPair:
    def __init__(self, slm: B.Model, llm: Optional[B.Model], max_ctx: int, scale_table: torch.Tensor):
        """scale_table: fp32 [max_ctx + 1]; entry p scales the logits that predict position p."""
        self.models = [slm, llm]
        self.max_ctx = max_ctx
        dev = slm.device
        self.max_rows = min(m.cfg.max_rows for m in self.models if m is not None)
        self.pos_table = torch.arange(max_ctx + 1, dtype=torch.int32, device=dev)
        self.slot0 = torch.zeros(1, dtype=torch.int32, device=dev)
        self.off_table = torch.tensor([[0, n] for n in range(self.max_rows + 1)], dtype=torch.int32, device=dev)
        self.scale = scale_table.to(device=dev, dtype=torch.float32).contiguous()
        assert self.scale.numel() >= max_ctx + 1
        self.seq = torch.zeros(max_ctx + 1, dtype=torch.int32).pin_memory()
        self.seq_np = self.seq.numpy()
        self.out = torch.zeros(6, dtype=torch.int32).pin_memory()
        self.out_i = self.out.numpy()
        self.out_f = self.out_i.view(np.float32)
        self._p_pos, self._p_off = self.pos_table.data_ptr(), self.off_table.data_ptr()
        self._p_seq, self._p_scale = self.seq.data_ptr(), self.scale.data_ptr()
        self._p_out, self._p_slot = self.out.data_ptr(), self.slot0.data_ptr()
        self.on_invocation: Optional[Callable[[int, int, int], None]] = None   # (model, pos0, n_rows) after sync

    def _forward(self, model: int, pos0: int, end: int, tau: float, stream_handle: int) -> None:
        """Feed sequence positions pos0 .. end-1 to `model`; the record of the last chunk lands in self.out."""
        h = self.models[model].handle
        lib = B.lib
        p = pos0
        while p < end:
            n = min(self.max_rows, end - p)
            # only the chunk that reaches `end` predicts position `end`
            scale_ptr = self._p_scale + 4 * end
            if n == 1:
                rc = lib.rs_decode_step(h, 1, self._p_slot, self._p_seq + 4 * p, self._p_pos + 4 * p, scale_ptr,
                                        tau, model, self._p_out, None, stream_handle)
            else:
                rc = lib.rs_catchup_prefill(h, 1, n, self._p_slot, self._p_seq + 4 * p, self._p_off + 8 * n,
                                            self._p_pos + 4 * p, scale_ptr, tau, model, self._p_out, None,
                                            stream_handle)
            if rc != 0:
                raise B.RsError(rc, B.rs_last_error())
            p += n

    def generate(self, prompt: Sequence[int], tau: float, n_tokens: int, single_model: Optional[int] = None,
                 keep_trace: bool = True, stop_after: Optional[Callable[[int], bool]] = None) -> StitchRun:
        """Algorithm 1 until n_tokens tokens are accepted.  single_model = SLM or LLM runs that model
        alone (every token accepted) while still reporting its entropies."""
        stream = torch.cuda.current_stream()
        sh = stream.cuda_stream
        n0 = len(prompt)
        if n0 + n_tokens > self.max_ctx + 1:
            raise ValueError("prompt + tokens exceed max_ctx")
        self.seq_np[:n0] = np.asarray(prompt, dtype=np.int32)
        length = n0
        n_kv = [0, 0]
        active = SLM if single_model is None else single_model
        run = StitchRun()
        sync = stream.synchronize
        while len(run.output) < n_tokens:
            pos0 = n_kv[active]
            self._forward(active, pos0, length, tau, sh)
            sync()
            n_kv[active] = length
            token, flags = int(self.out_i[0]), int(self.out_i[1]) & 0xFFFFFFFF
            if self.on_invocation is not None:
                self.on_invocation(active, pos0, length - pos0)
            if flags & (B.FLAG_BADARG | B.FLAG_NONFINITE):
                raise RuntimeError(f"router flagged the step: flags={flags} model={active} pos0={pos0}")
            if keep_trace:
                run.trace.append(Invocation(active, pos0, length - pos0, token, float(self.out_f[3]), flags))
            if single_model is None:
                if active == SLM and (flags & B.FLAG_HI):
                    active = LLM
                    continue
                if active == LLM and not (flags & B.FLAG_HI):
                    active = SLM
            self.seq_np[length] = token
            length += 1
            run.output.append(token)
            if stop_after is not None and stop_after(len(run.output)):
                break
        return run
