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
reads one 24-byte record.  The span tokens, its first position, the logit scale
and the record live at FIXED addresses in pinned host memory that the GPU reads
and writes directly: nothing is allocated or copied per step, and because the
call arguments repeat, the library replays a cached launch graph per (model,
span length) instead of launching ~170 kernels one by one.
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
    status: int = B.STITCH_DONE          # generate_on_device: how the kernel's loop ended
    loop_ms: float = 0.0                 # generate_on_device: GPU time of the call (events on its stream)


class StitchedPair:
    def __init__(self, slm: B.Model, llm: Optional[B.Model], max_ctx: int, scale_table: torch.Tensor):
        """scale_table: fp32 [max_ctx + 1]; entry p scales the logits that predict position p."""
        self.models = [slm, llm]
        self.max_ctx = max_ctx
        dev = slm.device
        self.max_rows = min(m.cfg.max_rows for m in self.models if m is not None)
        self.stream = torch.cuda.Stream(device=dev)          # a capturable (non-default) stream
        self.slot0 = torch.zeros(1, dtype=torch.int32, device=dev)
        self.off_table = torch.tensor([[0, n] for n in range(self.max_rows + 1)], dtype=torch.int32, device=dev)
        self.scale_np = scale_table.to(dtype=torch.float32).cpu().numpy()
        assert self.scale_np.size >= max_ctx + 1
        self.seq_np = np.zeros(max_ctx + 1, dtype=np.int32)  # prompt + accepted tokens (host)
        # fixed-address staging in pinned memory: [0:max_rows] span tokens, then pos0, then scale (as bits), then the record
        self.stage = torch.zeros(self.max_rows + 2 + 6, dtype=torch.int32).pin_memory()
        self.stage_i = self.stage.numpy()
        self.stage_f = self.stage_i.view(np.float32)
        base = self.stage.data_ptr()
        self._p_tok = base
        self._p_pos = base + 4 * self.max_rows
        self._p_scale = base + 4 * (self.max_rows + 1)
        self._p_out = base + 4 * (self.max_rows + 2)
        self._o = self.max_rows + 2                         # index of the record inside the staging array
        self._p_off, self._p_slot = self.off_table.data_ptr(), self.slot0.data_ptr()
        torch.cuda.synchronize()
        self.on_invocation: Optional[Callable[[int, int, int], None]] = None   # (model, pos0, n_rows) after sync

    def _forward(self, model: int, pos0: int, end: int, tau: float) -> None:
        """Feed sequence positions pos0 .. end-1 to `model`; the record of the last chunk lands in the staging array."""
        h = self.models[model].handle
        lib = B.lib
        sh = self.stream.cuda_stream
        p = pos0
        while p < end:
            n = min(self.max_rows, end - p)
            if p > pos0:
                self.stream.synchronize()                    # the previous chunk still reads the staging buffers
            self.stage_i[:n] = self.seq_np[p:p + n]
            self.stage_i[self.max_rows] = p
            self.stage_f[self.max_rows + 1] = self.scale_np[end]      # only the chunk that reaches `end` predicts position `end`
            if n == 1:
                rc = lib.rs_decode_step(h, 1, self._p_slot, self._p_tok, self._p_pos, self._p_scale,
                                        tau, model, self._p_out, None, sh)
            else:
                rc = lib.rs_catchup_prefill(h, 1, n, self._p_slot, self._p_tok, self._p_off + 8 * n,
                                            self._p_pos, self._p_scale, tau, model, self._p_out, None, sh)
            if rc != 0:
                raise B.RsError(rc, B.rs_last_error())
            p += n

    def prefill_prompt(self, model: int, prompt: Sequence[int], tau: float) -> None:
        """Feed the whole prompt to `model` ahead of generate(..., llm_prefilled=True): the prefill a model does
        when it first takes part (Section "KV Cache management"), moved out of the loop.  The K/V rows are the
        ones the loop would write; the record of this call is not used."""
        n0 = len(prompt)
        self.seq_np[:n0] = np.asarray(prompt, dtype=np.int32)
        self._forward(model, 0, n0, tau)
        self.stream.synchronize()

    def generate_random(self, prompt: Sequence[int], p_slm: float, u_table: Sequence[float], n_tokens: int) -> StitchRun:
        """Random-routing baseline (Section "Experiments", "Latency-accuracy trade-off"): the token at absolute
        position t is produced by the small model iff u_table[t] < p_slm, by the large model otherwise; the
        assigned model catches up with what it has not seen, its token is always kept.  The assignment uses no
        output of the step, so it is made here before the call; tau is set so that no record is flagged HI."""
        n0 = len(prompt)
        if n0 + n_tokens > self.max_ctx + 1:
            raise ValueError("prompt + tokens exceed max_ctx")
        self.seq_np[:n0] = np.asarray(prompt, dtype=np.int32)
        length, n_kv, run, o = n0, [0, 0], StitchRun(), self._o
        while len(run.output) < n_tokens:
            model = SLM if float(u_table[length]) < p_slm else LLM
            pos0 = n_kv[model]
            self._forward(model, pos0, length, 2.0)
            self.stream.synchronize()
            n_kv[model] = length
            token, flags = int(self.stage_i[o]), int(self.stage_i[o + 1]) & 0xFFFFFFFF
            if flags & (B.FLAG_BADARG | B.FLAG_NONFINITE | B.FLAG_ABORTED):
                raise RuntimeError(f"router flagged the step: flags={flags} model={model} pos0={pos0}")
            run.trace.append(Invocation(model, pos0, length - pos0, token, float(self.stage_f[o + 3]), flags))
            self.seq_np[length] = token
            length += 1
            run.output.append(token)
        return run

    def generate(self, prompt: Sequence[int], tau: float, n_tokens: int, single_model: Optional[int] = None,
                 keep_trace: bool = True, stop_after: Optional[Callable[[int], bool]] = None,
                 llm_prefilled: bool = False, router_plus: Optional[B.RouterPlus] = None,
                 sampling_key: Optional[int] = None, slm_prefilled: bool = False) -> StitchRun:
        """Algorithm 1 until n_tokens tokens are accepted.  single_model = SLM or LLM runs that model
        alone (every token accepted) while still reporting its entropies.  llm_prefilled: the large model's
        cache already holds the prompt (prefill_prompt), so its first participation only catches up with the
        tokens accepted since (slm_prefilled: the same for the small model).  router_plus: the R-Stitch+ branch of Algorithm 1: after every small-model call the
        learned router (rs_route_plus, enqueued behind the call) may turn a hand-over into "keep the token and stay".
        sampling_key: tokens are sampled from each step's distribution (rs_set_sampling with this 64-bit key on both
        models) instead of taken greedily."""
        for mdl in self.models:
            if mdl is not None:
                B.rs_set_sampling(mdl.handle, sampling_key is not None, sampling_key or 0)
        n0 = len(prompt)
        if n0 + n_tokens > self.max_ctx + 1:
            raise ValueError("prompt + tokens exceed max_ctx")
        self.seq_np[:n0] = np.asarray(prompt, dtype=np.int32)
        length = n0
        # a prefilled large model still has to produce a distribution the first time it is asked, which may be before
        # any token was accepted: it re-runs the last prompt token then (the same K/V row is written again)
        n_kv = [n0 - 1 if slm_prefilled else 0, n0 - 1 if llm_prefilled else 0]
        active = SLM if single_model is None else single_model
        run = StitchRun()
        sync = self.stream.synchronize
        o = self._o
        while len(run.output) < n_tokens:
            pos0 = n_kv[active]
            self._forward(active, pos0, length, tau)
            if router_plus is not None and active == SLM:
                B.rs_route_plus(self.models[SLM].handle, None, 1, router_plus, SLM, self._p_out, None, self.stream)
            sync()
            n_kv[active] = length
            token, flags = int(self.stage_i[o]), int(self.stage_i[o + 1]) & 0xFFFFFFFF
            if self.on_invocation is not None:
                self.on_invocation(active, pos0, length - pos0)
            if flags & (B.FLAG_BADARG | B.FLAG_NONFINITE | B.FLAG_ABORTED):
                raise RuntimeError(f"router flagged the step: flags={flags} model={active} pos0={pos0}")
            if keep_trace:
                run.trace.append(Invocation(active, pos0, length - pos0, token, float(self.stage_f[o + 3]), flags))
            if single_model is None:
                if not (flags & B.FLAG_ACCEPT):
                    active = LLM                             # small-model token discarded; the large model redoes this position
                    continue
                active = LLM if (flags & B.FLAG_NEXT_LLM) else SLM
            self.seq_np[length] = token
            length += 1
            run.output.append(token)
            if stop_after is not None and stop_after(len(run.output)):
                break
        return run


    def generate_on_device(self, prompt: Sequence[int], tau: float, n_tokens: int, prompt_prefilled: bool = False,
                           eos: int = -1, max_records: Optional[int] = None) -> StitchRun:
        """Algorithm 1 with the loop on the device (rs_stitch_generate): one kernel runs every invocation and
        applies the routing flags itself; the host reads the sequence, the trace and the result once, at the end.
        prompt_prefilled: both models first take all but the last prompt token through rs_catchup_prefill (the
        matrix-core path), so the kernel starts each of them at the last prompt token.  The run's `status` is one
        of binding.STITCH_*."""
        n0 = len(prompt)
        if n0 + n_tokens > self.max_ctx + 1:
            raise ValueError("prompt + tokens exceed max_ctx")
        dev = self.models[SLM].device
        seen = 0
        if prompt_prefilled and n0 > 1:
            self.seq_np[:n0] = np.asarray(prompt, dtype=np.int32)
            for model in (SLM, LLM):
                self._forward(model, 0, n0 - 1, tau)
                self.stream.synchronize()
            seen = n0 - 1
        cap = 2 * n_tokens if max_records is None else max_records
        d_seq = torch.zeros(n0 + n_tokens, dtype=torch.int32, device=dev)
        d_seq[:n0] = torch.as_tensor(np.asarray(prompt, dtype=np.int32), device=dev)
        d_scale = torch.as_tensor(self.scale_np[:n0 + n_tokens], device=dev)
        d_trace = torch.zeros(cap, B.STITCH_RECORD_INTS, dtype=torch.int32, device=dev)
        d_result = torch.zeros(B.STITCH_RESULT_INTS, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(self.stream)
        B.rs_stitch_generate(self.models[SLM].handle, self.models[LLM].handle, 0, d_seq, n0, n_tokens, seen, seen,
                             d_scale, tau, eos, d_trace, cap, d_result, self.stream)
        e1.record(self.stream)
        self.stream.synchronize()
        result = d_result.cpu().numpy()
        trace_i = d_trace.cpu().numpy()
        trace_f = trace_i.view(np.float32)
        run = StitchRun()
        run.status = int(result[0])
        run.loop_ms = e0.elapsed_time(e1)
        run.output = d_seq.cpu().numpy()[n0:int(result[1])].tolist()
        for r in range(int(result[2])):
            run.trace.append(Invocation(int(trace_i[r, 0]), int(trace_i[r, 1]), int(trace_i[r, 2]), int(trace_i[r, 4]),
                                        float(trace_f[r, 7]), int(trace_i[r, 5]) & 0xFFFFFFFF))
        return run


class StitchedBatch:
    """Algorithm 1 for several independent sequences that share the two models, with per-sequence
    routing (the batch-8 setting of the paper's batch-size study).

    Every sequence keeps its own state (tokens, cached length per model, active model) and its own
    KV slot in both models.  A round advances, with as few library calls as possible, first every
    sequence whose active model is the small one, then every sequence on the large one: the unseen
    suffixes of a group are packed back to back into one ragged rs_catchup_prefill call (or one
    rs_decode_step when every suffix is a single token), chunked when they exceed max_rows.  A
    sequence the small model gives up on in the first half of a round is picked up by the large
    model in the second half.  Because sequences never interact, each one's outcome equals the
    single-sequence loop's.
    """

    def __init__(self, slm: B.Model, llm: B.Model, max_ctx: int, scale_tables: Sequence[torch.Tensor]):
        self.models = [slm, llm]
        self.max_ctx = max_ctx
        self.n_slots = min(slm.cfg.max_seqs, llm.cfg.max_seqs)
        if len(scale_tables) > self.n_slots:
            raise ValueError("more sequences than KV slots")
        self.max_rows = min(slm.cfg.max_rows, llm.cfg.max_rows)
        self.stream = torch.cuda.Stream(device=slm.device)
        self.scale_np = [t.to(dtype=torch.float32).cpu().numpy() for t in scale_tables]
        ns, mr = self.n_slots, self.max_rows
        # fixed-address pinned staging: slots[ns] tokens[mr] offsets[ns+1] pos0[ns] scales[ns] records[6*ns]
        self.stage = torch.zeros(ns + mr + (ns + 1) + ns + ns + 6 * ns, dtype=torch.int32).pin_memory()
        self.stage_i = self.stage.numpy()
        self.stage_f = self.stage_i.view(np.float32)
        self._o_slot, self._o_tok = 0, ns
        self._o_off = ns + mr
        self._o_pos = self._o_off + ns + 1
        self._o_scale = self._o_pos + ns
        self._o_rec = self._o_scale + ns
        self._base = self.stage.data_ptr()
        self.calls = 0
        self.call_log: List[tuple] = []                            # (model, context length per sequence, rows) of every call
        self.on_call: Optional[Callable[[int], None]] = None     # (accepted tokens so far, all sequences) after each call
        torch.cuda.synchronize()

    def _ptr(self, index: int) -> int:
        return self._base + 4 * index

    def _call(self, model: int, entries, tau: float, lengths) -> None:
        self.raw_call(model, entries, tau, lengths)
        self.stream.synchronize()
        self.calls += 1
        self.call_log.append((model, [p0 + n for _, p0, n in entries], sum(n for _, _, n in entries)))

    def prefill_prompts(self, model: int, prompts: Sequence[Sequence[int]], tau: float) -> None:
        """Feed every prompt to `model` ahead of generate(..., llm_prefilled=True) (see StitchedPair.prefill_prompt)."""
        self.seqs = [np.zeros(self.max_ctx + 1, dtype=np.int32) for _ in prompts]
        lengths = [len(p) for p in prompts]
        for b, p in enumerate(prompts):
            self.seqs[b][:len(p)] = np.asarray(p, dtype=np.int32)
            for c0 in range(0, len(p), self.max_rows):
                self.raw_call(model, [(b, c0, min(self.max_rows, len(p) - c0))], tau, lengths)
                self.stream.synchronize()

    def raw_call(self, model: int, entries, tau: float, lengths) -> None:
        """One library call, enqueued only.
        entries: (sequence, first position, row count), at most n_slots of them and max_rows rows in all."""
        si, sf = self.stage_i, self.stage_f
        row = 0
        for i, (b, p0, n) in enumerate(entries):
            si[self._o_slot + i] = b
            si[self._o_tok + row:self._o_tok + row + n] = self.seqs[b][p0:p0 + n]
            si[self._o_off + i] = row
            si[self._o_pos + i] = p0
            sf[self._o_scale + i] = self.scale_np[b][lengths[b]]
            row += n
        si[self._o_off + len(entries)] = row
        h, lib, sh = self.models[model].handle, B.lib, self.stream.cuda_stream
        if row == len(entries):
            rc = lib.rs_decode_step(h, len(entries), self._ptr(self._o_slot), self._ptr(self._o_tok), self._ptr(self._o_pos),
                                    self._ptr(self._o_scale), tau, model, self._ptr(self._o_rec), None, sh)
        else:
            rc = lib.rs_catchup_prefill(h, len(entries), row, self._ptr(self._o_slot), self._ptr(self._o_tok),
                                        self._ptr(self._o_off), self._ptr(self._o_pos), self._ptr(self._o_scale),
                                        tau, model, self._ptr(self._o_rec), None, sh)
        if rc != 0:
            raise B.RsError(rc, B.rs_last_error())

    def generate(self, prompts: Sequence[Sequence[int]], tau: float, n_tokens: int,
                 single_model: Optional[int] = None, llm_prefilled: bool = False) -> List[StitchRun]:
        nb = len(prompts)
        if nb > len(self.scale_np):
            raise ValueError("more prompts than scale tables")
        self.seqs = [np.zeros(self.max_ctx + 1, dtype=np.int32) for _ in range(nb)]
        lengths = []
        for b, p in enumerate(prompts):
            if len(p) + n_tokens > self.max_ctx + 1:
                raise ValueError("prompt + tokens exceed max_ctx")
            self.seqs[b][:len(p)] = np.asarray(p, dtype=np.int32)
            lengths.append(len(p))
        # (a prefilled large model re-runs the last prompt token at its first participation, see StitchedPair.generate)
        n_kv = [[0] * nb, [n - 1 for n in lengths] if llm_prefilled else [0] * nb]
        active = [SLM if single_model is None else single_model] * nb
        runs = [StitchRun() for _ in range(nb)]
        live = set(range(nb))
        while live:
            for model in (SLM, LLM):
                group = [b for b in sorted(live) if active[b] == model]
                fed = {b: n_kv[model][b] for b in group}
                while group:
                    entries, rows = [], 0
                    for b in group:
                        if rows >= self.max_rows or len(entries) >= self.n_slots:
                            break
                        n = min(lengths[b] - fed[b], self.max_rows - rows)
                        entries.append((b, fed[b], n))
                        rows += n
                    self._call(model, entries, tau, lengths)
                    for i, (b, p0, n) in enumerate(entries):
                        fed[b] += n
                        if fed[b] < lengths[b]:
                            continue                       # more of this suffix to feed: the record is not the final one
                        o = self._o_rec + 6 * i
                        token, flags = int(self.stage_i[o]), int(self.stage_i[o + 1]) & 0xFFFFFFFF
                        if flags & (B.FLAG_BADARG | B.FLAG_NONFINITE | B.FLAG_ABORTED):
                            raise RuntimeError(f"router flagged the step: flags={flags} model={model} sequence={b}")
                        runs[b].trace.append(Invocation(model, n_kv[model][b], lengths[b] - n_kv[model][b], token,
                                                        float(self.stage_f[o + 3]), flags))
                        n_kv[model][b] = lengths[b]
                        group.remove(b)
                        if single_model is None:
                            if not (flags & B.FLAG_ACCEPT):
                                active[b] = LLM            # rejected: the large model redoes this position
                                continue
                            active[b] = LLM if (flags & B.FLAG_NEXT_LLM) else SLM
                        self.seqs[b][lengths[b]] = token
                        lengths[b] += 1
                        runs[b].output.append(token)
                        if len(runs[b].output) >= n_tokens:
                            live.discard(b)
                    if self.on_call is not None:
                        self.on_call(sum(len(r.output) for r in runs))
        return runs
