#!/usr/bin/env python3
"""Headline benchmark: stitched decode tokens/s at batch 1 on the 1.5B + 7B shapes
(workload cfg3_s15_m7), with the fraction of the per-token HBM roofline.

A "step" is one ACCEPTED token of the live stitched run (Algorithm 1 driven from
the host through the C ABI): it costs one or more model invocations - small-model
decode steps (accepted or rejected), large-model catch-up prefills and decode
steps.  All inputs (weights, prompt, logit-scale schedule) are seeded synthetic
data resident in HBM before the timed region starts, and BOTH models have
processed the prompt before it starts (the large model's first participation,
a prefill of the whole prompt, is set-up and is reported as such), so a timed
window of any length measures steady-state stitched decoding.

Prints ONE JSON line.  Extra objects:
  roofline      live HIP-event timing of the dominant kernel (the large model's
                single-row gate/up projection, picked by name) against the
                8 TB/s HBM peak, plus the whole-step fraction of each model
  per_model     decode ms/token of each model alone and its roofline fraction
  stitched      invocation mix of the timed region and its roofline fraction
  device_loop   Algorithm 1 as one kernel (rs_stitch_generate) on a few tokens beside the host-driven loop
  latency_fit   Eq. 5-6 of the paper re-fitted to this machine's timings
  cpu_baseline  the CPU oracle timed on this machine's cores on a bounded sample
"""
from __future__ import annotations

import argparse
import ctypes as C
import dataclasses
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12   # bytes/s, MI355X published
DTYPE = "bf16 weights, f32 activations and accumulation"


# (timed accepted tokens, warm-up tokens) of a run without --steps / --warmup
DEFAULT_STEPS = {"cfg2_s15_decode": (448, 64), "cfg3_s15_m7": (4032, 64), "cfg4_s15_m14": (256, 32)}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class HipEvents:
    """Raw hipEvent_t pairs through the HIP runtime (torch's events only see torch's stream API)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventQuery.argtypes = [C.c_void_p]

    def create(self) -> int:
        ev = C.c_void_p()
        assert self.hip.hipEventCreate(C.byref(ev)) == 0
        return ev.value

    def record(self, ev: int, stream: int) -> None:
        assert self.hip.hipEventRecord(ev, stream) == 0

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), a, b)
        return ms.value if rc == 0 else float("nan")


def event_pair_overhead_ms(ev, stream, e0, e1):
    """What two event records add to a bracket around ONE kernel: the same bracket around one launch of a
    streaming kernel of about the same length (an in-place add over 2^24 floats, ~20 us), minus that kernel's
    duration when 50 of them run back to back inside one bracket.  Median over 30 brackets.  An unprofiled run
    gives 2.7-3.2 us; with a profiler attached every dispatch costs more and the figure no longer describes the
    bracket, so a value outside 0..5 us is dropped (returns 0.0, False) and raw brackets are reported."""
    import torch
    cal_x = torch.zeros(1 << 24, device="cuda")
    cal_s = torch.zeros(1 << 16, device="cuda")
    sh = stream.cuda_stream
    with torch.cuda.stream(stream):
        for _ in range(5):
            cal_x.add_(1.0)
        singles = []
        for _ in range(30):
            for _ in range(4):
                cal_s.add_(1.0)
            ev.record(e0, sh)
            cal_x.add_(1.0)
            ev.record(e1, sh)
            for _ in range(2):
                cal_s.add_(1.0)
            stream.synchronize()
            singles.append(ev.elapsed_ms(e0, e1))
        ev.record(e0, sh)
        for _ in range(50):
            cal_x.add_(1.0)
        ev.record(e1, sh)
        stream.synchronize()
        over = sorted(singles)[len(singles) // 2] - ev.elapsed_ms(e0, e1) / 50
    del cal_x, cal_s
    if not 0.0 <= over <= 5e-3:
        log(f"[bench] event-pair calibration gave {over * 1e3:.2f} us: not applied")
        return 0.0, False
    return over, True


def time_phase(ev, P, model, phase, layer, run_once, sync, n, e0, e1):
    """Mean time between an event pair that the library places around ONE kernel (phase, layer) of every call
    `run_once(i)` makes on `model` (plain launches while the timer is armed)."""
    P.rs_set_phase_timer(model.handle, phase, layer, e0, e1)
    tot = 0.0
    try:
        for i in range(n + 2):
            run_once(i)
            sync()
            if i >= 2:
                tot += ev.elapsed_ms(e0, e1)
    finally:
        P.rs_set_phase_timer(model.handle, -1)
    return tot / n


def measured_traffic(P, shape_name, key):
    """HBM bytes per launch of a kernel from the hardware-counter runs stored with the package
    (FETCH_SIZE + WRITE_SIZE of the counter-run driver, scaled by a copy kernel of known size), or None."""
    try:
        with open(os.path.join(os.path.dirname(os.path.abspath(P.__file__)), "measured_traffic.json")) as f:
            rec = json.load(f).get(shape_name, {}).get(key)
        return rec["fetch_bytes"] + rec["write_bytes"] if rec else None
    except (OSError, KeyError, ValueError):
        return None


def gateup_roofline(ev, P, model, shape, run_once, sync, rows, overhead_ms, overhead_ok, e0, e1, n=24):
    """The `roofline` object: the gate/up projection of `model` (the largest kernel of a step: over half of a
    layer's bytes) in a call of `rows` token rows, timed live with an event pair around that kernel."""
    bracket_ms = time_phase(ev, P, model, P.binding.PHASE_GATEUP, shape.n_layers // 2, run_once, sync, n, e0, e1)
    avg_s = (bracket_ms - overhead_ms) * 1e-3
    nbytes = 2 * shape.d_ffn * shape.d_model * 2
    fma = rows <= 2 or (rows <= 4 and shape.d_model <= 2048)         # the library's own rule for the FMA kernels
    name = (f"k_gemv<GATEUP> ({shape.name}, {rows} token row{'s' if rows > 1 else ''})" if fma
            else f"k_gemm_rows<GATEUP> ({shape.name}, {rows} token rows)")
    return {"bound": "hbm", "kernel": name, "launches": n, "avg_us": round(avg_s * 1e6, 2),
            "avg_us_between_events": round(bracket_ms * 1e3, 2),
            "event_pair_overhead_us": round(overhead_ms * 1e3, 2) if overhead_ok else None,
            "achieved": round(nbytes / avg_s / 1e9, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
            "frac": round(nbytes / avg_s / HBM_PEAK, 4),
            "traffic": measured_traffic(P, shape.name, "gateup_rows1") if rows == 1 else None,
            "bytes_per_launch": nbytes,
            "measured": "plain launches of the model's calls with one event pair around this kernel per call; avg_us = "
                        "time between the events minus what the event records add to such a bracket (calibrated in this run)"}


def oracle_sample(W, odec, wts, ctx, rows_list, k_layers=4, seed=77):
    """Seconds per oracle invocation of the FULL model, for each row count in rows_list, at context `ctx`.

    Bounded sample: the oracle (as it stands, fp64) runs on the first k_layers layers and on zero layers (embedding
    + final norm + LM head only); a full invocation is the zero-layer time plus n_layers / k_layers times the
    difference.  The K/V cache of the sample is filled with seeded noise up to `ctx` (the time does not depend on
    the values)."""
    import torch
    from workloads.recipes import ModelWeights
    shape = wts.shape
    k = min(k_layers, shape.n_layers)
    emb = wts.embed.to("cpu")
    lm = emb if shape.tied_lm_head else wts.lm_head.to("cpu")
    fn = wts.final_norm.to("cpu")
    layers = [type(l)(*(getattr(l, f).to("cpu") for f in ("attn_norm", "w_qkv", "w_o", "mlp_norm", "w_gate_up", "w_down")))
              for l in wts.layers[:k]]
    out = {}
    for n_l in (0, k):
        sub_shape = dataclasses.replace(shape, n_layers=n_l)
        sub = ModelWeights(sub_shape, emb, lm, fn, layers[:n_l])
        om = odec.OracleModel(sub, max_ctx=ctx + max(rows_list) + 1, keep_fp64_weights=False)
        if n_l:
            noise = W.rng.normal(seed, 5, 0, n_l * shape.n_kv_heads * ctx * shape.head_dim).view(n_l, shape.n_kv_heads, ctx, shape.head_dim)
            om.k_cache[:, 0, :, :ctx] = noise
            om.v_cache[:, 0, :, :ctx] = noise
        om.forward([1], ctx)                      # untimed: first touch of the caches and of the BLAS threads
        for rows in rows_list:
            best = float("inf")
            for _ in range(2):                    # the better of two: the layer share is scaled up, and with it any hiccup
                t0 = time.perf_counter()
                om.forward(list(range(1, rows + 1)), ctx)
                best = min(best, time.perf_counter() - t0)
            out[(n_l, rows)] = best
        del om
    return {rows: out[(0, rows)] + (out[(k, rows)] - out[(0, rows)]) * shape.n_layers / k for rows in rows_list}, k


def cpu_baseline(W, models, inv, steps, ctx):
    """`cpu_baseline` object.  models: {tag: (model id, weights)}; inv: (model id, pos0, rows) of the timed region."""
    import torch
    from oracle import decoder as odec
    torch.set_grad_enabled(False)
    t_inv, ks = {}, {}
    for tag, (mid, wts) in models.items():
        t0 = time.time()
        t_inv[mid], ks[tag] = oracle_sample(W, odec, wts, ctx, [1, 4])
        log(f"[bench] oracle {tag}: 1-row invocation {t_inv[mid][1]:.2f}s, 4-row {t_inv[mid][4]:.2f}s at context {ctx} "
            f"(extrapolated from {ks[tag]} layers; sample took {time.time() - t0:.1f}s)")
    total = 0.0
    for mid, _, rows in inv:
        t1, t4 = t_inv[mid][1], t_inv[mid][4]
        total += t1 + (t4 - t1) * (rows - 1) / 3.0
    per_tok = total / max(steps, 1)
    names = {tag: mid for tag, (mid, _) in models.items()}
    return {"value": round(1.0 / per_tok, 4), "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": (f"the fp64 oracle timed on 1-row and 4-row invocations at context {ctx} over a noise-filled cache, on "
                       f"{ {t: k for t, k in ks.items()} } layers of each model plus its LM head, scaled to the full layer count "
                       "and to each invocation's row count, summed over the invocation mix of the timed GPU run "
                       f"({len(inv)} invocations per {steps} tokens)"),
            "s_per_invocation": {tag: {"rows1": round(t_inv[mid][1], 2), "rows4": round(t_inv[mid][4], 2)} for tag, mid in names.items()}}


def fit_latency(samples):
    """Least-squares fit of the paper's latency model (Eq. 5): T = a N_inf N_kv + b N_inf^2 + c N_inf + d over
    samples (N_inf, N_kv, ms); Eq. 6 is its N_inf = 1 case.  Returns coefficients in ms and R^2."""
    import numpy as np
    a = np.array([[n * kv, n * n, n, 1.0] for n, kv, _ in samples], dtype=np.float64)
    y = np.array([t for _, _, t in samples], dtype=np.float64)
    coef, *_ = np.linalg.lstsq(a, y, rcond=None)
    pred = a @ coef
    ss_res, ss_tot = float(((y - pred) ** 2).sum()), float(((y - y.mean()) ** 2).sum())
    return {"a": float(coef[0]), "b": float(coef[1]), "c": float(coef[2]), "d": float(coef[3]),
            "r2": round(1.0 - ss_res / ss_tot, 4) if ss_tot > 0 else None, "samples": len(samples)}


PAPER_LATENCY_A100_MS = {   # Section "Latency Regression Results" (one A100, vLLM engines): a, b, c, d in ms
    "s15": (0.000021, 0.000231, -0.121046, 27.090929), "m7": (0.000027, 0.000031, -0.045256, 27.040801),
    "m14": (0.000045, 0.000123, -0.082998, 45.118931),
}


def bench_single_model(args, wl) -> int:
    """Workload without a large model: the small model decodes alone after its prompt (no routing)."""
    import torch
    import workloads as W
    from workloads import shapes as S
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedPair, SLM

    w_s = W.make_weights(wl.slm, wl.seed, 0, device="cuda")
    max_ctx = wl.max_ctx
    slm = P.Model(w_s, max_ctx=max_ctx, max_rows=128)
    pair = StitchedPair(slm, None, max_ctx, W.logit_scale(wl, 0, max_ctx + 1))
    prompt = W.make_prompt(wl).tolist()
    marks = {}

    def stop_after(n_acc):
        if n_acc == args.warmup:
            torch.cuda.synchronize()
            marks["t0"] = time.perf_counter()
        return False

    if args.warmup == 0:
        torch.cuda.synchronize()
        marks["t0"] = time.perf_counter()
    pair.generate(prompt, 2.0, args.warmup + args.steps, single_model=SLM, keep_trace=False, stop_after=stop_after)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - marks["t0"]
    ctx_mid = len(prompt) + args.warmup + args.steps // 2
    ideal = S.step_bytes(wl.slm, [ctx_mid]) / HBM_PEAK

    ev = HipEvents()
    e0, e1 = ev.create(), ev.create()
    over, ok = event_pair_overhead_ms(ev, pair.stream, e0, e1)
    roofline = gateup_roofline(ev, P, slm, wl.slm, lambda i: pair._forward(SLM, ctx_mid + i, ctx_mid + i + 1, 2.0),
                               pair.stream.synchronize, 1, over, ok, e0, e1)
    roofline["step_frac"] = {"slm": round(ideal / (elapsed / args.steps), 4)}
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(W, {"slm": (SLM, w_s)}, [(SLM, ctx_mid, 1)] * args.steps, args.steps, ctx_mid)
    print(json.dumps({
        "metric": f"decode tokens/s at batch 1 ({wl.slm.name} shape alone)", "value": round(args.steps / elapsed, 2),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": args.workload, "slm": wl.slm.name, "batch": 1, "prompt_len": len(prompt), "max_ctx": max_ctx},
        "roofline": roofline, "cpu_baseline": cpu,
        "per_model": {"slm": {"shape": wl.slm.name, "ctx": ctx_mid, "ms_per_token_wall": round(elapsed / args.steps * 1e3, 4),
                              "roofline_ms": round(ideal * 1e3, 4), "roofline_frac": round(ideal / (elapsed / args.steps), 4)}},
    }), flush=True)
    return 0


def bench_batched(args, wl) -> int:
    """Several sequences with per-sequence routing on one pair of models (the batch-8 workload)."""
    import torch
    import workloads as W
    from workloads import shapes as S
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedBatch, SLM, LLM

    nb = args.seqs or wl.n_seqs
    t0 = time.time()
    w_s = W.make_weights(wl.slm, wl.seed, 0, device="cuda")
    w_l = W.make_weights(wl.llm, wl.seed, 1, device="cuda")
    torch.cuda.synchronize()
    log(f"[bench] weights generated on the GPU in {time.time() - t0:.1f}s")
    prompts = [W.make_prompt(wl, seq=b).tolist() for b in range(nb)]
    n_total = args.warmup + args.steps
    n_tau = args.tau_steps or 128
    max_ctx = max(len(p) for p in prompts) + max(n_total, n_tau) + 8
    max_rows = 64 if nb <= 64 else 128
    slm = P.Model(w_s, max_ctx=max_ctx, max_seqs=nb, max_rows=max_rows)
    llm = P.Model(w_l, max_ctx=max_ctx, max_seqs=nb, max_rows=max_rows)
    batch = StitchedBatch(slm, llm, max_ctx, [W.logit_scale(wl, 0, max_ctx + 1, seq=b) for b in range(nb)])
    ln_v = math.log(wl.slm.vocab)
    solo = batch.generate(prompts, 2.0, n_tau, single_model=SLM)
    tau = W.pick_tau([t.h_norm for r in solo for t in r.trace], wl.tau_percentile, 4e-3 / ln_v)
    log(f"[bench] small-model-only run of {n_tau} tokens per sequence; tau = {tau:.6f}")
    # set-up: the large model processes every prompt before the timed region (its first participation)
    t0 = time.perf_counter()
    batch.prefill_prompts(LLM, prompts, tau)
    torch.cuda.synchronize()
    setup_ms = (time.perf_counter() - t0) * 1e3
    marks = {}
    calls_log = []

    def progress(accepted_total):
        if "t0" not in marks and accepted_total >= args.warmup * nb:
            torch.cuda.synchronize()
            marks["t0"] = time.perf_counter()
            marks["acc0"] = accepted_total
            marks["calls0"] = batch.calls
            marks["log0"] = len(batch.call_log)

    batch.on_call = progress
    if args.warmup == 0:
        progress(0)
    runs = batch.generate(prompts, tau, n_total, llm_prefilled=True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - marks["t0"]
    accepted = sum(len(r.output) for r in runs) - marks["acc0"]
    calls = batch.calls - marks["calls0"]
    calls_log = batch.call_log[marks["log0"]:]
    llm_tok = sum(1 for r in runs for t in r.trace if t.model == LLM and t.accept)
    all_tok = sum(len(r.output) for r in runs)
    shapes = {SLM: wl.slm, LLM: wl.llm}
    # algorithmic bytes of every library call of the timed region: weights once per call, each sequence's cache once
    ideal_s = sum(S.step_bytes(shapes[m], ctxs, rows) for m, ctxs, rows in calls_log) / HBM_PEAK
    frac = llm_tok / max(all_tok, 1)

    # the large model alone on the same prompts (the row the paper's batch-size table compares with): a short run,
    # after the timed region
    batch.on_call = None
    n_llm = min(n_total, 24)
    batch.generate(prompts, tau, 4, single_model=LLM, llm_prefilled=True)          # captures the launch graphs
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    batch.generate(prompts, tau, n_llm, single_model=LLM, llm_prefilled=True)
    torch.cuda.synchronize()
    llm_only_s = time.perf_counter() - t0

    ev = HipEvents()
    e0, e1 = ev.create(), ev.create()
    over, ok = event_pair_overhead_ms(ev, batch.stream, e0, e1)
    lengths = [len(p) + n_total - 2 for p in prompts]
    entries = [(b, lengths[b] - 1, 1) for b in range(nb)]
    roofline = gateup_roofline(ev, P, llm, wl.llm, lambda i: batch.raw_call(LLM, entries, tau, lengths),
                               batch.stream.synchronize, nb, over, ok, e0, e1, n=12)
    roofline["step_frac"] = {"stitched": round(ideal_s / elapsed, 4)}
    cpu = None
    if not args.no_cpu_baseline:
        ctx = sum(lengths) // nb
        inv = [(m, 0, rows) for m, _, rows in calls_log]
        cpu = cpu_baseline(W, {"slm": (SLM, w_s), "llm": (LLM, w_l)}, inv, accepted, ctx)
        cpu["sample"] += "; a call over several sequences is costed as one oracle invocation of its total row count"
    print(json.dumps({
        "metric": f"stitched decode tokens/s over {nb} sequences ({wl.llm.name}+{wl.slm.name} shapes)",
        "value": round(accepted / elapsed, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / max(accepted, 1) * nb * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": args.workload + (f" with {nb} sequences" if nb != wl.n_seqs else ""), "slm": wl.slm.name,
                   "llm": wl.llm.name, "batch": nb, "prompt_lens": [len(p) for p in prompts], "tau": round(tau, 6), "tau_percentile": wl.tau_percentile,
                   "max_ctx": max_ctx},
        "roofline": roofline, "cpu_baseline": cpu,
        "setup": {"llm_prompt_prefill_ms": round(setup_ms, 2)},
        "llm_only": {"tokens_per_s": round(nb * n_llm / llm_only_s, 2), "ms_per_step": round(llm_only_s / n_llm * 1e3, 4),
                     "tokens_per_sequence": n_llm, "stitched_speedup": round(accepted / elapsed / (nb * n_llm / llm_only_s), 3)},
        "stitched": {"accepted_tokens": accepted, "library_calls": calls, "llm_token_frac": round(frac, 4),
                     "ms_per_call": round(elapsed / max(calls, 1) * 1e3, 4),
                     "rejected_slm_steps": sum(1 for r in runs for t in r.trace if not t.accept),
                     "roofline_ms_per_token": round(ideal_s / max(accepted, 1) * 1e3, 4),
                     "roofline_frac": round(ideal_s / elapsed, 4)},
    }), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="accepted tokens in the timed region (default per workload: 4032 for cfg3, 448 for cfg2, 256 for "
                         "cfg4, 96 per sequence for a workload of several sequences)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="accepted tokens before the timed region (default 64; 32 for cfg4, 16 for several sequences)")
    ap.add_argument("--workload", default="cfg3_s15_m7")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-latency-fit", action="store_true")
    ap.add_argument("--no-device-loop", action="store_true")
    ap.add_argument("--tau-steps", type=int, default=None, help="small-model-only tokens used to place tau")
    ap.add_argument("--seqs", type=int, default=None, help="run a two-model workload over this many sequences (1..128) with per-sequence routing, through the batched driver")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain elementwise kernel that reads and writes 256 MiB, three times: the "
                         "known-size dispatch that hardware byte counters of a profiler run are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    import workloads as W
    from workloads import shapes as S
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedPair, SLM, LLM

    if args.workload not in W.WORKLOADS:
        print(f"bench.py: unknown workload {args.workload!r}; known: {', '.join(W.WORKLOADS)}", file=sys.stderr)
        return 2
    wl = W.WORKLOADS[args.workload]
    if wl.max_ctx < 1024:
        print(f"bench.py: {args.workload} is a parity-test workload (a context of {wl.max_ctx}): the timed passes here "
              "assume the real shapes", file=sys.stderr)
        return 2
    several = wl.n_seqs > 1 or args.seqs is not None
    d_steps, d_warmup = DEFAULT_STEPS.get(args.workload, (256, 32))
    if several:
        d_steps, d_warmup = 96, 16
    if args.warmup is None:
        args.warmup = d_warmup
    if args.steps is None:
        args.steps = d_steps if several else min(d_steps, wl.n_decode - args.warmup)
    if args.steps < 1 or args.warmup < 0 or (not several and args.warmup + args.steps > wl.n_decode):
        print(f"bench.py: need steps >= 1, warmup >= 0 and warmup + steps <= {wl.n_decode}", file=sys.stderr)
        return 2
    if args.seqs is not None and not 1 <= args.seqs <= 128:
        print("bench.py: --seqs must be in 1..128", file=sys.stderr)
        return 2
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if wl.llm is None:
        return bench_single_model(args, wl)
    if wl.n_seqs > 1 or args.seqs is not None:
        return bench_batched(args, wl)
    dev = "cuda"
    t0 = time.time()
    w_s = W.make_weights(wl.slm, wl.seed, 0, device=dev)
    w_l = W.make_weights(wl.llm, wl.seed, 1, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] weights generated on the GPU in {time.time() - t0:.1f}s")
    max_ctx = wl.max_ctx
    slm = P.Model(w_s, max_ctx=max_ctx, max_rows=128)
    llm = P.Model(w_l, max_ctx=max_ctx, max_rows=128)
    prompt = W.make_prompt(wl).tolist()
    scales = W.logit_scale(wl, 0, max_ctx + 1)
    pair = StitchedPair(slm, llm, max_ctx, scales)
    ln_v = math.log(wl.slm.vocab)

    # ---- tau: percentile of the small model's normalised entropies over a small-model-only run
    n_tau = wl.n_decode if args.tau_steps is None else args.tau_steps
    t0 = time.time()
    solo = pair.generate(prompt, 2.0, n_tau, single_model=SLM)
    tau = W.pick_tau([t.h_norm for t in solo.trace], wl.tau_percentile, 4e-3 / ln_v)
    log(f"[bench] small-model-only run: {n_tau} tokens in {time.time() - t0:.2f}s; tau = {tau:.6f}")

    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)           # one dispatch: 2^28 bytes read, 2^28 bytes written
        torch.cuda.synchronize()
        del src, dst

    ev = HipEvents()
    stats = {"timed": False, "inv": [], "dt": [], "t_prev": 0.0}

    def on_inv(model, pos0, n_rows):
        now = time.perf_counter()
        if stats["timed"]:
            stats["inv"].append((model, pos0, n_rows))
            stats["dt"].append(now - stats["t_prev"])          # wall time of this invocation (call, sync, host loop)
        stats["t_prev"] = now

    # ---- set-up: the large model's first participation (a prefill of the whole prompt, Section "KV Cache
    # management") happens here, before the timed region, whatever the warm-up length is.  Its K/V rows are the
    # ones the loop would have written at the first hand-over.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pair.prefill_prompt(LLM, prompt, tau)
    torch.cuda.synchronize()
    setup_ms = (time.perf_counter() - t0) * 1e3
    log(f"[bench] set-up: large-model prompt prefill of {len(prompt)} tokens in {setup_ms:.1f} ms")
    pair.on_invocation = on_inv

    # ---- live stitched run: warmup tokens, then the timed region
    marks = {}

    def stop_after(n_acc):
        if n_acc == args.warmup:
            torch.cuda.synchronize()
            stats["timed"] = True
            marks["t0"] = time.perf_counter()
            stats["t_prev"] = marks["t0"]
        return False

    if args.warmup == 0:
        stats["timed"] = True
        torch.cuda.synchronize()
        marks["t0"] = time.perf_counter()
        stats["t_prev"] = marks["t0"]
    run = pair.generate(prompt, tau, args.warmup + args.steps, stop_after=stop_after, llm_prefilled=True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - marks["t0"]
    pair.on_invocation = None
    tokens_per_s = args.steps / elapsed

    # ---- invocation mix and stitched roofline of the timed region (an invocation longer than max_rows is fed in
    # chunks, each of which reads the weights once)
    inv = stats["inv"]
    shapes = {SLM: wl.slm, LLM: wl.llm}
    mr = pair.max_rows

    def inv_bytes(m, p0, n):
        return sum(S.step_bytes(shapes[m], [p0 + c0 + min(mr, n - c0)], min(mr, n - c0)) for c0 in range(0, n, mr))

    ideal_s = sum(inv_bytes(m, p0, n) for m, p0, n in inv) / HBM_PEAK
    n_llm_inv = sum(1 for m, _, _ in inv if m == LLM)
    n_slm_inv = len(inv) - n_llm_inv
    timed_trace = run.trace[-len(inv):] if inv else []
    llm_tokens = sum(1 for t in timed_trace if t.model == LLM and t.accept)
    rejected = sum(1 for t in timed_trace if not t.accept)
    spans = [n for m, _, n in inv if m == LLM]
    # decode steps against catch-up calls, per model: count and mean wall time by span length
    by_span = {"slm": {}, "llm": {}}
    for (m_, _, n), dt in zip(inv, stats["dt"]):
        key = str(n) if n <= 4 else ("5-8" if n <= 8 else ("9-16" if n <= 16 else ("17-32" if n <= 32 else "33+")))
        rec = by_span["slm" if m_ == SLM else "llm"].setdefault(key, [0, 0.0])
        rec[0] += 1
        rec[1] += dt
    by_span = {k: {sp: {"calls": c, "ms": round(t / c * 1e3, 3)} for sp, (c, t) in sorted(v.items(), key=lambda kv: (len(kv[0]), kv[0]))}
               for k, v in by_span.items()}
    switches = sum(1 for i in range(1, len(inv)) if inv[i][0] != inv[i - 1][0])

    # ---- each model alone: decode steps at the end of the context, GPU time per step from an
    # event pair around every call (wall time per step, with the host round trip, beside it)
    per_model = {}
    sh = pair.stream.cuda_stream
    a, b = ev.create(), ev.create()
    for tag, mid, shape in (("slm", SLM, wl.slm), ("llm", LLM, wl.llm)):
        n_steps, p_start = 64, max_ctx - 64 - 1
        gpu_ms, t_wall = 0.0, 0.0
        for rep in range(2):                      # first pass warms up (and captures the launch graph)
            gpu_ms = 0.0
            t_w0 = time.perf_counter()
            for i in range(n_steps):
                ev.record(a, sh)
                pair._forward(mid, p_start + i, p_start + i + 1, tau)
                ev.record(b, sh)
                pair.stream.synchronize()
                gpu_ms += ev.elapsed_ms(a, b)
            t_wall = time.perf_counter() - t_w0
        ms = gpu_ms / n_steps
        bytes_step = S.step_bytes(shape, [p_start + n_steps // 2 + 1])
        per_model[tag] = {"shape": shape.name, "ctx": p_start + n_steps // 2, "ms_per_token": round(ms, 4),
                          "ms_per_token_wall": round(t_wall / n_steps * 1e3, 4),
                          "roofline_ms": round(bytes_step / HBM_PEAK * 1e3, 4),
                          "roofline_frac": round(bytes_step / HBM_PEAK / (ms * 1e-3), 4)}

    # ---- dominant kernel, picked by name: the large model's single-row gate/up projection (over half of the
    # bytes of the largest model's step), in plain-launch decode steps at the end of the context
    e0, e1 = ev.create(), ev.create()
    event_overhead_ms, overhead_ok = event_pair_overhead_ms(ev, pair.stream, e0, e1)
    p_roof = max_ctx - 40
    roofline = gateup_roofline(ev, P, llm, wl.llm, lambda i: pair._forward(LLM, p_roof + i, p_roof + i + 1, tau),
                               pair.stream.synchronize, 1, event_overhead_ms, overhead_ok, e0, e1)
    # the whole decode step of each model against its own roofline (weights + KV bytes per token at 8 TB/s): the
    # figure the target is stated on; the kernel above is the best-placed part of it
    roofline["step_frac"] = {"slm": per_model["slm"]["roofline_frac"], "llm": per_model["llm"]["roofline_frac"],
                             "min": min(per_model["slm"]["roofline_frac"], per_model["llm"]["roofline_frac"]),
                             "stitched_run": round(ideal_s / elapsed, 4)}

    # ---- what the router costs: the fused LM head + softmax-state kernel of each model (event pair around that
    # kernel in a plain-launch decode step) beside the standalone router of the same rows (rs_route on logits in
    # HBM: two small kernels after an LM head that would have to write V floats and read them back).  The paper
    # reports 0.028 ms per token for its separate entropy evaluation.
    router = {}
    vocab = wl.slm.vocab
    logits = torch.randn(1, vocab, device=dev, dtype=torch.float32)
    r_out = P.binding.new_route_out(1, device=dev)
    r_scratch = torch.empty(P.binding.rs_route_scratch_bytes(1, vocab), dtype=torch.uint8, device=dev)
    for _ in range(3):
        P.binding.rs_route(logits, 1, vocab, None, tau, 0, r_out, r_scratch, sh)
    pair.stream.synchronize()
    ev.record(a, sh)
    for _ in range(20):
        P.binding.rs_route(logits, 1, vocab, None, tau, 0, r_out, r_scratch, sh)
    ev.record(b, sh)
    pair.stream.synchronize()
    router["standalone_rs_route_us"] = round(ev.elapsed_ms(a, b) / 20 * 1e3, 2)
    for tag, mid, mdl in (("slm", SLM, slm), ("llm", LLM, llm)):
        lm_ms = time_phase(ev, P, mdl, P.binding.PHASE_LMHEAD, 0,
                           lambda i, mid=mid: pair._forward(mid, max_ctx - 16 + i, max_ctx - 15 + i, tau),
                           pair.stream.synchronize, 8, e0, e1) - event_overhead_ms
        shape = wl.slm if mid == SLM else wl.llm
        lm_bytes = shape.vocab * shape.d_model * 2
        router[f"{tag}_lm_head_with_fused_router_us"] = round(lm_ms * 1e3, 2)
        router[f"{tag}_lm_head_gbps"] = round(lm_bytes / (lm_ms * 1e-3) / 1e9, 1)
    router["paper_separate_entropy_us"] = 28.0

    # ---- Algorithm 1 with the loop itself on the device (rs_stitch_generate: one kernel, nothing read by the host
    # until the end) on a bounded number of tokens, beside the host-driven loop over the same tokens; both start
    # with all but the last prompt token in both caches
    device_loop = None
    # (a process that has launched a cooperative kernel was seen to crash inside rocprofv3's exit handler, after
    # the result line was printed: under the profiler this leg is left out)
    profiled = any("rocprofiler" in os.environ.get(k, "") for k in ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES", "HSA_TOOLS_LIB"))
    if profiled and not args.no_device_loop:
        log("[bench] a rocprofiler tool is loaded: the device-resident loop leg is skipped")
        device_loop = {"skipped": "rocprofiler tool loaded"}
    elif not args.no_device_loop:
        n_dl = min(48, args.steps)
        pair.on_invocation = None
        for mid in (SLM, LLM):
            pair.prefill_prompt(mid, prompt, tau)
        pair.generate(prompt, tau, 4, llm_prefilled=True, slm_prefilled=True)          # graphs of this start
        t0 = time.perf_counter()
        host_run = pair.generate(prompt, tau, n_dl, llm_prefilled=True, slm_prefilled=True)
        host_s = time.perf_counter() - t0
        dev_run = pair.generate_on_device(prompt, tau, n_dl, prompt_prefilled=True)
        device_loop = {"tokens": n_dl, "status": dev_run.status, "invocations": len(dev_run.trace),
                       "tokens_per_s": round(n_dl / (dev_run.loop_ms * 1e-3), 2),
                       "ms_per_token": round(dev_run.loop_ms / n_dl, 4),
                       "host_loop_tokens_per_s": round(n_dl / host_s, 2),
                       "same_tokens_as_host_loop": dev_run.output == host_run.output}

    # ---- latency model of the paper (Eq. 5-6) re-fitted to this machine: GPU time of calls with N_inf token rows
    # on a cache of N_kv positions, each model; coefficients in ms beside the paper's A100 ones
    latency_fit = None
    if not args.no_latency_fit:
        latency_fit = {}
        for tag, mid, shape in (("slm", SLM, wl.slm), ("llm", LLM, wl.llm)):
            samples = []
            for n_inf in (1, 2, 4, 8, 16, 32, 64):
                for n_kv in (256, max_ctx // 4, max_ctx // 2, max_ctx - 72):
                    for rep in range(3):            # the last of three (graph captured by then)
                        ev.record(a, sh)
                        pair._forward(mid, n_kv, n_kv + n_inf, tau)
                        ev.record(b, sh)
                        pair.stream.synchronize()
                    samples.append((n_inf, n_kv, ev.elapsed_ms(a, b)))
            fit = fit_latency(samples)
            fit["decode_ms_at"] = {str(kv): round(t, 4) for n, kv, t in samples if n == 1}
            fit["paper_a100_ms"] = dict(zip("abcd", PAPER_LATENCY_A100_MS.get(shape.name, (None,) * 4)))
            latency_fit[tag] = fit

    # ---- CPU oracle on a bounded sample of the benchmarked work
    cpu = None
    if not args.no_cpu_baseline:
        ctx_mid = len(prompt) + args.warmup + args.steps // 2
        cpu = cpu_baseline(W, {"slm": (SLM, w_s), "llm": (LLM, w_l)}, inv, args.steps, ctx_mid)

    line = {
        "metric": ("stitched decode tokens/s at batch 1 (7B+1.5B shapes)" if args.workload == "cfg3_s15_m7"
                   else f"stitched decode tokens/s at batch 1 ({wl.llm.name}+{wl.slm.name} shapes)"),
        "value": round(tokens_per_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": args.workload, "slm": wl.slm.name, "llm": wl.llm.name, "batch": 1,
                   "prompt_len": len(prompt), "tau": round(tau, 6), "tau_percentile": wl.tau_percentile,
                   "max_ctx": max_ctx},
        "roofline": roofline,
        "per_model": per_model,
        "setup": {"llm_prompt_prefill_ms": round(setup_ms, 2), "llm_prompt_tokens": len(prompt)},
        "stitched": {"invocations": len(inv), "slm_invocations": n_slm_inv, "llm_invocations": n_llm_inv,
                     "llm_token_frac": round(llm_tokens / max(args.steps, 1), 4), "rejected_slm_steps": rejected,
                     "llm_span_mean": round(sum(spans) / max(len(spans), 1), 2), "llm_span_max": max(spans) if spans else 0,
                     "model_switches": switches, "calls_by_span": by_span,
                     "roofline_ms_per_token": round(ideal_s / args.steps * 1e3, 4),
                     "roofline_frac": round(ideal_s / elapsed, 4)},
        "router": router,
        "device_loop": device_loop,
        "latency_fit": latency_fit,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
