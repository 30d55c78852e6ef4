#!/usr/bin/env python3
"""Headline benchmark: stitched decode tokens/s at batch 1 on the 1.5B + 7B shapes
(workload cfg3_s15_m7), with the fraction of the per-token HBM roofline.

A "step" is one ACCEPTED token of the live stitched run (Algorithm 1 driven from
the host through the C ABI): it costs one or more model invocations - small-model
decode steps (accepted or rejected), large-model catch-up prefills and decode
steps.  All inputs (weights, prompt, logit-scale schedule) are seeded synthetic
data resident in HBM before the timed region starts.

Prints ONE JSON line.  Extra objects:
  roofline      live HIP-event timing of the dominant kernel (the large model's
                gate/up projection) against the 8 TB/s HBM peak
  per_model     decode ms/token of each model alone and its roofline fraction
  stitched      invocation mix of the timed region and its roofline fraction
  cpu_baseline  the CPU oracle timed on this machine's cores on a small sample
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12   # bytes/s, MI355X published


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


def bench_single_model(args, wl) -> int:
    """Workload without a large model: the small model decodes alone after its prompt (no routing)."""
    import torch
    import workloads as W
    from workloads import shapes as S
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedPair, SLM

    w_s = W.make_weights(wl.slm, wl.seed, 0, device="cuda")
    max_ctx = wl.max_ctx
    slm = P.Model(w_s, max_ctx=max_ctx, max_rows=64)
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
    print(json.dumps({
        "metric": f"decode tokens/s at batch 1 ({wl.slm.name} shape alone)", "value": round(args.steps / elapsed, 2),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights, f32 activations and accumulation", "data": "synthetic",
        "config": {"workload": args.workload, "slm": wl.slm.name, "batch": 1, "prompt_len": len(prompt), "max_ctx": max_ctx},
        "roofline": None, "cpu_baseline": None,
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

    nb = wl.n_seqs
    t0 = time.time()
    w_s = W.make_weights(wl.slm, wl.seed, 0, device="cuda")
    w_l = W.make_weights(wl.llm, wl.seed, 1, device="cuda")
    torch.cuda.synchronize()
    log(f"[bench] weights generated on the GPU in {time.time() - t0:.1f}s")
    prompts = [W.make_prompt(wl, seq=b).tolist() for b in range(nb)]
    n_total = args.warmup + args.steps
    max_ctx = max(len(p) for p in prompts) + max(n_total, args.tau_steps or 0) + 8
    slm = P.Model(w_s, max_ctx=max_ctx, max_seqs=nb, max_rows=64)
    llm = P.Model(w_l, max_ctx=max_ctx, max_seqs=nb, max_rows=64)
    batch = StitchedBatch(slm, llm, max_ctx, [W.logit_scale(wl, 0, max_ctx + 1, seq=b) for b in range(nb)])
    ln_v = math.log(wl.slm.vocab)
    n_tau = args.tau_steps or 128
    solo = batch.generate(prompts, 2.0, n_tau, single_model=SLM)
    tau = W.pick_tau([t.h_norm for r in solo for t in r.trace], wl.tau_percentile, 4e-3 / ln_v)
    log(f"[bench] small-model-only run of {n_tau} tokens per sequence; tau = {tau:.6f}")
    marks = {}

    def progress(accepted_total):
        if "t0" not in marks and accepted_total >= args.warmup * nb:
            torch.cuda.synchronize()
            marks["t0"] = time.perf_counter()
            marks["acc0"] = accepted_total
            marks["calls0"] = batch.calls

    batch.on_call = progress
    runs = batch.generate(prompts, tau, n_total)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - marks["t0"]
    accepted = sum(len(r.output) for r in runs) - marks["acc0"]
    calls = batch.calls - marks["calls0"]
    llm_tok = sum(1 for r in runs for t in r.trace if t.model == LLM and t.accept)
    all_tok = sum(len(r.output) for r in runs)
    # roofline of one round in which every sequence takes a small-model step and the routed share a large-model step
    ctx = [len(p) + n_total // 2 for p in prompts]
    frac = llm_tok / max(all_tok, 1)
    ideal_round = (S.step_bytes(wl.slm, ctx) + frac * S.step_bytes(wl.llm, ctx)) / HBM_PEAK
    print(json.dumps({
        "metric": f"stitched decode tokens/s over {nb} sequences ({wl.llm.name}+{wl.slm.name} shapes)",
        "value": round(accepted / elapsed, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / max(accepted, 1) * nb * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 weights, f32 activations and accumulation", "data": "synthetic",
        "config": {"workload": args.workload, "slm": wl.slm.name, "llm": wl.llm.name, "batch": nb,
                   "prompt_lens": [len(p) for p in prompts], "tau": round(tau, 6), "tau_percentile": wl.tau_percentile,
                   "max_ctx": max_ctx},
        "roofline": None, "cpu_baseline": None,
        "stitched": {"accepted_tokens": accepted, "library_calls": calls, "llm_token_frac": round(frac, 4),
                     "ms_per_call": round(elapsed / max(calls, 1) * 1e3, 4),
                     "rejected_slm_steps": sum(1 for r in runs for t in r.trace if not t.accept),
                     "roofline_ms_per_round_estimate": round(ideal_round * 1e3, 4)},
    }), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4032, help="accepted tokens in the timed region")
    ap.add_argument("--warmup", type=int, default=64, help="accepted tokens before the timed region")
    ap.add_argument("--workload", default="cfg3_s15_m7")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tau-steps", type=int, default=None, help="small-model-only tokens used to place tau")
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

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    wl = W.WORKLOADS[args.workload]
    if wl.llm is None:
        return bench_single_model(args, wl)
    if wl.n_seqs > 1:
        return bench_batched(args, wl)
    if args.warmup + args.steps > wl.n_decode:
        print(f"bench.py: warmup + steps must not exceed {wl.n_decode}", file=sys.stderr)
        return 2
    dev = "cuda"
    t0 = time.time()
    w_s = W.make_weights(wl.slm, wl.seed, 0, device=dev)
    w_l = W.make_weights(wl.llm, wl.seed, 1, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] weights generated on the GPU in {time.time() - t0:.1f}s")
    max_ctx = wl.max_ctx
    slm = P.Model(w_s, max_ctx=max_ctx, max_rows=64)
    llm = P.Model(w_l, max_ctx=max_ctx, max_rows=64)
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

    pair.on_invocation = on_inv

    # ---- live stitched run: warmup tokens, then the timed region
    marks = {}

    def stop_after(n_acc):
        if n_acc == args.warmup:
            torch.cuda.synchronize()
            stats["timed"] = True
            marks["t0"] = time.perf_counter()
        return False

    if args.warmup == 0:
        stats["timed"] = True
        torch.cuda.synchronize()
        marks["t0"] = time.perf_counter()
    run = pair.generate(prompt, tau, args.warmup + args.steps, stop_after=stop_after)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - marks["t0"]
    pair.on_invocation = None
    tokens_per_s = args.steps / elapsed

    # ---- invocation mix and stitched roofline of the timed region
    inv = stats["inv"]
    shapes = {SLM: wl.slm, LLM: wl.llm}
    ideal_s = sum(S.step_bytes(shapes[m], [p0 + n], n) for m, p0, n in inv) / HBM_PEAK
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

    # ---- dominant kernel: the large model's gate/up projection.  The launch graphs of the timed
    # region cannot carry event records, so the same invocations (same kernels, grids and data) are
    # replayed right after it as plain launches with an event pair around that one kernel.
    e0, e1 = ev.create(), ev.create()
    gateup_bytes = 2 * wl.llm.d_ffn * wl.llm.d_model * 2
    kern = {}
    P.rs_set_phase_timer(llm.handle, P.binding.PHASE_GATEUP, wl.llm.n_layers // 2, e0, e1)
    for m_, p0, n in [x for x in inv if x[0] == LLM][:96]:
        if n > pair.max_rows:
            continue
        pair._forward(LLM, p0, p0 + n, tau)
        pair.stream.synchronize()
        name = "k_gemv<GATEUP,rows<=1>" if n == 1 else f"k_gemm_rows<GATEUP,NB={1 if n <= 16 else (2 if n <= 32 else 4)}>"
        k = kern.setdefault(name, [0, 0.0])
        k[0] += 1
        k[1] += ev.elapsed_ms(e0, e1)
    P.rs_set_phase_timer(llm.handle, -1)
    # What the two event records themselves add to such a bracket: the same bracket around one launch of a
    # streaming kernel of about the same length (an in-place add over 2^24 floats, ~20 us), minus that kernel's
    # duration when 50 of them run back to back inside one bracket.  Medians over 30 brackets.
    cal_x = torch.zeros(1 << 24, device=dev)
    cal_s = torch.zeros(1 << 16, device=dev)
    sh_cal = pair.stream.cuda_stream
    with torch.cuda.stream(pair.stream):
        for _ in range(5):
            cal_x.add_(1.0)
        singles = []
        for _ in range(30):
            for _ in range(4):
                cal_s.add_(1.0)
            ev.record(e0, sh_cal)
            cal_x.add_(1.0)
            ev.record(e1, sh_cal)
            for _ in range(2):
                cal_s.add_(1.0)
            pair.stream.synchronize()
            singles.append(ev.elapsed_ms(e0, e1))
        ev.record(e0, sh_cal)
        for _ in range(50):
            cal_x.add_(1.0)
        ev.record(e1, sh_cal)
        pair.stream.synchronize()
        event_overhead_ms = sorted(singles)[len(singles) // 2] - ev.elapsed_ms(e0, e1) / 50
    del cal_x, cal_s
    # an unprofiled run gives 2.7-3.2 us; with a profiler attached every dispatch costs more and the figure
    # no longer describes the bracket, so a value outside 0..5 us is dropped and the raw bracket is reported
    overhead_ok = 0.0 <= event_overhead_ms <= 5e-3
    if not overhead_ok:
        log(f"[bench] event-pair calibration gave {event_overhead_ms * 1e3:.2f} us: not applied")
        event_overhead_ms = 0.0
    dom = max(kern.items(), key=lambda kv: kv[1][1]) if kern else None
    roofline = None
    if dom:
        name, (cnt, tot_ms) = dom
        avg_events_s = tot_ms / cnt * 1e-3
        avg_s = avg_events_s - event_overhead_ms * 1e-3
        # HBM bytes per launch of that kernel from hardware-counter runs (FETCH_SIZE + WRITE_SIZE, scaled by a
        # copy kernel of known size), stored with the package; only the single-row kernel has been counted
        traffic = None
        try:
            with open(os.path.join(os.path.dirname(os.path.abspath(P.__file__)), "measured_traffic.json")) as f:
                rec = json.load(f).get(wl.llm.name, {}).get("gateup_rows1")
            if rec and name == "k_gemv<GATEUP,rows<=1>":
                traffic = rec["fetch_bytes"] + rec["write_bytes"]
        except OSError:
            pass
        roofline = {"bound": "hbm", "kernel": name, "launches": cnt, "avg_us": round(avg_s * 1e6, 2),
                    "avg_us_between_events": round(avg_events_s * 1e6, 2),
                    "event_pair_overhead_us": round(event_overhead_ms * 1e3, 2) if overhead_ok else None,
                    "achieved": round(gateup_bytes / avg_s / 1e9, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                    "frac": round(gateup_bytes / avg_s / HBM_PEAK, 4), "traffic": traffic,
                    "bytes_per_launch": gateup_bytes,
                    "measured": "replay of the timed region's large-model invocations as plain launches, one event "
                                "pair around this kernel per invocation; avg_us = time between the events minus what "
                                "the event records add to such a bracket (calibrated in this run)",
                    "all_variants": {k: {"launches": v[0], "avg_us": round((v[1] / v[0] - event_overhead_ms) * 1e3, 2)}
                                     for k, v in kern.items()}}

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
        P.rs_set_phase_timer(mdl.handle, P.binding.PHASE_LMHEAD, 0, e0, e1)
        tot = 0.0
        for i in range(8):
            pair._forward(mid, max_ctx - 16 + i, max_ctx - 15 + i, tau)
            pair.stream.synchronize()
            tot += ev.elapsed_ms(e0, e1)
        P.rs_set_phase_timer(mdl.handle, -1)
        shape = wl.slm if mid == SLM else wl.llm
        lm_bytes = shape.vocab * shape.d_model * 2
        lm_ms = tot / 8 - event_overhead_ms          # the same bracket as the roofline kernel's, same correction
        router[f"{tag}_lm_head_with_fused_router_us"] = round(lm_ms * 1e3, 2)
        router[f"{tag}_lm_head_gbps"] = round(lm_bytes / (lm_ms * 1e-3) / 1e9, 1)
    router["paper_separate_entropy_us"] = 28.0

    # ---- CPU oracle on a bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import decoder as odec
        torch.set_grad_enabled(False)
        t_inv = {}
        for tag, wts in (("slm", w_s), ("llm", w_l)):
            t0 = time.time()
            w_cpu = wts.to("cpu")
            om = odec.OracleModel(w_cpu, max_ctx=8, keep_fp64_weights=False)
            t1 = time.time()
            om.forward(prompt[:1], 0)
            t_inv[tag] = time.time() - t1
            log(f"[bench] oracle {tag}: one invocation {t_inv[tag]:.1f}s (+{t1 - t0:.1f}s to copy weights to the host)")
            del om, w_cpu
        per_tok = (n_slm_inv * t_inv["slm"] + n_llm_inv * t_inv["llm"]) / max(args.steps, 1)
        cpu = {"value": round(1.0 / per_tok, 4), "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
               "sample": ("one 1-token invocation of each full-shape oracle model (fp64, weights converted from bf16 per "
                          "layer), combined with the invocation mix of the timed GPU run: "
                          f"{n_slm_inv} small-model and {n_llm_inv} large-model invocations per {args.steps} tokens"),
               "s_per_invocation": {k: round(v, 2) for k, v in t_inv.items()}}

    line = {
        "metric": ("stitched decode tokens/s at batch 1 (7B+1.5B shapes)" if args.workload == "cfg3_s15_m7"
                   else f"stitched decode tokens/s at batch 1 ({wl.llm.name}+{wl.slm.name} shapes)"),
        "value": round(tokens_per_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 weights, f32 activations and accumulation", "data": "synthetic",
        "config": {"workload": args.workload, "slm": wl.slm.name, "llm": wl.llm.name, "batch": 1,
                   "prompt_len": len(prompt), "tau": round(tau, 6), "tau_percentile": wl.tau_percentile,
                   "max_ctx": max_ctx},
        "roofline": roofline,
        "per_model": per_model,
        "stitched": {"invocations": len(inv), "slm_invocations": n_slm_inv, "llm_invocations": n_llm_inv,
                     "llm_token_frac": round(llm_tokens / max(args.steps, 1), 4), "rejected_slm_steps": rejected,
                     "llm_span_mean": round(sum(spans) / max(len(spans), 1), 2), "llm_span_max": max(spans) if spans else 0,
                     "model_switches": switches, "calls_by_span": by_span,
                     "roofline_ms_per_token": round(ideal_s / args.steps * 1e3, 4),
                     "roofline_frac": round(ideal_s / elapsed, 4)},
        "router": router,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
