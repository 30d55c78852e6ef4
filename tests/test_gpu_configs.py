"""GPU parity at the REAL shapes of configurations 2-5, element by element against the oracle, through the C ABI.

  * cfg2: the whole 28-layer 1.5B shape; the model itself prefills a prompt, then 16 consecutive decode steps are
    checked one by one (the oracle's tokens AND cache rows are teacher-forced: the rows the GPU writes are compared
    with the oracle's, then replaced by them, see check_and_force_rows);
  * cfg3: a stitched prefix on the whole 1.5B + 7B pair: the oracle runs Algorithm 1 (entropy threshold from its
    own small-model-only run), the GPU replays every invocation of that trace - small-model steps, rejected
    steps, large-model catch-up prefills of several tokens, hand-backs - and is compared per invocation (calls of
    several rows in two parts, see check_span);
  * cfg4 / cfg5: ALL 48 layers of the 14B shape and ALL 64 layers of the 32B shape, one decode step and one
    multi-row catch-up at the full context of the configuration (the cache under them is seeded noise: an oracle
    prefill of 9-10k tokens at these sizes would take hours);
  * cfg5: eight sequences in distinct cache slots at the 1.5B and 32B layer shapes (two layers, full vocabulary,
    full 10240-position caches): one ragged rs_catchup_prefill and one batched rs_decode_step against the oracle
    run sequence by sequence.
The oracle keeps its weights in bf16 and converts a layer at a time where fp64 copies would not fit.
"""
import gc
import math
import sys
import time

import pytest
import torch

import workloads as W
from oracle import decoder, router, stitch
from parity import check_invocation

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def release():
    gc.collect()
    torch.cuda.empty_cache()


def check_and_force_rows(gpu, ref, slot, pos0, n, where):
    """The K/V rows pos0 .. pos0+n-1 the GPU has just written against the oracle's: every element equal or one bf16
    step away (both sides round nearly equal fp32 / fp64 values to bf16; once a first rounding has flipped, the rows of
    deeper layers see inputs that differ by ~1e-4 .. 1e-3 and up to a third of their elements flip too: measured 31 %
    for the 65-row first prefill of the 7B shape).  Then the oracle's rows replace the GPU's.

    Why they are replaced: the cache is state that later invocations read.  A flipped bf16 rounding in a cached row is
    a 2^-8 relative change that both sides then carry forward differently; over a hundred positions and 28 layers
    such flips move the entropy of a later step by more than the 1e-3 nats the task allows (measured without the
    replacement: step 16 of the 1.5B-shape run below is off by 1.35e-3 nats, steps 1-15 are inside the tolerance; the
    oracle alone shows the same amplification, tests/test_oracle_rounding_contract.py).  The comparison is teacher-forced so
    that drift cannot cascade: like the token sequence, the cache contents are the oracle's at every invocation."""
    for name, cache in (("k", ref.k_cache), ("v", ref.v_cache)):
        view = gpu.kv_view(name)[:, slot, :, pos0:pos0 + n]
        r = cache[:, slot, :, pos0:pos0 + n]
        g = view.float().cpu().double()
        # element by element: one bf16 step of the element (spacing at most 2^-7 of its value) plus what the values
        # differed by before rounding, at most 2^-8 of the layer's largest entry (measured: up to 1.2e-3 of it in the
        # deepest layers of a 65-row prefill of the 7B shape, where the flipped roundings of 27 layers have fed forward;
        # a wrong row, head, position or rotation would be off by the entry's own size)
        scale = r.abs().amax(dim=(1, 2, 3), keepdim=True)
        worst = float(((g - r).abs() - 2 ** -7 * r.abs() - 2 ** -8 * scale).max())
        assert worst <= 0.0, f"{where}: a {name} element is further from the oracle's than rounding explains ({worst})"
        rel = float(((g - r) ** 2).sum().sqrt() / (r ** 2).sum().sqrt())
        assert rel <= 2 ** -8, f"{where}: {name} rows differ by {rel} in relative Frobenius norm"
        view.copy_(r.to(torch.float32).to(torch.bfloat16).cuda())


DRIFT_ENTROPY_TOL = 1e-2      # whole multi-row invocation against the oracle's own run (see check_span)
DRIFT_LOGIT_TOL = 6e-2


def check_span(gpu, ref, slot, span, pos0, scale, got, lg, ref_logits, tau, active, where):
    """A call over SEVERAL rows whose K/V rows the model writes itself, on a deep model.

    Inside such a call the rows of later layers are computed from K/V rows written earlier in the same call, so the
    bf16 roundings that flip between the two sides feed forward through all layers and no cache row can be
    teacher-forced in between.  What the two sides must agree on is therefore checked in two parts:
      * the rows written (check_and_force_rows, by the caller): every K/V element equal or one bf16 step apart;
      * the distribution of the LAST row given the cache contents: the oracle is run on that one row over the rows
        the GPU wrote for the earlier positions of the span, and the GPU's record and logits must match it within the
        tolerances of the task (this is what the router sees).
    The whole call against the oracle's own run is held to looser bounds only, 6e-2 on the logits and 1e-2 nats
    (measured: 2.3e-2 on logits of magnitude ~40 for the 65-row first prefill of the 7B shape, 2.4e-3 nats for the
    64-row prefill of the 1.5B shape; two runs of the oracle alone whose inputs differ by a few parts in 10^6 move as
    much, tests/test_oracle_rounding_contract.py)."""
    n = len(span)
    err = float((lg.detach().cpu().double() - ref_logits).abs().max())
    assert err <= DRIFT_LOGIT_TOL, f"{where}: logits max-abs error {err} against the oracle's own run"
    dh = abs(got.h_nats - router.entropy_nats(ref_logits))
    assert dh <= DRIFT_ENTROPY_TOL, f"{where}: entropy drifts by {dh} nats against the oracle's own run"
    saved = [c[:, slot, :, pos0:pos0 + n].clone() for c in (ref.k_cache, ref.v_cache)]
    for name, cache in (("k", ref.k_cache), ("v", ref.v_cache)):
        cache[:, slot, :, pos0:pos0 + n - 1] = gpu.kv_view(name)[:, slot, :, pos0:pos0 + n - 1].float().cpu().double()
    want = ref.forward([span[-1]], pos0 + n - 1, slot=slot, logit_scale=scale)["logits"]
    for c, keep in zip((ref.k_cache, ref.v_cache), saved):
        c[:, slot, :, pos0:pos0 + n] = keep
    return check_invocation(got, lg, want, tau, active, where=where + " (last row over the rows the GPU wrote)")


def noise_cache(gpu, ref, slot, n_ctx, seed):
    """Positions [0, n_ctx) of one slot of both caches get the same seeded bf16 noise (generated once, on the GPU)."""
    c = gpu.cfg
    cnt = c.n_layers * c.n_kv_heads * n_ctx * c.head_dim
    for which, tag in (("k", 1), ("v", 2)):
        vals = torch.empty(cnt, dtype=torch.bfloat16, device="cuda")
        step = 1 << 24
        for s in range(0, cnt, step):
            vals[s:s + step] = W.rng.normal(seed, 900 + 8 * slot + tag, s, min(step, cnt - s), "cuda").to(torch.float32).to(torch.bfloat16)
        vals = vals.view(c.n_layers, c.n_kv_heads, n_ctx, c.head_dim)
        gpu.kv_view(which)[:, slot, :, :n_ctx] = vals
        cache = ref.k_cache if which == "k" else ref.v_cache
        cache[:, slot, :, :n_ctx] = vals.cpu().double()
        del vals


# ------------------------------------------------------------------------------------------------ cfg2
def test_cfg2_sixteen_consecutive_decode_steps_on_a_cache_the_model_prefilled():
    import paper_2507_17307_amd as P
    wl = W.WORKLOADS["cfg2_s15_decode"]
    n_prompt, n_steps = 96, 16
    w_gpu = W.make_weights(wl.slm, wl.seed, 0, device="cuda")
    ref = decoder.OracleModel(w_gpu.to("cpu"), n_prompt + n_steps + 1)
    gpu = P.Model(w_gpu, max_ctx=n_prompt + n_steps + 1, max_rows=64)
    prompt = W.make_prompt(wl, length=n_prompt).tolist()
    scales = W.logit_scale(wl, 0, n_prompt + n_steps + 2)
    tau = 0.8
    # prefill: the oracle in one invocation, the GPU in chunks of 64 rows; the last chunk's record is compared
    want = ref.forward(prompt, 0, logit_scale=float(scales[n_prompt]))["logits"]
    got, lg = gpu.forward_span(prompt, 0, tau, P.RS_SLM, float(scales[n_prompt]), want_logits=True)
    torch.cuda.synchronize()
    check_span(gpu, ref, 0, prompt, 0, float(scales[n_prompt]), got[0], lg[0], want, tau, router.SLM, "cfg2 prompt prefill")
    check_and_force_rows(gpu, ref, 0, 0, n_prompt, "cfg2 prompt prefill")
    tok = router.greedy_token(want)
    for i in range(n_steps):
        pos = n_prompt + i
        want = ref.forward([tok], pos, logit_scale=float(scales[pos + 1]))["logits"]
        got, lg = gpu.forward_span([tok], pos, tau, P.RS_SLM, float(scales[pos + 1]), want_logits=True)
        torch.cuda.synchronize()
        check_invocation(got[0], lg[0], want, tau, router.SLM, where=f"cfg2 decode step {i} at {pos}")
        check_and_force_rows(gpu, ref, 0, pos, 1, f"cfg2 decode step {i}")
        tok = router.greedy_token(want)               # teacher forcing: the oracle's token goes to both sides
    del gpu, ref, w_gpu
    release()


# ------------------------------------------------------------------------------------------------ cfg3
def test_cfg3_stitched_prefix_on_the_full_pair_teacher_forced():
    import paper_2507_17307_amd as P
    wl = W.WORKLOADS["cfg3_s15_m7"]
    n_prompt, n_tok, percentile = 64, 24, 60.0
    w_s = W.make_weights(wl.slm, wl.seed, 0, device="cuda")
    w_l = W.make_weights(wl.llm, wl.seed, 1, device="cuda")
    ws_cpu, wl_cpu = w_s.to("cpu"), w_l.to("cpu")
    max_ctx = n_prompt + n_tok + 2
    prompt = W.make_prompt(wl, length=n_prompt).tolist()
    scales = W.logit_scale(wl, 0, max_ctx + 1)
    sc = lambda p: float(scales[p])  # noqa: E731
    # the small model's fp64 weights fit the host (12 GB); the large model is converted layer by layer per invocation
    mk = lambda: [decoder.OracleModel(ws_cpu, max_ctx), decoder.OracleModel(wl_cpu, max_ctx, keep_fp64_weights=False)]  # noqa: E731
    t0 = time.time()
    solo = stitch.generate(prompt, stitch.decoder_forward(mk(), sc), 2.0, n_tok)
    tau = W.pick_tau([t.h_norm for t in solo.trace], percentile, 4e-3 / math.log(wl.slm.vocab))
    ref_logits = []
    models = mk()
    res = stitch.generate(prompt, stitch.decoder_forward(models, sc, ref_logits), tau, n_tok)
    say(f"[cfg3] oracle runs took {time.time() - t0:.0f}s; tau {tau:.5f}; {len(res.trace)} invocations, "
        f"{res.n_rejected} rejected, {res.n_llm_tokens} large-model tokens, "
        f"large-model spans {[len(t.span) for t in res.trace if t.model == 1]}")
    # the trace must exercise what the configuration is about
    assert res.n_rejected >= 2 and 0 < res.n_llm_tokens < n_tok
    assert any(t.model == 1 and not t.hi for t in res.trace), "no hand-back to the small model"
    assert any(t.model == 1 and 3 <= len(t.span) <= 63 for t in res.trace), "no multi-token catch-up"
    assert any(t.model == 0 and len(t.span) >= 2 and t.pos0 > 0 for t in res.trace), "no small-model catch-up"
    gpu = [P.Model(w_s, max_ctx=max_ctx, max_rows=64), P.Model(w_l, max_ctx=max_ctx, max_rows=64)]
    for i, inv in enumerate(res.trace):
        got, lg = gpu[inv.model].forward_span(inv.span, inv.pos0, tau, inv.model, sc(inv.pos0 + len(inv.span)), want_logits=True)
        torch.cuda.synchronize()
        where = f"cfg3 invocation {i} model {inv.model} span {len(inv.span)} at {inv.pos0}"
        if len(inv.span) == 1:
            want = check_invocation(got[0], lg[0], ref_logits[i], tau, inv.model, where=where)
            assert bool(want["flags"] & 2) == inv.accept
        else:
            check_span(gpu[inv.model], models[inv.model], 0, inv.span, inv.pos0, sc(inv.pos0 + len(inv.span)), got[0], lg[0],
                       ref_logits[i], tau, inv.model, where)
        check_and_force_rows(gpu[inv.model], models[inv.model], 0, inv.pos0, len(inv.span), f"cfg3 invocation {i}")
    del gpu, models, w_s, w_l, ws_cpu, wl_cpu
    release()


# ------------------------------------------------------------------------------------------------ cfg4 / cfg5 depth
FULL_DEPTH = [
    # name, shape, seed, cached context, spans
    ("m14_all_48_layers", W.M14, 3, 9216 - 8, [1, 5]),
    ("m32_all_64_layers", W.M32, 4, 10240 - 6, [1, 3]),
]


@pytest.mark.parametrize("name,shape,seed,n_ctx,spans", FULL_DEPTH, ids=[f[0] for f in FULL_DEPTH])
def test_full_depth_large_models_at_full_context(name, shape, seed, n_ctx, spans):
    import paper_2507_17307_amd as P
    t0 = time.time()
    w_gpu = W.make_weights(shape, seed, 1, device="cuda")
    torch.cuda.synchronize()
    w_cpu = w_gpu.to("cpu")
    say(f"[{name}] weights generated and copied to the host in {time.time() - t0:.0f}s")
    max_ctx = n_ctx + sum(spans) + 1
    gpu = P.Model(w_gpu, max_ctx=max_ctx, max_rows=64)
    ref = decoder.OracleModel(w_cpu, max_ctx, keep_fp64_weights=False)
    noise_cache(gpu, ref, 0, n_ctx, seed=12)
    toks = W.rng.randint(13, 5, 0, sum(spans), shape.vocab).tolist()
    pos, tau = n_ctx, 0.5
    for k, span in enumerate(spans):
        chunk, toks = toks[:span], toks[span:]
        scale = 2.0 + 1.5 * k
        t0 = time.time()
        out = ref.forward(chunk, pos, logit_scale=scale)["logits"]
        say(f"[{name}] oracle invocation of {span} rows at {pos}: {time.time() - t0:.0f}s")
        got, lg = gpu.forward_span(chunk, pos, tau, P.RS_LLM, scale, want_logits=True)
        torch.cuda.synchronize()
        err = float((lg[0].cpu().double() - out).abs().max())
        say(f"[{name}] span {span}: logits max-abs error {err:.2e} on logits of magnitude {float(out.abs().max()):.1f}")
        check_invocation(got[0], lg[0], out, tau, router.LLM, where=f"{name} span {span} at {pos}")
        pos += span
    del gpu, ref, w_gpu, w_cpu
    release()


# ------------------------------------------------------------------------------------------------ cfg5 batch of 8
def two_layers(shape):
    return W.ModelShape(shape.name + "_2layers", 2, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                        shape.d_ffn, shape.vocab, shape.tied_lm_head)


BATCH8 = [("s15", W.S15, 0), ("m32", W.M32, 1)]


@pytest.mark.parametrize("name,shape,role", BATCH8, ids=[b[0] for b in BATCH8])
def test_cfg5_eight_sequences_ragged_catchup_and_batched_decode_at_real_layer_shapes(name, shape, role):
    import paper_2507_17307_amd as P
    shape = two_layers(shape)
    max_ctx, n = 10240, 8
    w_gpu = W.make_weights(shape, 4, role, device="cuda")
    ref = decoder.OracleModel(w_gpu.to("cpu"), max_ctx, n_slots=n)
    gpu = P.Model(w_gpu, max_ctx=max_ctx, max_seqs=n, max_rows=64)
    slots = [3, 0, 7, 1, 6, 2, 5, 4]                            # sequence i lives in cache slot slots[i]
    ctx = [700, 9000, 3000, 64, 5000, 10100, 1500, 8000]        # cached positions per sequence, in different context slices
    spans = [5, 33, 1, 1, 3, 2, 1, 7]                           # 53 rows in one call
    for i in range(n):
        noise_cache(gpu, ref, slots[i], ctx[i], seed=40 + i)
    toks = [W.rng.randint(4, 600 + i, 0, spans[i] + 1, shape.vocab).tolist() for i in range(n)]
    scales = [1.0 + 0.5 * i for i in range(n)]
    tau = 0.7
    got, lg = gpu.catchup_prefill([toks[i][:spans[i]] for i in range(n)], ctx, tau, P.RS_LLM, scales, slots, want_logits=True)
    torch.cuda.synchronize()
    for i in range(n):
        want = ref.forward(toks[i][:spans[i]], ctx[i], slot=slots[i], logit_scale=scales[i])["logits"]
        check_invocation(got[i], lg[i], want, tau, router.LLM, where=f"{name} ragged catch-up, sequence {i} ({spans[i]} rows at {ctx[i]})")
    pos = [ctx[i] + spans[i] for i in range(n)]
    nxt = [toks[i][spans[i]] for i in range(n)]
    got, lg = gpu.decode_step(nxt, pos, tau, P.RS_SLM, scales, slots, want_logits=True)
    torch.cuda.synchronize()
    for i in range(n):
        want = ref.forward([nxt[i]], pos[i], slot=slots[i], logit_scale=scales[i])["logits"]
        check_invocation(got[i], lg[i], want, tau, router.SLM, where=f"{name} batched decode, sequence {i} at {pos[i]}")
    # a partial batch (per-sequence routing leaves each model a subset of the sequences): three of them, other slots
    sub = [1, 4, 6]
    pos2 = [pos[i] + 1 for i in sub]
    nxt2 = [W.rng.randint(4, 700 + i, 0, 1, shape.vocab).tolist()[0] for i in sub]
    got, lg = gpu.decode_step(nxt2, pos2, tau, P.RS_LLM, [scales[i] for i in sub], [slots[i] for i in sub], want_logits=True)
    torch.cuda.synchronize()
    for k, i in enumerate(sub):
        want = ref.forward([nxt2[k]], pos2[k], slot=slots[i], logit_scale=scales[i])["logits"]
        check_invocation(got[k], lg[k], want, tau, router.LLM, where=f"{name} partial batch, sequence {i}")
    del gpu, ref, w_gpu
    release()


# ------------------------------------------------------------------------------------------------ batches beyond 16
BIG_BATCH = [("s15_128seqs", W.S15, 0, 128, 40), ("m7_48seqs", W.M7, 1, 48, 20)]


@pytest.mark.parametrize("name,shape,role,n,n_ragged", BIG_BATCH, ids=[b[0] for b in BIG_BATCH])
def test_batches_beyond_sixteen_sequences_at_real_layer_shapes(name, shape, role, n, n_ragged):
    """The batch sizes of the paper's batch-size analysis (Section "Batch Size Analysis": up to 128 sequences) at real
    layer shapes: a ragged catch-up over some of the sequences, then one decode step of all of them (several 16-row
    blocks in the LM head, several 32-row blocks in the layers), each sequence against its own oracle cache."""
    import paper_2507_17307_amd as P
    shape = two_layers(shape)
    max_ctx = 1024
    w_gpu = W.make_weights(shape, 6, role, device="cuda")
    ref = decoder.OracleModel(w_gpu.to("cpu"), max_ctx, n_slots=n)
    gpu = P.Model(w_gpu, max_ctx=max_ctx, max_seqs=n, max_rows=128)
    slots = [(5 * i + 3) % n for i in range(n)]                  # 5 is coprime with 128 and 48
    assert len(set(slots)) == n
    ctx = [40 + (37 * i) % 900 for i in range(n)]
    for i in range(n):
        noise_cache(gpu, ref, slots[i], ctx[i], seed=100 + i)
    spans = [1 + (i * i) % 5 for i in range(n_ragged)]           # 1..5 rows per sequence
    while sum(spans) > 128:
        spans[spans.index(max(spans))] -= 1
    toks = [W.rng.randint(6, 800 + i, 0, 8, shape.vocab).tolist() for i in range(n)]
    scales = [1.0 + 0.5 * (i % 12) for i in range(n)]
    tau = 0.7
    sub = list(range(0, n, n // n_ragged))[:n_ragged]            # the sequences of the ragged call
    got, lg = gpu.catchup_prefill([toks[i][:spans[k]] for k, i in enumerate(sub)], [ctx[i] for i in sub], tau, P.RS_LLM,
                                  [scales[i] for i in sub], [slots[i] for i in sub], want_logits=True)
    torch.cuda.synchronize()
    fed = [0] * n
    for k, i in enumerate(sub):
        want = ref.forward(toks[i][:spans[k]], ctx[i], slot=slots[i], logit_scale=scales[i])["logits"]
        check_invocation(got[k], lg[k], want, tau, router.LLM, where=f"{name} ragged catch-up, sequence {i} ({spans[k]} rows at {ctx[i]})")
        fed[i] = spans[k]
    pos = [ctx[i] + fed[i] for i in range(n)]
    nxt = [toks[i][fed[i]] for i in range(n)]
    got, lg = gpu.decode_step(nxt, pos, tau, P.RS_SLM, scales, slots, want_logits=True)
    torch.cuda.synchronize()
    for i in range(n):
        want = ref.forward([nxt[i]], pos[i], slot=slots[i], logit_scale=scales[i])["logits"]
        check_invocation(got[i], lg[i], want, tau, router.SLM, where=f"{name} decode of {n} sequences, sequence {i} at {pos[i]}")
    del gpu, ref, w_gpu
    release()
