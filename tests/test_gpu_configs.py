"""GPU parity at the REAL shapes of configurations 2-5, element by element against the oracle, through the C ABI.

  * cfg2: the whole 28-layer 1.5B shape; the model itself prefills a prompt, then 16 consecutive decode steps are
    checked one by one (the oracle's tokens are teacher-forced), and the K/V rows both sides wrote are compared;
  * cfg3: a stitched prefix on the whole 1.5B + 7B pair: the oracle runs Algorithm 1 (entropy threshold from its
    own small-model-only run), the GPU replays every invocation of that trace - small-model steps, rejected
    steps, large-model catch-up prefills of several tokens, hand-backs - and is compared per invocation;
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


def assert_caches_agree(gpu, ref, n, where):
    """K/V rows 0..n-1 of slot 0: bf16 roundings of nearly equal fp32 values (a value may flip by one bf16 step)."""
    for name, cache in (("k", ref.k_cache), ("v", ref.v_cache)):
        g = gpu.kv_view(name)[:, 0, :, :n].float().cpu().double()
        r = cache[:, 0, :, :n]
        err = float((g - r).abs().max())
        assert err <= 2 ** -7 * float(r.abs().max()) + 1e-6, f"{where}: {name} cache differs by {err}"
        # and almost every element is identical
        assert float((g != r).double().mean()) < 2e-2, f"{where}: too many {name} elements differ"


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
    check_invocation(got[0], lg[0], want, tau, router.SLM, where="cfg2 prompt prefill")
    tok = router.greedy_token(want)
    for i in range(n_steps):
        pos = n_prompt + i
        want = ref.forward([tok], pos, logit_scale=float(scales[pos + 1]))["logits"]
        got, lg = gpu.forward_span([tok], pos, tau, P.RS_SLM, float(scales[pos + 1]), want_logits=True)
        torch.cuda.synchronize()
        check_invocation(got[0], lg[0], want, tau, router.SLM, where=f"cfg2 decode step {i} at {pos}")
        tok = router.greedy_token(want)               # teacher forcing: the oracle's token goes to both sides
    assert_caches_agree(gpu, ref, n_prompt + n_steps, "cfg2")
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
        want = check_invocation(got[0], lg[0], ref_logits[i], tau, inv.model,
                                where=f"cfg3 invocation {i} model {inv.model} span {len(inv.span)} at {inv.pos0}")
        assert bool(want["flags"] & 2) == inv.accept
    n = n_prompt + n_tok - 1
    for m in (0, 1):
        held = max(t.pos0 + len(t.span) for t in res.trace if t.model == m)      # rows this model has written
        assert_caches_agree(gpu[m], models[m], min(n, held), f"cfg3 model {m}")
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
