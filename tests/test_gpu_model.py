"""GPU parity of rs_decode_step / rs_catchup_prefill against the oracle, through the C ABI.

The oracle's token sequence and routing decisions are teacher-forced: the GPU replays the
oracle's invocations and its outputs are never fed forward.
"""
import math

import pytest
import torch

import workloads as W
from oracle import decoder, router, stitch
from workloads.recipes import misc_normal
import parity
from parity import check_invocation

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["kernel_per_phase", "single_kernel_step"])
def decode_path(request, monkeypatch):
    """Tests that take this fixture run twice: single-row steps as one kernel per phase (the default) and as one
    experimental persistent kernel with grid-wide waits (RSTITCH_DECODE=persistent, read when a model is
    created).  The full-size cases run the default path only."""
    if request.param == "single_kernel_step":
        monkeypatch.setenv("RSTITCH_DECODE", "persistent")
    else:
        monkeypatch.delenv("RSTITCH_DECODE", raising=False)
    return request.param


def pair_run(wl, n_tokens=None):
    """Oracle run of a stitched workload; returns weights, trace, logits per invocation, tau, scales."""
    ws, wl_ = W.make_weights(wl.slm, wl.seed, 0), W.make_weights(wl.llm, wl.seed, 1)
    prompt = W.make_prompt(wl).tolist()
    n = wl.n_decode if n_tokens is None else n_tokens
    scales = W.logit_scale(wl, 0, wl.max_ctx + 1)
    mk = lambda: [decoder.OracleModel(ws, wl.max_ctx + 1), decoder.OracleModel(wl_, wl.max_ctx + 1)]  # noqa: E731
    sc = lambda p: float(scales[p])  # noqa: E731
    hs = [t.h_norm for t in stitch.generate(prompt, stitch.decoder_forward(mk(), sc), 2.0, n).trace]
    tau = W.pick_tau(hs, wl.tau_percentile, 4e-3 / math.log(wl.slm.vocab))
    log = []
    models = mk()
    res = stitch.generate(prompt, stitch.decoder_forward(models, sc, log), tau, n)
    return (ws, wl_), models, res, log, tau, scales


def test_config1_tiny_pair_teacher_forced(decode_path):
    import paper_2507_17307_amd as P
    wl = W.WORKLOADS["cfg1_tiny_pair"]
    weights, oracle_models, res, ref_logits, tau, scales = pair_run(wl)
    assert 0 < res.n_llm_tokens < wl.n_decode and res.n_rejected > 0
    gpu = [P.Model(w.to("cuda"), max_ctx=wl.max_ctx + 1, max_rows=64) for w in weights]
    for i, inv in enumerate(res.trace):
        got, lg = gpu[inv.model].forward_span(inv.span, inv.pos0, tau, inv.model,
                                              float(scales[inv.pos0 + len(inv.span)]), want_logits=True)
        torch.cuda.synchronize()
        want = check_invocation(got[0], lg[0], ref_logits[i], tau, inv.model, where=f"invocation {i} {inv.model} span {len(inv.span)}")
        assert bool(want["flags"] & 2) == inv.accept
    # the caches the two sides built agree to bf16 rounding of nearly equal fp32 values
    for m in (0, 1):
        n = len(W.make_prompt(wl)) + wl.n_decode - 1
        for name, ref in (("k", oracle_models[m].k_cache), ("v", oracle_models[m].v_cache)):
            g = gpu[m].kv_view(name)[:, 0, :, :n].float().cpu().double()
            r = ref[:, 0, :, :n]
            assert float((g - r).abs().max()) <= 2 ** -7 * float(r.abs().max()) + 1e-6


def test_catchup_equals_sequential_decode_on_gpu(decode_path):
    import paper_2507_17307_amd as P
    w = W.make_weights(W.TINY_L, 3, 1).to("cuda")
    toks = W.rng.randint(3, 77, 0, 40, 1024).tolist()
    a, b = P.Model(w, 64), P.Model(w, 64)
    ra, la = a.forward_span(toks[:23], 0, 0.5, P.RS_LLM, 2.0, want_logits=True)
    ra, la = a.forward_span(toks[23:], 23, 0.5, P.RS_LLM, 2.0, want_logits=True)
    for i, t in enumerate(toks):
        rb, lb = b.forward_span([t], i, 0.5, P.RS_LLM, 2.0, want_logits=True)
    torch.cuda.synchronize()
    assert float((la - lb).abs().max()) <= 2e-2
    assert abs(ra[0].h_nats - rb[0].h_nats) <= 1e-3 and ra[0].token == rb[0].token
    ka, kb = a.kv_view("k").float(), b.kv_view("k").float()
    assert float((ka - kb).abs().max()) <= 2 ** -7 * float(ka.abs().max())


@pytest.mark.parametrize("spans", [[1, 1, 1], [3, 1, 17, 2], [16, 16, 16, 16], [5, 33, 1, 1, 1, 1, 1, 2],
                                   [1] * 16, [2, 1, 7, 1, 1, 3, 1, 1, 9, 1, 1, 2, 1, 5, 1, 4],
                                   [1] * 17, [64, 64], [1, 2, 5, 1, 1, 3, 1, 9, 1, 1] * 4, [1] * 128, [1, 3] * 32],
                         ids=lambda s: f"{len(s)}seqs_{sum(s)}rows")
def test_batched_ragged_calls_match_per_sequence_oracle(spans, decode_path):
    """Several sequences in one call (ragged spans, distinct slots) against one oracle model per slot."""
    import paper_2507_17307_amd as P
    shape = W.TINY_L
    w = W.make_weights(shape, 4, 1)
    n = len(spans)
    n_slots = next(k for k in (8, 16, 32, 64, 128) if k >= n)
    gpu = P.Model(w.to("cuda"), max_ctx=96, max_seqs=n_slots, max_rows=64 if sum(spans) <= 64 else 128)
    refs = [decoder.OracleModel(w, 96) for _ in range(n)]
    slots = [(3 * i + 1) % n_slots for i in range(n)]
    pre = [7 + (5 * i) % 61 for i in range(n)]                # every sequence already holds a different prefix
    toks = [W.rng.randint(4, 200 + i, 0, pre[i] + spans[i] + 1, shape.vocab).tolist() for i in range(n)]
    for i in range(n):
        refs[i].forward(toks[i][:pre[i]], 0)
        gpu.forward_span(toks[i][:pre[i]], 0, 0.5, P.RS_LLM, slot=slots[i])
    scales = [1.0 + i % 16 for i in range(n)]                 # scaled logits stay of the magnitude the tolerance is stated for
    got, lg = gpu.catchup_prefill([toks[i][pre[i]:pre[i] + spans[i]] for i in range(n)], pre, 0.7, P.RS_LLM,
                                  scales, slots, want_logits=True)
    torch.cuda.synchronize()
    for i in range(n):
        ref = refs[i].forward(toks[i][pre[i]:pre[i] + spans[i]], pre[i], logit_scale=scales[i])["logits"]
        check_invocation(got[i], lg[i], ref, 0.7, router.LLM, where=f"seq {i}")
    # then one batched decode step for all of them
    nxt = [toks[i][pre[i] + spans[i]] for i in range(n)]
    pos = [pre[i] + spans[i] for i in range(n)]
    got, lg = gpu.decode_step(nxt, pos, 0.7, P.RS_SLM, scales, slots, want_logits=True)
    torch.cuda.synchronize()
    for i in range(n):
        ref = refs[i].forward([nxt[i]], pos[i], logit_scale=scales[i])["logits"]
        check_invocation(got[i], lg[i], ref, 0.7, router.SLM, where=f"decode seq {i}")


TILE_CASES = [("one_span_17", [17]), ("one_span_24", [24]), ("two_spans_31", [11, 20]), ("decode_32", [1] * 32), ("one_span_33", [33]), ("one_span_64", [64]), ("one_span_100", [100]), ("two_spans_128", [59, 69]),
              ("ragged_20_seqs_90_rows", [1, 9, 2, 7, 3, 8, 4, 6, 5, 5, 1, 9, 2, 7, 3, 8, 4, 2, 3, 1]), ("decode_128", [1] * 128)]


@pytest.mark.parametrize("name,spans", TILE_CASES, ids=[c[0] for c in TILE_CASES])
def test_calls_of_17_to_128_rows_on_a_2048_wide_shape_match_the_oracle(name, spans):
    """Calls of more than 16 rows take the kernel in which one workgroup holds all rows of the call against a block of
    output columns (up to 32 rows: two waves per 16-row block, each with half of the column tiles; up to 64: four waves of 16
    rows; above: eight; K split over workgroups for QKV / O-proj / down) for every matrix whose workgroups fill the machine: here QKV (192 tiles), gate/up (640 tiles in
    groups of three: a ragged last group) and down (128 tiles, 160 k windows split over eight workgroups); the O projection
    (128 tiles, 32 windows) stays on the 32-row-block kernel, so both activation formats are in play in one call."""
    import paper_2507_17307_amd as P
    from workloads.shapes import ModelShape
    shape = ModelShape("wide_2layers", 2, 2048, 16, 4, 128, 10240, 8192, tied_lm_head=False)
    w = W.make_weights(shape, 31, 1)
    n = len(spans)
    n_slots = next(k for k in (2, 32, 128) if k >= n)
    max_ctx = 160
    gpu = P.Model(w.to("cuda"), max_ctx=max_ctx, max_seqs=n_slots, max_rows=128)
    ref = decoder.OracleModel(w, max_ctx, n_slots=n_slots)
    slots = [(7 * i + 3) % n_slots for i in range(n)]
    pre = [5 + (11 * i) % 23 for i in range(n)]
    toks = [W.rng.randint(31, 400 + i, 0, pre[i] + spans[i] + 1, shape.vocab).tolist() for i in range(n)]
    for i in range(n):
        ref.forward(toks[i][:pre[i]], 0, slot=slots[i])
        gpu.forward_span(toks[i][:pre[i]], 0, 0.5, P.RS_LLM, slot=slots[i])
    scales = [1.0 + 0.5 * (i % 10) for i in range(n)]
    if all(sp == 1 for sp in spans):
        got, lg = gpu.decode_step([toks[i][pre[i]] for i in range(n)], pre, 0.7, P.RS_LLM, scales, slots, want_logits=True)
    else:
        got, lg = gpu.catchup_prefill([toks[i][pre[i]:pre[i] + spans[i]] for i in range(n)], pre, 0.7, P.RS_LLM,
                                      scales, slots, want_logits=True)
    torch.cuda.synchronize()
    for i in range(n):
        want = ref.forward(toks[i][pre[i]:pre[i] + spans[i]], pre[i], slot=slots[i], logit_scale=scales[i])["logits"]
        check_invocation(got[i], lg[i], want, 0.7, router.LLM, where=f"{name} sequence {i} ({spans[i]} rows at {pre[i]})")
    # the K/V rows the call wrote, every layer: they are what later calls read
    kg, vg = gpu.kv_view("k").float().cpu().double(), gpu.kv_view("v").float().cpu().double()
    for i in range(n):
        sl, lo, hi = slots[i], pre[i], pre[i] + spans[i]
        for got_c, want_c, what in ((kg, ref.k_cache, "k"), (vg, ref.v_cache, "v")):
            g_rows, w_rows = got_c[:, sl, :, lo:hi], want_c[:, sl, :, lo:hi]
            err = float((g_rows - w_rows).abs().max())
            assert err <= 2.0 ** -7 * float(w_rows.abs().max()) + 1e-6, f"{name}: {what} rows of sequence {i} differ by {err}"


@pytest.mark.parametrize("rows", [40, 100])
def test_long_spans_on_the_narrowest_shape(rows):
    """The tiny small-model shape (d_model 128: two 64-element k windows, fewer than the kernel keeps in flight; d_ffn 384)
    with spans that take the all-rows-per-workgroup kernel: every request past the last window is a clamped duplicate."""
    import paper_2507_17307_amd as P
    shape = W.TINY_S
    w = W.make_weights(shape, 23, 0)
    gpu = P.Model(w.to("cuda"), max_ctx=128, max_seqs=1, max_rows=128)
    ref = decoder.OracleModel(w, 128)
    toks = W.rng.randint(23, 9, 0, rows + 12, shape.vocab).tolist()
    ref.forward(toks[:11], 0)
    gpu.forward_span(toks[:11], 0, 0.5, P.RS_SLM)
    got, lg = gpu.catchup_prefill([toks[11:11 + rows]], [11], 0.6, P.RS_SLM, [3.0], [0], want_logits=True)
    torch.cuda.synchronize()
    want = ref.forward(toks[11:11 + rows], 11, logit_scale=3.0)["logits"]
    check_invocation(got[0], lg[0], want, 0.6, router.SLM, where=f"{rows} rows")
    kg = gpu.kv_view("k").float().cpu().double()[:, 0, :, 11:11 + rows]
    kw = ref.k_cache[:, 0, :, 11:11 + rows]
    assert float((kg - kw).abs().max()) <= 2.0 ** -7 * float(kw.abs().max()) + 1e-6


def test_many_sequences_with_a_vocabulary_that_is_not_a_multiple_of_the_tile_width():
    """40 sequences in one decode step on a model with 1003 vocabulary entries: the last block of vocabulary columns of
    the LM head is ragged (62 full tiles of 16 and one of 11), and so is the last group of column tiles."""
    import paper_2507_17307_amd as P
    from workloads.shapes import ModelShape
    shape = ModelShape("ragged_vocab", 2, 256, 4, 2, 64, 512, 1003, tied_lm_head=True)
    w = W.make_weights(shape, 17, 0)
    n = 40
    gpu = P.Model(w.to("cuda"), max_ctx=16, max_seqs=64, max_rows=64)
    ref = decoder.OracleModel(w, 16, n_slots=64)
    slots = [(3 * i + 1) % 64 for i in range(n)]
    toks = W.rng.randint(17, 5, 0, 2 * n, shape.vocab).tolist()
    for i in range(n):
        ref.forward([toks[2 * i]], 0, slot=slots[i])
        gpu.forward_span([toks[2 * i]], 0, 0.5, P.RS_SLM, slot=slots[i])
    scales = [1.0 + i % 9 for i in range(n)]
    got, lg = gpu.decode_step([toks[2 * i + 1] for i in range(n)], [1] * n, 0.5, P.RS_SLM, scales, slots, want_logits=True)
    torch.cuda.synchronize()
    for i in range(n):
        want = ref.forward([toks[2 * i + 1]], 1, slot=slots[i], logit_scale=scales[i])["logits"]
        check_invocation(got[i], lg[i], want, 0.5, router.SLM, where=f"sequence {i}")


def test_batched_decode_over_large_caches_matches_per_sequence_oracle():
    """Three sequences, one token each, on a model whose caches (three slots of 2 KV heads x 2048 positions x
    128 channels) are large enough that the single-row attention kernel waits for each row's position before it
    requests K and V: the rows of a batched step go through that variant side by side."""
    import paper_2507_17307_amd as P
    from workloads.shapes import ModelShape
    shape = ModelShape("batched_large_cache", 2, 256, 4, 2, 128, 512, 1024, tied_lm_head=False)
    w = W.make_weights(shape, 21, 1)
    n, max_ctx = 3, 2048
    gpu = P.Model(w.to("cuda"), max_ctx=max_ctx, max_seqs=4, max_rows=64)
    refs = [decoder.OracleModel(w, max_ctx) for _ in range(n)]
    slots = [2, 0, 3]
    pre = [130, 61, 200]                                      # prefixes that end in different context slices
    toks = [W.rng.randint(21, 300 + i, 0, pre[i] + 3, shape.vocab).tolist() for i in range(n)]
    for i in range(n):
        refs[i].forward(toks[i][:pre[i]], 0)
        for c0 in range(0, pre[i], 64):
            gpu.forward_span(toks[i][c0:min(c0 + 64, pre[i])], c0, 0.5, P.RS_LLM, slot=slots[i])
    scales = [1.5, 2.5, 4.0]
    for step in range(2):
        nxt = [toks[i][pre[i] + step] for i in range(n)]
        pos = [pre[i] + step for i in range(n)]
        got, lg = gpu.decode_step(nxt, pos, 0.6, P.RS_SLM, scales, slots, want_logits=True)
        torch.cuda.synchronize()
        for i in range(n):
            ref = refs[i].forward([nxt[i]], pos[i], logit_scale=scales[i])["logits"]
            check_invocation(got[i], lg[i], ref, 0.6, router.SLM, where=f"step {step} seq {i}")


def test_device_side_argument_errors_are_flagged_not_faulted(decode_path):
    import paper_2507_17307_amd as P
    w = W.make_weights(W.TINY_S, 5, 0).to("cuda")
    m = P.Model(w, max_ctx=16, max_seqs=2, max_rows=8)
    ok = m.decode_step([3], [0], 0.5, P.RS_SLM)
    assert not ok[0].flags & P.FLAG_BADARG
    assert m.decode_step([3], [16], 0.5, P.RS_SLM)[0].flags & P.FLAG_BADARG          # position beyond the cache
    assert m.decode_step([3], [-1], 0.5, P.RS_SLM)[0].flags & P.FLAG_BADARG
    assert m.decode_step([1024], [1], 0.5, P.RS_SLM)[0].flags & P.FLAG_BADARG        # token out of vocabulary
    assert m.decode_step([3], [1], 0.5, P.RS_SLM, slots=[2])[0].flags & P.FLAG_BADARG  # slot out of range
    r = m.decode_step([3, 4], [1, 1], 0.5, P.RS_SLM, slots=[1, 1])                    # duplicate slots
    assert r[0].flags & P.FLAG_BADARG and r[1].flags & P.FLAG_BADARG
    r = m.catchup_prefill([[1, 2, 3]], [14], 0.5, P.RS_SLM)                           # span runs past max_ctx
    assert r[0].flags & P.FLAG_BADARG
    r = m.catchup_prefill([[1, 2, 3], [4]], [0, 0], 0.5, P.RS_SLM)                    # one good, one good
    assert not (r[0].flags | r[1].flags) & P.FLAG_BADARG
    with pytest.raises(P.RsError):
        m.catchup_prefill([[1] * 9], [0], 0.5, P.RS_SLM)                               # more rows than max_rows
    with pytest.raises(P.RsError):
        m.decode_step([1, 2, 3], [0, 0, 0], 0.5, P.RS_SLM)                             # more sequences than max_seqs
    torch.cuda.synchronize()


def synthetic_cache(gpu, ref, n_ctx, seed):
    """Fill positions [0, n_ctx) of slot 0 of both caches with the same bf16 noise."""
    c = gpu.cfg
    shape = (c.n_layers, c.n_kv_heads, n_ctx, c.head_dim)
    cnt = c.n_layers * c.n_kv_heads * n_ctx * c.head_dim
    for which, tag in (("k", 1), ("v", 2)):
        vals = torch.empty(cnt, dtype=torch.bfloat16)
        step = 1 << 22
        for s in range(0, cnt, step):
            vals[s:s + step] = W.rng.normal(seed, 900 + tag, s, min(step, cnt - s)).to(torch.float32).to(torch.bfloat16)
        vals = vals.view(shape)
        gpu.kv_view(which)[:, 0, :, :n_ctx] = vals.cuda()
        cache = ref.k_cache if which == "k" else ref.v_cache
        cache[:, 0, :, :n_ctx] = vals.double()


FULL_SHAPES = [
    # (shape, layers kept, context already cached, spans to run)
    ("s15", W.S15, 28, 2559 - 8, [1, 7]),
    ("m7", W.M7, 28, 4607 - 40, [1, 2, 37]),
    ("m14_4layers", W.ModelShape("m14_4", 4, 5120, 40, 8, 128, 13824, 152064, False), 4, 9215 - 20, [1, 19]),
    ("m32_2layers", W.ModelShape("m32_2", 2, 5120, 40, 8, 128, 27648, 152064, False), 2, 10239 - 70, [1, 64, 5]),
    # a cache longer than 192 slices of 64 positions: every context slice is two passes
    ("long_cache_small_model", W.ModelShape("long_cache", 2, 512, 4, 2, 128, 768, 2048, False), 2, 13000, [1, 5, 1]),
]


@pytest.mark.parametrize("name,shape,n_layers,n_ctx,spans", FULL_SHAPES, ids=[f[0] for f in FULL_SHAPES])
def test_full_size_shapes_at_full_context(name, shape, n_layers, n_ctx, spans):
    """Full layer dimensions, vocabulary and context length of configs 2-5.  The KV cache is
    pre-filled with seeded noise on both sides (the oracle cannot afford a 4k-10k token prefill),
    then decode steps and catch-up spans run on top of it."""
    import paper_2507_17307_amd as P
    w_gpu = W.make_weights(shape, seed=11, role=1, device="cuda")
    w_cpu = w_gpu.to("cpu")
    max_ctx = n_ctx + sum(spans) + 1
    gpu = P.Model(w_gpu, max_ctx=max_ctx, max_rows=64)
    ref = decoder.OracleModel(w_cpu, max_ctx, keep_fp64_weights=(shape.d_model <= 1536))
    synthetic_cache(gpu, ref, n_ctx, seed=12)
    toks = W.rng.randint(13, 5, 0, sum(spans), shape.vocab).tolist()
    pos, tau = n_ctx, 0.5
    for k, span in enumerate(spans):
        chunk, toks = toks[:span], toks[span:]
        scale = 2.0 + 1.5 * k
        out = ref.forward(chunk, pos, logit_scale=scale)["logits"]
        got, lg = gpu.forward_span(chunk, pos, tau, P.RS_LLM, scale, want_logits=True)
        torch.cuda.synchronize()
        check_invocation(got[0], lg[0], out, tau, router.LLM, where=f"{name} span {span} at {pos}")
        pos += span


def test_bounded_wait_gives_up_instead_of_hanging(decode_path):
    """A spin limit of one poll makes the first grid-wide wait of the single-kernel step give up:
    the step must end, flag its record, and the model must refuse further steps; a fresh model works."""
    import paper_2507_17307_amd as P
    if decode_path != "single_kernel_step":
        pytest.skip("only the single-kernel step has grid-wide waits")
    w = W.make_weights(W.TINY_S, 5, 0).to("cuda")
    m = P.Model(w, max_ctx=16)
    good = m.decode_step([3], [0], 0.5, P.RS_SLM)[0]
    assert not good.flags & P.FLAG_ABORTED
    P.rs_set_spin_limit(m.handle, 1)
    r = m.decode_step([4], [1], 0.5, P.RS_SLM)[0]
    torch.cuda.synchronize()
    assert r.flags & P.FLAG_ABORTED and r.token == -1
    P.rs_set_spin_limit(m.handle, 0)
    assert m.decode_step([4], [1], 0.5, P.RS_SLM)[0].flags & P.FLAG_ABORTED      # sticky
    m2 = P.Model(w, max_ctx=16)
    again = m2.decode_step([3], [0], 0.5, P.RS_SLM)[0]
    assert again.token == good.token and abs(again.h_nats - good.h_nats) < 1e-6


def test_live_stitched_run_through_the_host_driver_matches_the_oracle_run(decode_path):
    """Algorithm 1 run LIVE on the GPU by the package's own host driver (fixed staging buffers, so the
    library replays launch graphs from the second step on) against the oracle's run of config 1:
    same accepted tokens, same model per invocation, same spans, entropies within tolerance."""
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedPair
    wl = W.WORKLOADS["cfg1_tiny_pair"]
    weights, _, res, ref_logits, tau, scales = pair_run(wl)
    gpu = [P.Model(w.to("cuda"), max_ctx=wl.max_ctx + 1, max_rows=64) for w in weights]
    pair = StitchedPair(gpu[0], gpu[1], wl.max_ctx, scales)
    run = pair.generate(W.make_prompt(wl).tolist(), tau, wl.n_decode)
    assert run.output == res.output
    assert [(t.model, t.pos0, t.n_rows, t.accept) for t in run.trace] == \
           [(t.model, t.pos0, len(t.span), t.accept) for t in res.trace]
    assert max(abs(a.h_norm - b.h_norm) for a, b in zip(run.trace, res.trace)) <= 1e-3 / math.log(1024)
    # and again on the same pair: the caches are overwritten with identical values, graphs are replayed
    again = pair.generate(W.make_prompt(wl).tolist(), tau, wl.n_decode)
    assert again.output == run.output and [t.flags for t in again.trace] == [t.flags for t in run.trace]


def test_random_routing_baseline_run_matches_the_oracle_run():
    """The random-routing baseline (each token assigned to the small model with probability p) live on the GPU
    against the oracle's run of it on config 1: same model, first position and span per invocation, same tokens,
    entropies within tolerance."""
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedPair
    wl = W.WORKLOADS["cfg1_tiny_pair"]
    ws, wl_ = W.make_weights(wl.slm, wl.seed, 0), W.make_weights(wl.llm, wl.seed, 1)
    prompt = W.make_prompt(wl).tolist()
    scales = W.logit_scale(wl, 0, wl.max_ctx + 2)
    u = W.uniform01(wl.seed, 4242, 0, wl.max_ctx + 2).tolist()
    models = [decoder.OracleModel(ws, wl.max_ctx + 1), decoder.OracleModel(wl_, wl.max_ctx + 1)]
    res = stitch.generate_random(prompt, stitch.decoder_forward(models, lambda p: float(scales[p])), 0.7, lambda t: u[t], wl.n_decode)
    n_llm = sum(1 for t in res.trace if t.model == 1)
    assert 5 < n_llm < wl.n_decode - 5 and any(len(t.span) > 2 and t.pos0 > 0 for t in res.trace)
    gpu = [P.Model(x.to("cuda"), max_ctx=wl.max_ctx + 1, max_rows=64) for x in (ws, wl_)]
    run = StitchedPair(gpu[0], gpu[1], wl.max_ctx, scales).generate_random(prompt, 0.7, u, wl.n_decode)
    assert run.output == res.output
    assert [(t.model, t.pos0, t.n_rows) for t in run.trace] == [(t.model, t.pos0, len(t.span)) for t in res.trace]
    assert max(abs(a.h_norm - b.h_norm) for a, b in zip(run.trace, res.trace)) <= 1e-3 / math.log(1024)


def test_batched_stitched_run_with_per_sequence_routing_matches_per_sequence_oracle_runs(decode_path):
    """Four sequences with different prompt lengths share the two tiny models (one KV slot each) and are
    routed independently by the batched host driver; each must reproduce the oracle's single-sequence
    Algorithm 1 run on its own prompt and logit-scale schedule: same tokens, same model / first position /
    span / acceptance per invocation, entropies within tolerance."""
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedBatch
    wl = W.WORKLOADS["cfg1_tiny_pair"]
    ws, wl_ = W.make_weights(wl.slm, wl.seed, 0), W.make_weights(wl.llm, wl.seed, 1)
    lens, n_tok = [20, 32, 7, 45], 24
    max_ctx = max(lens) + n_tok + 3
    prompts = [W.make_prompt(wl, seq=b, length=n).tolist() for b, n in enumerate(lens)]
    scales = [W.logit_scale(wl, 0, max_ctx + 1, seq=b) for b in range(len(lens))]
    mk = lambda: [decoder.OracleModel(ws, max_ctx + 1), decoder.OracleModel(wl_, max_ctx + 1)]  # noqa: E731
    hs = []
    for b in range(len(lens)):
        sc = lambda p, b=b: float(scales[b][p])  # noqa: E731
        hs += [t.h_norm for t in stitch.generate(prompts[b], stitch.decoder_forward(mk(), sc), 2.0, n_tok).trace]
    tau = W.pick_tau(hs, 60.0, 4e-3 / math.log(wl.slm.vocab))
    ref = []
    for b in range(len(lens)):
        sc = lambda p, b=b: float(scales[b][p])  # noqa: E731
        ref.append(stitch.generate(prompts[b], stitch.decoder_forward(mk(), sc), tau, n_tok))
    gpu = [P.Model(w.to("cuda"), max_ctx=max_ctx + 1, max_seqs=4, max_rows=64) for w in (ws, wl_)]
    batch = StitchedBatch(gpu[0], gpu[1], max_ctx, scales)
    runs = batch.generate(prompts, tau, n_tok)
    assert any(t.model == 1 for r in ref for t in r.trace) and any(not t.accept for r in ref for t in r.trace)
    for b, (run, res) in enumerate(zip(runs, ref)):
        assert run.output == res.output, f"sequence {b}"
        assert [(t.model, t.pos0, t.n_rows, t.accept) for t in run.trace] == \
               [(t.model, t.pos0, len(t.span), t.accept) for t in res.trace], f"sequence {b}"
        assert max(abs(x.h_norm - y.h_norm) for x, y in zip(run.trace, res.trace)) <= 1e-3 / math.log(1024)
    # fewer library calls than the four sequences would need one by one
    assert batch.calls < sum(len(r.trace) for r in ref)


def test_full_1p5b_model_self_consistency_at_bench_configuration(monkeypatch):
    """The whole 28-layer 1.5B-shape model (too large for an oracle run) in the configuration bench.py times
    (fixed staging buffers, launch-graph replay): properties that hold at any size.
      * replayed launch graphs and plain launches give bit-identical records, step by step;
      * a catch-up call over k tokens equals k single-token steps: logits, entropy, argmax, cache rows;
      * 0 <= H <= ln V, tokens in range, flags consistent with Eq. 2 for the tau in use."""
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedPair, SLM
    wl = W.WORKLOADS["cfg2_s15_decode"]
    w = W.make_weights(wl.slm, wl.seed, 0, device="cuda")
    n_prompt, n_dec, max_ctx = 160, 24, 256
    prompt = W.make_prompt(wl, length=n_prompt).tolist()
    scales = W.logit_scale(wl, 0, max_ctx + 1)
    monkeypatch.setenv("RSTITCH_GRAPHS", "0")
    plain = P.Model(w, max_ctx=max_ctx, max_rows=64)
    monkeypatch.delenv("RSTITCH_GRAPHS")
    graphs = P.Model(w, max_ctx=max_ctx, max_rows=64)
    tau = 0.8
    runs = []
    for mdl in (plain, graphs):
        pair = StitchedPair(mdl, None, max_ctx, scales)
        runs.append(pair.generate(prompt, tau, n_dec, single_model=SLM))
    a, b = runs
    assert a.output == b.output
    assert [(t.flags, t.h_norm) for t in a.trace] == [(t.flags, t.h_norm) for t in b.trace]      # bit-identical
    ln_v = math.log(wl.slm.vocab)
    for t in a.trace:
        assert 0 <= t.token < wl.slm.vocab and 0.0 <= t.h_norm <= 1.0 + 1e-6
        hi = bool(t.flags & P.binding.FLAG_HI)
        assert hi == (t.h_norm > tau) and bool(t.flags & P.binding.FLAG_ACCEPT) == (not hi)      # the small model rejects iff hi
    # catch-up of the last 9 positions on one model against single-token steps on the other (both caches hold 0..end)
    seq = prompt + a.output
    end = len(seq) - 1
    r_c, l_c = graphs.forward_span(seq[end - 9:end], end - 9, tau, P.RS_SLM, float(scales[end]), want_logits=True)
    for i in range(end - 9, end):
        r_s, l_s = plain.forward_span([seq[i]], i, tau, P.RS_SLM, float(scales[end]), want_logits=True)
    torch.cuda.synchronize()
    assert float((l_c - l_s).abs().max()) <= parity.LOGIT_TOL
    assert abs(r_c[0].h_nats - r_s[0].h_nats) <= parity.ENTROPY_TOL
    top2 = torch.topk(l_s[0], 2).values
    assert r_c[0].token == r_s[0].token or float(top2[0] - top2[1]) < parity.ARGMAX_GAP
    assert r_c[0].h_nats <= ln_v + 1e-3
    ka, kb = graphs.kv_view("k")[:, 0, :, end - 9:end].float(), plain.kv_view("k")[:, 0, :, end - 9:end].float()
    assert float((ka - kb).abs().max()) <= 2 ** -7 * float(kb.abs().max())


def test_counter_run_driver_runs_decode_and_catchup_calls():
    """The stand-alone driver used for hardware-counter runs (no framework in the process) links against the
    library, builds a two-layer 1.5B-shape model and finishes decode steps and a 5-row catch-up with a sane record."""
    import os
    import subprocess
    import paper_2507_17307_amd as P
    probe = os.path.join(os.path.dirname(os.path.abspath(P.__file__)), "traffic_probe")
    assert os.path.exists(probe), "build the package first (paper_2507_17307_amd.build)"
    # the driver always runs one kernel per phase: a second process cannot take the device's cooperative-launch
    # queue while this one holds it
    env = {k: v for k, v in os.environ.items() if k != "RSTITCH_DECODE"}
    for extra in ([], ["5"]):
        r = subprocess.run([probe, "s15", "2", "2", "300"] + extra, capture_output=True, text=True, timeout=120, env=env)
        assert r.returncode == 0, r.stderr
        assert "traffic_probe s15 layers=2 steps=2 position=300" in r.stdout and "h_norm" in r.stdout


ODD_SHAPES = [
    # name, layers, d, n_q, n_kv, head_dim, ffn, vocab: head_dim 64 and the extreme group sizes
    ("mha_hd64", 2, 256, 4, 4, 64, 512, 2048),          # G = 1: sixteen rows share one matrix-core pass
    ("g8_hd64", 2, 512, 8, 1, 64, 640, 1536),           # G = 8: two rows per pass, one KV head
    ("g3_hd128", 1, 384, 3, 1, 128, 384, 1280),         # G = 3: five rows per pass, one column unused
]


@pytest.mark.parametrize("name,n_layers,d,n_q,n_kv,hd,ffn,vocab", ODD_SHAPES, ids=[s[0] for s in ODD_SHAPES])
def test_other_head_shapes_decode_and_catchup_against_oracle(name, n_layers, d, n_q, n_kv, hd, ffn, vocab, decode_path):
    """Head sizes and group sizes the five configurations do not use (head_dim 64, G = 1, 3, 8): a prompt fed as
    catch-up calls, single-token steps, a ragged two-sequence call and a 40-row span, each against the oracle."""
    import paper_2507_17307_amd as P
    from workloads.shapes import ModelShape
    shape = ModelShape(name, n_layers, d, n_q, n_kv, hd, ffn, vocab, tied_lm_head=False)
    w = W.make_weights(shape, 11, 1)
    max_ctx = 200
    ref = decoder.OracleModel(w, max_ctx, n_slots=2)
    gpu = P.Model(w.to("cuda"), max_ctx=max_ctx, max_seqs=2, max_rows=64)
    toks = W.rng.randint(11, 5, 0, 160, vocab).tolist()
    tau = 0.6

    def both(span, pos0, slot, scale):
        lr = ref.forward(span, pos0, slot=slot, logit_scale=scale)["logits"]
        got, lg = gpu.forward_span(span, pos0, tau, P.RS_LLM, scale, slot=slot, want_logits=True)
        torch.cuda.synchronize()
        check_invocation(got[0], lg[0], lr, tau, P.RS_LLM, where=f"{name} span {len(span)} at {pos0} slot {slot}")

    both(toks[:70], 0, 0, 3.0)                 # 64 + 6 rows
    for i in range(70, 73):
        both([toks[i]], i, 0, 1.0 + i % 3)
    both(toks[73:113], 73, 0, 5.0)             # 40 rows crossing a context-slice boundary
    both(toks[:9], 0, 1, 2.0)                  # second slot
    # ragged call over both slots at once
    spans, pos0 = [toks[113:116], toks[9:26]], [113, 9]
    want = [ref.forward(s, p, slot=i, logit_scale=2.5)["logits"] for i, (s, p) in enumerate(zip(spans, pos0))]
    got, lg = gpu.catchup_prefill(spans, pos0, tau, P.RS_SLM, [2.5, 2.5], want_logits=True)
    torch.cuda.synchronize()
    for i in range(2):
        check_invocation(got[i], lg[i], want[i], tau, P.RS_SLM, where=f"{name} ragged sequence {i}")
