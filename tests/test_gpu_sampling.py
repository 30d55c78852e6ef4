"""GPU parity of sampled tokens (rs_set_sampling: Gumbel-max fused behind the LM head) against oracle/router.sample_token,
through the C ABI.  Both sides draw the same uniforms: the generator is a counter-based hash, the GPU implements it
itself, the oracle takes the numbers from workloads.rng."""
import dataclasses
import math

import pytest
import torch

import workloads as W
from oracle import decoder, router, stitch
from parity import check_invocation

pytestmark = pytest.mark.gpu

GAP = 1e-3       # sampled tokens are compared unless the two largest noisy logits are closer than this


def expected_token(ref_logits, key, pos_pred):
    v = ref_logits.numel()
    u = W.uniform23(key, pos_pred * v, v)
    noisy = ref_logits - torch.log(-torch.log(u))
    top2 = torch.topk(noisy, 2).values
    return router.sample_token(ref_logits, u), float(top2[0] - top2[1])


@pytest.mark.parametrize("shape_name", ["tiny_l", "wide_vocab"])
def test_sampled_tokens_of_every_lm_head_path_match_the_oracle(shape_name):
    """One-row steps, a 3-sequence step (FMA LM head with several rows), a 9-row span and a 5-sequence ragged call
    (matrix-core LM head); entropy and flags must be what they are without sampling."""
    import paper_2507_17307_amd as P
    shape = W.TINY_L if shape_name == "tiny_l" else W.ModelShape("wide_vocab", 2, 256, 4, 2, 64, 512, 50304, False)
    w = W.make_weights(shape, 9, 1)
    n, max_ctx = 5, 80
    key = W.stream_key(9, 31337)
    gpu = P.Model(w.to("cuda"), max_ctx=max_ctx, max_seqs=8, max_rows=64)
    P.rs_set_sampling(gpu.handle, True, key)
    ref = decoder.OracleModel(w, max_ctx, n_slots=8)
    toks = [W.rng.randint(9, 50 + i, 0, 60, shape.vocab).tolist() for i in range(n)]
    tau, compared = 0.6, 0

    def run(spans, pos0, slots, scales):
        nonlocal compared
        if all(len(s) == 1 for s in spans):
            got, lg = gpu.decode_step([s[0] for s in spans], pos0, tau, P.RS_LLM, scales, slots, want_logits=True)
        else:
            got, lg = gpu.catchup_prefill(spans, pos0, tau, P.RS_LLM, scales, slots, want_logits=True)
        torch.cuda.synchronize()
        for i, (s, p, sl, sc) in enumerate(zip(spans, pos0, slots, scales)):
            where = f"{shape_name} slot {sl} span {len(s)} at {p}"
            want = ref.forward(s, p, slot=sl, logit_scale=sc)["logits"]
            # entropy, flags and logits are what they are without sampling; only the token field differs
            check_invocation(dataclasses.replace(got[i], token=router.greedy_token(want)), lg[i], want, tau, router.LLM, where=where)
            tok, gap = expected_token(want, key, p + len(s))
            if gap >= GAP:
                compared += 1
                assert got[i].token == tok, f"{where}: sampled {got[i].token}, oracle {tok} (gap {gap})"

    run([toks[0][:9]], [0], [0], [3.0])                                  # 9-row span: matrix-core LM head, one sequence
    for i in range(9, 14):
        run([[toks[0][i]]], [i], [0], [1.0 + i % 4])                     # one-row steps
    run([toks[1][:2]], [0], [1], [2.0])                                  # two rows: FMA path
    run([toks[i][:3 + i] for i in range(2, 5)], [0, 0, 0], [2, 3, 4], [1.5, 2.5, 3.5])     # ragged, three sequences
    run([[toks[i][3 + i]] for i in range(2, 5)], [3 + i for i in range(2, 5)], [2, 3, 4], [4.0, 1.0, 2.0])   # 3-sequence step
    run([[toks[0][14]], [toks[1][2]], [toks[2][6]], [toks[3][7]], [toks[4][8]]], [14, 2, 6, 7, 8], [0, 1, 2, 3, 4],
        [1.0, 2.0, 3.0, 4.0, 5.0])                                       # 5-sequence step: matrix-core LM head, five rows
    assert compared >= 10
    # switching sampling off gives the arg max again
    P.rs_set_sampling(gpu.handle, False, 0)
    got, lg = gpu.decode_step([toks[0][15]], [15], tau, P.RS_LLM, [2.0], [0], want_logits=True)
    torch.cuda.synchronize()
    check_invocation(got[0], lg[0], ref.forward([toks[0][15]], 15, slot=0, logit_scale=2.0)["logits"], tau, router.LLM, where="greedy again")


def test_sampled_tokens_of_a_step_over_more_than_sixteen_sequences_match_the_oracle():
    """24 and 70 sequences in one decode step: the LM head in which one workgroup holds all rows (one and two blocks of 16
    rows per wave)."""
    import paper_2507_17307_amd as P
    shape = W.TINY_L
    w = W.make_weights(shape, 13, 1)
    key = W.stream_key(13, 4242)
    for n in (24, 70):
        gpu = P.Model(w.to("cuda"), max_ctx=32, max_seqs=128, max_rows=128)
        P.rs_set_sampling(gpu.handle, True, key)
        ref = decoder.OracleModel(w, 32, n_slots=128)
        slots = [(5 * i + 2) % 128 for i in range(n)]
        toks = W.rng.randint(13, 70 + n, 0, n, shape.vocab).tolist()
        pos = [i % 7 for i in range(n)]
        for i in range(n):                                     # earlier positions of every sequence, one call per sequence
            if pos[i]:
                pre = W.rng.randint(13, 500 + i, 0, pos[i], shape.vocab).tolist()
                ref.forward(pre, 0, slot=slots[i])
                gpu.forward_span(pre, 0, 0.5, P.RS_LLM, slot=slots[i])
        scales = [1.0 + 0.25 * (i % 16) for i in range(n)]
        got, lg = gpu.decode_step(toks, pos, 0.6, P.RS_SLM, scales, slots, want_logits=True)
        torch.cuda.synchronize()
        compared = 0
        for i in range(n):
            want = ref.forward([toks[i]], pos[i], slot=slots[i], logit_scale=scales[i])["logits"]
            check_invocation(dataclasses.replace(got[i], token=router.greedy_token(want)), lg[i], want, 0.6, router.SLM, where=f"{n} sequences, sequence {i}")
            tok, gap = expected_token(want, key, pos[i] + 1)
            if gap >= GAP:
                compared += 1
                assert got[i].token == tok, f"{n} sequences, sequence {i}: sampled {got[i].token}, oracle {tok} (gap {gap})"
        assert compared >= n - 3


def test_sampled_draws_follow_the_distribution_on_the_gpu():
    """The same step run under 4000 different keys: the frequencies of the drawn tokens follow the step's softmax
    probabilities (a property check that does not involve the oracle's generator)."""
    import paper_2507_17307_amd as P
    shape = W.ModelShape("few_tokens", 1, 128, 4, 2, 32, 128, 8, False)
    w = W.make_weights(shape, 12, 1)
    gpu = P.Model(w.to("cuda"), max_ctx=8)
    ref = decoder.OracleModel(w, 8)
    logits = ref.forward([3], 0, logit_scale=4.0)["logits"]
    p = router.softmax(logits)
    counts = torch.zeros(8)
    n = 4000
    for k in range(n):
        P.rs_set_sampling(gpu.handle, True, W.stream_key(100, k))
        counts[gpu.decode_step([3], [0], 0.5, P.RS_SLM, [4.0])[0].token] += 1
    sigma = torch.sqrt(p * (1 - p) / n).float()
    assert bool(((counts / n - p.float()).abs() <= 4.5 * sigma + 1e-3).all()), (counts / n, p)
    assert float(p.max()) < 0.9                                         # the step is not a degenerate one


def test_live_sampled_run_matches_the_oracles_sampled_run():
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedPair
    wl = W.WORKLOADS["cfg1_tiny_pair"]
    ws, wl_ = W.make_weights(wl.slm, wl.seed, 0), W.make_weights(wl.llm, wl.seed, 1)
    prompt = W.make_prompt(wl).tolist()
    scales = W.logit_scale(wl, 0, wl.max_ctx + 2)
    key = W.stream_key(wl.seed, 777)
    v = wl.slm.vocab
    uni = lambda p: W.uniform23(key, p * v, v)  # noqa: E731
    mk = lambda: [decoder.OracleModel(ws, wl.max_ctx + 1), decoder.OracleModel(wl_, wl.max_ctx + 1)]  # noqa: E731
    sc = lambda p: float(scales[p])  # noqa: E731
    solo = stitch.generate(prompt, stitch.decoder_forward(mk(), sc, uniforms_of_pos=uni), 2.0, wl.n_decode)
    tau = W.pick_tau([t.h_norm for t in solo.trace], wl.tau_percentile, 4e-3 / math.log(v))
    log = []
    res = stitch.generate(prompt, stitch.decoder_forward(mk(), sc, log, uniforms_of_pos=uni), tau, wl.n_decode)
    gaps = []
    for t, lg in zip(res.trace, log):
        noisy = lg - torch.log(-torch.log(uni(t.pos0 + len(t.span))))
        top2 = torch.topk(noisy, 2).values
        gaps.append(float(top2[0] - top2[1]))
    assert min(gaps) > GAP, "a draw of this key sits on a knife edge; pick another key"
    assert len(set(res.output)) > 8 and res.n_rejected > 0                # sampling makes the run non-degenerate
    gpu = [P.Model(x.to("cuda"), max_ctx=wl.max_ctx + 1, max_rows=64) for x in (ws, wl_)]
    run = StitchedPair(gpu[0], gpu[1], wl.max_ctx, scales).generate(prompt, tau, wl.n_decode, sampling_key=key)
    assert run.output == res.output
    assert [(t.model, t.pos0, t.n_rows, t.accept) for t in run.trace] == [(t.model, t.pos0, len(t.span), t.accept) for t in res.trace]
