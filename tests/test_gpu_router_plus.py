"""GPU parity of rs_route_plus (the learned router of R-Stitch+) against oracle/router_plus.py, through the C ABI."""
import math

import pytest
import torch

import workloads as W
from oracle import decoder, router, router_plus as rp, stitch
from workloads.recipes import misc_normal

pytestmark = pytest.mark.gpu

GAP = 1e-3          # decisions are compared unless the two outputs are closer than this


def records(P, flags_list):
    out = P.binding.new_route_out(len(flags_list))
    host = torch.zeros(len(flags_list), 6, dtype=torch.int32)
    for i, f in enumerate(flags_list):
        host[i, 1] = f
    out.copy_(host)
    return out


@pytest.mark.parametrize("d,r,n", [(1536, 8, 5), (128, 8, 3), (256, 64, 2), (3584, 16, 4)])
def test_router_outputs_and_flag_rewrite_on_given_hidden_states(d, r, n):
    import paper_2507_17307_amd as P
    w = W.make_router_weights(d, r, seed=7)
    rt = P.RouterPlus(w.to("cuda"))
    hidden = (misc_normal(9, d % 89, n * d).view(n, d) * 0.7).to(torch.float32)
    want = rp.router_logits(w, hidden.double())
    hi_accept = P.FLAG_HI | P.FLAG_NEXT_LLM                      # what the entropy rule leaves for an uncertain small-model step
    for active in (P.RS_SLM, P.RS_LLM):
        flags_in = [hi_accept if i % 2 == 0 else P.FLAG_ACCEPT for i in range(n)]          # odd rows: low entropy, not for the router
        if active == P.RS_LLM:
            flags_in = [f | P.FLAG_ACCEPT for f in flags_in]
        out = records(P, flags_in)
        lg = torch.zeros(n, 2, device="cuda")
        P.rs_route_plus(None, hidden.cuda(), n, rt, active, out, lg)
        torch.cuda.synchronize()
        got = lg.cpu().double()
        assert float((got - want).abs().max()) <= 1e-3 * max(1.0, float(want.abs().max())), (got, want)
        flags = [int(x) & 0xFFFFFFFF for x in out.cpu()[:, 1]]
        for i in range(n):
            if abs(float(want[i, 1] - want[i, 0])) < GAP:
                continue
            stay = not bool(want[i, 1] > want[i, 0])
            hi, accept, nxt = rp.switch_plus(2.0 if flags_in[i] & P.FLAG_HI else 0.0, 1.0, active, not stay)
            expect = (P.FLAG_HI if hi else 0) | (P.FLAG_ACCEPT if accept else 0) | (P.FLAG_NEXT_LLM if nxt == 1 else 0)
            if active == P.RS_SLM and hi and stay:
                expect |= P.FLAG_ROUTER_STAY
            assert flags[i] == expect, (i, active, flags[i], expect)


def test_router_reads_the_hidden_state_of_the_models_last_call():
    """After a forward call the router takes the final hidden state (before the final RMSNorm) of the last row of
    each sequence from the model's workspace: compared with the oracle's hidden state of the same call."""
    import paper_2507_17307_amd as P
    shape = W.TINY_L
    wts = W.make_weights(shape, 4, 1)
    w = W.make_router_weights(shape.d_model, 8, seed=8)
    rt = P.RouterPlus(w.to("cuda"))
    ref = decoder.OracleModel(wts, 64, n_slots=2)
    gpu = P.Model(wts.to("cuda"), max_ctx=64, max_seqs=2, max_rows=64)
    toks = W.rng.randint(4, 11, 0, 40, shape.vocab).tolist()
    for spans, pos0 in (([toks[:9], toks[9:12]], [0, 0]), ([toks[20:21], toks[21:22]], [9, 3])):
        hid = [ref.forward(s, p, slot=i, want_hidden=True)["hidden"][-1] for i, (s, p) in enumerate(zip(spans, pos0))]
        want = torch.stack([rp.router_logits(w, h) for h in hid])
        if len(spans[0]) == 1:
            out = P.binding.new_route_out(2)
            P.rs_decode_step(gpu.handle, 2, gpu._i32([0, 1]), gpu._i32([s[0] for s in spans]), gpu._i32(pos0), None, -1.0, P.RS_SLM, out)
        else:
            flat = spans[0] + spans[1]
            out = P.binding.new_route_out(2)
            P.rs_catchup_prefill(gpu.handle, 2, len(flat), gpu._i32([0, 1]), gpu._i32(flat), gpu._i32([0, len(spans[0]), len(flat)]),
                                 gpu._i32(pos0), None, -1.0, P.RS_SLM, out)
        lg = torch.zeros(2, 2, device="cuda")
        P.rs_route_plus(gpu.handle, None, 2, rt, P.RS_SLM, out, lg)
        torch.cuda.synchronize()
        assert float((lg.cpu().double() - want).abs().max()) <= 1e-3 * max(1.0, float(want.abs().max()))
        recs = P.binding.read_route_out(out)
        for i in range(2):                                     # tau = -1: every step is "uncertain", so the router decides
            if abs(float(want[i, 1] - want[i, 0])) >= GAP:
                stay = not bool(want[i, 1] > want[i, 0])
                assert bool(recs[i].flags & P.FLAG_ROUTER_STAY) == stay and recs[i].accept == stay


def test_live_run_with_the_router_matches_the_oracles_r_stitch_plus_run():
    """Algorithm 1 with its R-Stitch+ branch, live on the GPU through the host driver, against the oracle's run on
    config 1 with a seeded synthetic router: same tokens, same model, span and acceptance per invocation."""
    import paper_2507_17307_amd as P
    from paper_2507_17307_amd.stitch import StitchedPair
    wl = W.WORKLOADS["cfg1_tiny_pair"]
    ws, wl_ = W.make_weights(wl.slm, wl.seed, 0), W.make_weights(wl.llm, wl.seed, 1)
    w = W.make_router_weights(wl.slm.d_model, 8, seed=7)
    prompt = W.make_prompt(wl).tolist()
    scales = W.logit_scale(wl, 0, wl.max_ctx + 2)
    models = [decoder.OracleModel(ws, wl.max_ctx + 1), decoder.OracleModel(wl_, wl.max_ctx + 1)]
    gaps = []

    def forward_state(model, span, pos0):
        out = models[model].forward(span, pos0, logit_scale=float(scales[pos0 + len(span)]), want_hidden=True)
        return router.greedy_token(out["logits"]), router.normalised_entropy(out["logits"]), out["hidden"][-1]

    def says_llm(hidden):
        o = rp.router_logits(w, hidden)
        gaps.append(abs(float(o[1] - o[0])))
        return bool(o[1] > o[0])

    solo = stitch.generate_plus(prompt, forward_state, lambda s: False, 2.0, wl.n_decode)
    tau = W.pick_tau([t.h_norm for t in solo.trace], 50.0, 4e-3 / math.log(wl.slm.vocab))
    models = [decoder.OracleModel(ws, wl.max_ctx + 1), decoder.OracleModel(wl_, wl.max_ctx + 1)]
    res = stitch.generate_plus(prompt, forward_state, says_llm, tau, wl.n_decode)
    assert min(gaps) > GAP, "a router decision of this seed sits on the knife edge; pick another seed"
    stays = sum(1 for t in res.trace if t.model == 0 and t.hi and t.accept)
    assert stays > 0 and res.n_rejected > 0, "the run must contain both router outcomes"
    models = [decoder.OracleModel(ws, wl.max_ctx + 1), decoder.OracleModel(wl_, wl.max_ctx + 1)]
    plain = stitch.generate(prompt, lambda m, s, p: forward_state(m, s, p)[:2], tau, wl.n_decode)
    assert [(t.model, t.pos0) for t in plain.trace] != [(t.model, t.pos0) for t in res.trace], \
        "the router must change the course of the run, or the comparison below proves nothing"
    gpu = [P.Model(x.to("cuda"), max_ctx=wl.max_ctx + 1, max_rows=64) for x in (ws, wl_)]
    pair = StitchedPair(gpu[0], gpu[1], wl.max_ctx, scales)
    run = pair.generate(prompt, tau, wl.n_decode, router_plus=P.RouterPlus(w.to("cuda")))
    assert run.output == res.output
    assert [(t.model, t.pos0, t.n_rows, t.accept) for t in run.trace] == [(t.model, t.pos0, len(t.span), t.accept) for t in res.trace]
    assert sum(1 for t in run.trace if t.flags & P.FLAG_ROUTER_STAY) == stays
