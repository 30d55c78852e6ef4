"""rs_route_static (the entry point that allocates nothing) against rs_route, through the C ABI.

Both run the same two kernels; only where the partial softmax states live differs (a device array
inside the library instead of a caller buffer), so the records must be identical bit for bit.  Two
calls in a row on the same stream, the second with a smaller input: the shared array keeps the first
call's states and none of them may leak into the second result.
"""
import pytest
import torch

from workloads.recipes import misc_normal, misc_uniform

pytestmark = pytest.mark.gpu


def both(P, logits, scales, tau, active):
    n, v = logits.shape
    d_logits = logits.to(torch.float32).cuda().contiguous()
    d_scale = torch.tensor(scales, dtype=torch.float32, device="cuda")
    ref, got = P.binding.new_route_out(n), P.binding.new_route_out(n)
    scratch = torch.zeros(P.rs_route_scratch_bytes(n, v), dtype=torch.uint8, device="cuda")
    P.rs_route(d_logits, n, v, d_scale, tau, active, ref, scratch)
    P.rs_route_static(d_logits, n, v, d_scale, tau, active, got)
    return ref, got


def test_static_scratch_route_equals_rs_route_on_two_calls_in_a_row():
    import paper_2507_17307_amd as P
    cases = [(152064, 8), (50257, 3), (1000, 64), (7, 1)]          # each call smaller than the one before in states used
    pending = []
    for k, (v, n) in enumerate(cases):
        x = misc_normal(31, k, n * v).view(n, v)
        sc = (0.5 + 7.5 * misc_uniform(32, k, n)).tolist()
        pending.append(both(P, x, sc, 0.6, P.RS_SLM if k % 2 == 0 else P.RS_LLM))
    torch.cuda.synchronize()
    for ref, got in pending:
        assert torch.equal(ref.cpu(), got.cpu())
    recs = P.binding.read_route_out(pending[0][1])
    assert all(0 <= r.token < 152064 and 0.0 < r.h_norm <= 1.0 for r in recs)


def test_static_scratch_route_rejects_what_does_not_fit():
    import paper_2507_17307_amd as P
    x = torch.zeros(65, 8, device="cuda")
    out = P.binding.new_route_out(65)
    with pytest.raises(P.RsError) as e:
        P.rs_route_static(x, 65, 8, None, 0.5, P.RS_SLM, out)
    assert e.value.status == -2 and "64" in str(e.value)
    with pytest.raises(P.RsError):
        P.rs_route_static(x, 1, 1, None, 0.5, P.RS_SLM, out)
    torch.cuda.synchronize()
