"""GPU parity of rs_route (Eq. 1, Eq. 2) against the oracle router, through the C ABI."""
import math

import pytest
import torch

from oracle import router
from workloads.recipes import misc_normal, misc_uniform
from parity import check_invocation

pytestmark = pytest.mark.gpu


def run_route(P, logits, scales, tau, active):
    n, v = logits.shape
    d_logits = logits.to(torch.float32).cuda().contiguous()
    d_scale = None if scales is None else torch.tensor(scales, dtype=torch.float32, device="cuda")
    out = P.binding.new_route_out(n)
    scratch = torch.zeros(P.rs_route_scratch_bytes(n, v), dtype=torch.uint8, device="cuda")
    P.rs_route(d_logits, n, v, d_scale, tau, active, out, scratch)
    torch.cuda.synchronize()
    return P.binding.read_route_out(out), d_logits


@pytest.mark.parametrize("v", [2, 3, 1000, 1024, 152064])
def test_closed_forms(v):
    import paper_2507_17307_amd as P
    rows = [torch.full((v,), 1.5, dtype=torch.float64)]                        # uniform: H = ln V
    onehot = torch.zeros(v, dtype=torch.float64); onehot[v - 1] = 100.0; rows.append(onehot)   # one-hot: H = 0
    two = torch.zeros(v, dtype=torch.float64); two[v // 3] = 4.0; rows.append(two)             # two-level
    got, _ = run_route(P, torch.stack(rows), None, 0.5, P.RS_SLM)
    assert got[0].h_nats == pytest.approx(math.log(v), abs=1e-4) and got[0].h_norm == pytest.approx(1.0, abs=1e-5)
    assert got[0].token == 0 and got[0].hi and not got[0].accept           # all equal: lowest index
    assert got[1].h_nats == pytest.approx(0.0, abs=1e-6) and got[1].token == v - 1 and got[1].accept
    p1 = math.exp(4.0) / (math.exp(4.0) + v - 1)
    h = -p1 * math.log(p1) - (1 - p1) * math.log((1 - p1) / (v - 1))
    assert got[2].h_nats == pytest.approx(h, abs=1e-4) and got[2].token == v // 3


@pytest.mark.parametrize("v,n", [(1024, 8), (152064, 5), (50257, 3), (7, 2)])
def test_random_rows_against_oracle(v, n):
    import paper_2507_17307_amd as P
    base = misc_normal(21, v % 97, n * v).view(n, v).to(torch.float32).double()     # fp32-representable logits
    scales = (0.5 + 7.5 * misc_uniform(22, v % 97, n)).to(torch.float32)
    for active in (P.RS_SLM, P.RS_LLM):
        got, _ = run_route(P, base, scales.tolist(), 0.6, active)
        for r in range(n):
            ref = (base[r].to(torch.float32) * scales[r]).double()       # the product the kernel forms, in fp32
            check_invocation(got[r], None, ref, 0.6, active, where=f"row {r}")


def test_entropy_thresholds_and_nonfinite_flags():
    import paper_2507_17307_amd as P
    v = 4096
    x = misc_normal(23, 1, v).to(torch.float32).double() * 3
    h = router.normalised_entropy(x)
    for tau, hi in ((h - 0.01, True), (h + 0.01, False)):
        got, _ = run_route(P, x.view(1, v), None, tau, P.RS_SLM)
        assert got[0].hi == hi and got[0].accept == (not hi)
        got, _ = run_route(P, x.view(1, v), None, tau, P.RS_LLM)
        assert got[0].hi == hi and got[0].accept
    y = x.clone().view(1, v); y[0, 17] = float("inf")
    got, _ = run_route(P, y, None, 0.5, P.RS_SLM)
    assert got[0].flags & P.FLAG_NONFINITE and got[0].hi and not got[0].accept and got[0].token == -1
