"""Shared comparison rules for GPU-versus-oracle parity (not a test module).

Tolerances are the ones the task states: scaled logits within 2e-2 (logits of
magnitude ~10), entropy within 1e-3 nats, argmax exact unless the two largest
logits are closer than 1e-3, routing flags exact unless the entropy is within
1e-3 nats of the threshold tau * ln V.
"""
import math

import torch

from oracle import router

LOGIT_TOL = 2e-2
ENTROPY_TOL = 1e-3
ARGMAX_GAP = 1e-3
TAU_BAND = 1e-3


def check_invocation(got, got_logits, ref_logits, tau, active, where=""):
    """got: binding.RouteOut; got_logits: fp32 tensor [V] (device or host) or None;
    ref_logits: fp64 oracle logits [V]."""
    v = ref_logits.numel()
    want = router.route(ref_logits, tau, active)
    if got_logits is not None:
        err = float((got_logits.detach().cpu().double() - ref_logits).abs().max())
        assert err <= LOGIT_TOL, f"{where}: logits max-abs error {err}"
    assert not (got.flags & (8 | 16)), f"{where}: unexpected flags {got.flags}"
    assert abs(got.h_nats - want["h_nats"]) <= ENTROPY_TOL, f"{where}: entropy {got.h_nats} vs {want['h_nats']}"
    assert abs(got.h_norm - want["h_norm"]) <= ENTROPY_TOL / math.log(v) + 1e-6, where
    assert abs(got.max_logit - want["max_logit"]) <= LOGIT_TOL and abs(got.log_z - want["log_z"]) <= LOGIT_TOL, where
    top2 = torch.topk(ref_logits, 2).values
    if float(top2[0] - top2[1]) >= ARGMAX_GAP:
        assert got.token == want["token"], f"{where}: token {got.token} vs {want['token']}"
    else:
        assert float(ref_logits[got.token]) >= float(top2[0]) - ARGMAX_GAP - LOGIT_TOL, where
    if abs(want["h_nats"] - tau * math.log(v)) >= TAU_BAND:
        assert (got.flags & 7) == (want["flags"] & 7), f"{where}: flags {got.flags} vs {want['flags']}"
    return want
