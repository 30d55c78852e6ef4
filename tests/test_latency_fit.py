"""The latency model of the paper (Eq. 5-6) as bench.py fits it to this machine's timings.

Pins: the coefficients bench.py prints beside its own are the ones the paper prints (fixture
tests/golden/latency_coefficients.txt); the fit recovers planted coefficients exactly; fitted to samples drawn from
the paper's own functions it returns the paper's coefficients; a decode step is the N_inf = 1 case (Eq. 6)."""
import os

import numpy as np
import pytest

import bench

ROOT = os.path.dirname(os.path.abspath(__file__))


def paper_rows():
    rows = {}
    for line in open(os.path.join(ROOT, "golden", "latency_coefficients.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, *vals = line.split()
        rows[name] = tuple(float(v) for v in vals)
    return rows


def test_bench_quotes_the_papers_coefficients():
    rows = paper_rows()
    assert bench.PAPER_LATENCY_A100_MS == {"s15": rows["1.5B"], "m7": rows["7B"], "m14": rows["14B"]}


def test_fit_recovers_planted_coefficients():
    a, b, c, d = 3.0e-6, 2.0e-4, 0.05, 1.2
    samples = [(n, kv, a * n * kv + b * n * n + c * n + d) for n in (1, 2, 5, 17, 64) for kv in (0, 100, 3000, 9000)]
    fit = bench.fit_latency(samples)
    assert (fit["a"], fit["b"], fit["c"], fit["d"]) == pytest.approx((a, b, c, d), rel=1e-9)
    assert fit["r2"] == 1.0 and fit["samples"] == 20


@pytest.mark.parametrize("model", ["1.5B", "7B", "14B"])
def test_fit_of_the_papers_own_functions_returns_the_papers_coefficients(model):
    a, b, c, d = paper_rows()[model]
    grid = [(n, kv) for n in (1, 4, 16, 64, 256, 1024) for kv in (0, 512, 4096, 16384)]
    fit = bench.fit_latency([(n, kv, a * n * kv + b * n * n + c * n + d) for n, kv in grid])
    assert (fit["a"], fit["b"], fit["c"], fit["d"]) == pytest.approx((a, b, c, d), rel=1e-7)
    # Eq. 6: a decode step is linear in the cache size with slope a and intercept b + c + d
    t = [fit["a"] * kv + fit["b"] + fit["c"] + fit["d"] for kv in (0, 8192)]
    assert t[0] == pytest.approx(b + c + d, rel=1e-7) and (t[1] - t[0]) / 8192 == pytest.approx(a, rel=1e-7)


def test_fit_with_noise_reports_r2_below_one():
    rng = np.random.default_rng(0)
    samples = [(n, kv, 1e-5 * n * kv + 0.1 * n + 2.0 + rng.normal(0, 0.05)) for n in (1, 2, 4, 8, 16, 32, 64) for kv in (256, 1024, 4096)]
    fit = bench.fit_latency(samples)
    assert 0.9 < fit["r2"] < 1.0 and fit["a"] == pytest.approx(1e-5, rel=0.2)
