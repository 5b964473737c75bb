"""Partitioning model (Section 4.2): pins of the numpy/scipy oracle against closed
forms and Monte-Carlo, then the library's C implementation against the oracle.
CPU only."""
import numpy as np
import pytest

from oracle import partition_oracle as po
from synthdata.generate import zipf_probabilities


@pytest.fixture(scope="module")
def lib():
    import os
    import paper_2504_08930_amd as pkg
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2504_08930_amd.build import build
        build()
    from paper_2504_08930_amd import binding
    binding.load_library()
    return binding


# ---------------- oracle pins ----------------
def test_oracle_min_hit_rate_closed_forms():
    # B = 1: the expected minimum is the mean
    for mean, s2 in ((0.2, 0.01), (0.5, 0.05), (0.83, 0.02)):
        assert abs(po.expected_min_hit_rate(mean, s2, 1) - mean) < 1e-9
    # mean 0.5 with sigma_max^2 = 1/12 is the uniform distribution: E[min of B] = 1/(B+1)
    for B in (1, 2, 5, 32):
        assert abs(po.expected_min_hit_rate(0.5, 1.0 / 12.0, B) - 1.0 / (B + 1)) < 1e-9
    # variance model: equals sigma_max^2 at mean 0.5, vanishes towards 0 and 1
    a, b = po.beta_params(0.5, 0.03)
    assert abs(a * b / ((a + b) ** 2 * (a + b + 1)) - 0.03) < 1e-12
    a, b = po.beta_params(0.9, 0.03)
    assert abs(a / (a + b) - 0.9) < 1e-12
    assert abs(a * b / ((a + b) ** 2 * (a + b + 1)) - 4 * 0.03 * 0.9 * 0.1) < 1e-12


def test_oracle_min_hit_rate_monte_carlo_and_monotone():
    rng = np.random.default_rng(0)
    for mean, s2, B in ((0.6, 0.02, 8), (0.3, 0.04, 16), (0.85, 0.01, 64)):
        a, b = po.beta_params(mean, s2)
        draws = rng.beta(a, b, size=(200_000, B)).min(1)
        est, se = draws.mean(), draws.std() / np.sqrt(draws.size)
        assert abs(po.expected_min_hit_rate(mean, s2, B) - est) < 5 * se + 1e-4
    vals = [po.expected_min_hit_rate(0.7, 0.02, B) for B in (1, 2, 4, 8, 16, 64, 256)]
    assert all(x >= y for x, y in zip(vals, vals[1:]))
    vals = [po.expected_min_hit_rate(m, 0.02, 16) for m in (0.1, 0.3, 0.5, 0.7, 0.9)]
    assert all(x < y for x, y in zip(vals, vals[1:]))


def test_oracle_hybrid_latency_hand_instance():
    # knots: b=1 -> (T_CQ 2, T_LUT 10); b=8 -> (4, 24).  At b=4: T_CQ = 2 + 2*3/7, T_LUT = 16.
    kb, cq, lut = [1, 8], [2, 4], [10, 24]
    assert abs(po.piecewise_linear(kb, lut, 4) - 16.0) < 1e-12
    assert abs(po.hybrid_latency(kb, cq, lut, 4, 0.25) - (2 + 6 / 7 + 0.75 * 16)) < 1e-12
    assert abs(po.hybrid_latency(kb, cq, lut, 4, 1.0) - (2 + 6 / 7)) < 1e-12          # all hits
    assert abs(po.piecewise_linear(kb, lut, 15) - 38.0) < 1e-12                        # extrapolated


# ---------------- library against the oracle ----------------
def _profile(nlist=64, s=1.0):
    p = zipf_probabilities(nlist, s)
    hit_cdf = np.concatenate([[0.0], np.cumsum(p)])
    hit_cdf[-1] = 1.0
    sizes = 50_000.0 + 20_000.0 * np.sin(np.arange(nlist))          # bytes per cluster
    mem = np.concatenate([[0.0], np.cumsum(sizes)])
    return hit_cdf, mem


def test_library_min_hit_rate_matches_oracle(lib):
    for mean in (0.05, 0.3, 0.5, 0.77, 0.95):
        for s2 in (0.005, 0.03, 1.0 / 12.0):
            for B in (1, 3, 16, 128):
                got = lib.ivf_model_min_hit_rate(mean, s2, B)
                assert abs(got - po.expected_min_hit_rate(mean, s2, B)) < 2e-6
    assert lib.ivf_model_min_hit_rate(0.0, 0.02, 4) == 0.0
    assert lib.ivf_model_min_hit_rate(1.0, 0.02, 4) == 1.0
    assert np.isnan(lib.ivf_model_min_hit_rate(0.5, 0.3, 4))


def test_library_latency_and_inverse_match_oracle(lib):
    kb, cq, lut = [1, 4, 16, 64], [1e-3, 1.5e-3, 3e-3, 9e-3], [4e-3, 6e-3, 14e-3, 50e-3]
    model = lib.LatencyModel(kb, cq, lut)
    for b in (1, 2.5, 4, 10, 64, 100):
        for eta in (0.0, 0.4, 1.0):
            assert abs(lib.ivf_model_hybrid_latency(model, b, eta) -
                       po.hybrid_latency(kb, cq, lut, b, eta)) < 1e-15
    hit_cdf, _ = _profile()
    for B in (1, 16):
        for target in (0.0, 0.3, 0.8, 0.999):
            got = lib.ivf_model_hitrate_to_coverage(hit_cdf, 0.02, B, target)
            ref = po.hitrate_to_coverage(hit_cdf, 0.02, B, target)
            assert abs(got - ref) <= 1.0 / 64 + 1e-12, (B, target, got, ref)


def test_library_partition_point_matches_oracle(lib):
    kb, cq, lut = [1, 4, 16, 64], [1e-3, 1.5e-3, 3e-3, 9e-3], [4e-3, 6e-3, 14e-3, 50e-3]
    model = lib.LatencyModel(kb, cq, lut)
    hit_cdf, mem = _profile()
    scenarios = [  # slo, eps, kv-cache bytes, LLM throughput (req/s), delta
        (20e-3, 1.0, 4 * mem[-1], 900.0, 1.0 / 64),
        (40e-3, 0.9, 2 * mem[-1], 600.0, 1.0 / 32),
    ]
    seen = set()
    for slo, eps, kv, mu0, delta in scenarios:
        got = lib.ivf_model_partition_point(model, hit_cdf, mem, 0.02, slo, eps, kv, mu0, delta)
        ref = po.partition_point(kb, cq, lut, hit_cdf, mem, 0.02, slo, eps, kv, mu0, delta)
        assert abs(got - ref) <= 1.0 / 64 + 1e-12, (slo, got, ref)
        seen.add(round(got, 3))
        # the returned coverage holds the latency target at the batch size it implies
        mu = (kv - mem[int(round(got * 64))]) / kv * mu0
        tau = slo / (1 + eps)
        B = max(1, int(np.floor(tau * mu)))
        eta = po.expected_min_hit_rate(float(hit_cdf[int(round(got * 64))]), 0.02, B)
        assert po.hybrid_latency(kb, cq, lut, B, eta) <= max(tau, B / mu) * 1.02
    assert len(seen) > 1          # the scenarios do not all collapse to one answer
    # a looser latency target never needs more coverage
    r1 = lib.ivf_model_partition_point(model, hit_cdf, mem, 0.02, 15e-3, 1.0, 4 * mem[-1], 900.0,
                                       1.0 / 64)
    r2 = lib.ivf_model_partition_point(model, hit_cdf, mem, 0.02, 60e-3, 1.0, 4 * mem[-1], 900.0,
                                       1.0 / 64)
    assert r2 <= r1 + 1.0 / 64
    with pytest.raises(lib.IvfError):
        lib.ivf_model_partition_point(model, hit_cdf, mem, 0.3, 15e-3, 1.0, 1.0, 1.0, 0.01)
