"""Partitioning model (Section 4.1): pins of the numpy/scipy oracle against closed
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


# ---------------- Algorithm 1: pins that do not go through its own listing ----------------
def test_infer_partition_hand_worked_instances(lib):
    """InferPartition of Algorithm 1 worked by hand (Section 4.1.3, "Rounding up" /
    "Rounding down"): four clusters whose hottest 0..4 cover 0, 1/2, 3/4, 9/10, 1 of the
    accesses; sigma_max^2 = 1/12, for which the hit-rate model at mean 1/2 is the uniform
    distribution (expected minimum of B draws = 1/(B+1)); tau_s = 10 ms, mu = 150 /s, so
    tau_s * mu = 1.5: B = 2 rounding up, B = 1 rounding down with the bound B/mu = 6.67 ms.

    (a) flat latency models T_CQ = 1 ms, T_LUT = 12 ms:
        eta_1 = (13 - 10) / 12 = 0.25; with B = 2 no coverage gives 0 and one cluster gives
        1/3 >= 0.25, so rho_1 = 1/4.
        eta_2 = (13 - 6.67) / 12 = 0.528; with B = 1 the expected minimum is the mean, and the
        first prefix that covers 0.528 is two clusters (0.75), so rho_2 = 1/2.  min = 1/4.
    (b) models through the origin, T_CQ = 1 ms * b, T_LUT = 16/3 ms * b:
        eta_1 = (2 + 10.67 - 10) / 10.67 = 0.25 -> rho_1 = 1/4;
        eta_2 = (1 + 5.33 - 6.67) / 5.33 < 0 -> no coverage needed, rho_2 = 0.  min = 0.
    (c) T_CQ = 1 ms, T_LUT = 8 ms at b = 1 and 12 ms at b = 2, where it matters that rounding down
        is held to B/mu and not to tau_s: eta_1 = 0.25 -> rho_1 = 1/4 as in (a);
        eta_2 = (9 - 6.67) / 8 = 0.29 -> one cluster (0.5), rho_2 = 1/4; min = 1/4.  (Held to
        tau_s, eta_2 = (9 - 10) / 8 < 0 would ask for no coverage and the minimum would be 0.)
    The library's InferPartition is reached through Algorithm 1 with an index that takes no
    memory (mu stays mu_LLM0, so every iteration returns the same value)."""
    hit_cdf = np.array([0.0, 0.5, 0.75, 0.9, 1.0])
    s2, tau, mu = 1.0 / 12.0, 10e-3, 150.0
    cases = [(([1.0, 2.0], [1e-3, 1e-3], [12e-3, 12e-3]), 0.25),
             (([1.0, 2.0], [1e-3, 2e-3], [16e-3 / 3, 32e-3 / 3]), 0.0),
             (([1.0, 2.0], [1e-3, 1e-3], [8e-3, 12e-3]), 0.25)]
    for (kb, cq, lut), want in cases:
        assert po.infer_partition(kb, cq, lut, hit_cdf, s2, tau, mu) == want
        model = lib.LatencyModel(kb, cq, lut)
        got = lib.ivf_model_partition_point(model, hit_cdf, np.zeros(5), s2, 2 * tau, 1.0, 1.0, mu,
                                            1.0 / 8)
        assert got == want
    # the two roundings apart, from the closed forms used above
    assert abs(po.expected_min_hit_rate(0.5, s2, 2) - 1.0 / 3.0) < 1e-9
    assert po.hitrate_to_coverage(hit_cdf, s2, 2, 0.25) == 0.25
    assert po.hitrate_to_coverage(hit_cdf, s2, 1, (13e-3 - 1 / 150.0) / 12e-3) == 0.5


_ETA_MEMO = {}


def _eta_min(mean, s2, B):
    """expected_min_hit_rate with a memo: the brute force asks for the same few batch sizes
    at every prefix of the profile."""
    key = (round(mean, 15), s2, B)
    if key not in _ETA_MEMO:
        _ETA_MEMO[key] = po.expected_min_hit_rate(mean, s2, B)
    return _ETA_MEMO[key]


def _coverage_needed_brute(kb, cq, lut, hit_cdf, s2, tau_s, mu):
    """What InferPartition must return, from the definitions and not from its algebra:
    for either rounding of B = tau_s * mu, the smallest prefix of clusters at which the
    latency of Eq. (1), with the expected smallest hit rate of Eq. (2), meets the bound
    (tau_s rounding up; B / mu rounding down), 1 if none does; then the smaller."""
    nlist = len(hit_cdf) - 1
    out = []
    for B, bound in ((max(1, int(np.ceil(tau_s * mu))), tau_s),
                     (max(1, int(np.floor(tau_s * mu))), None)):
        if bound is None:
            bound = B / mu
        need = 1.0
        for i in range(nlist + 1):
            eta = _eta_min(float(hit_cdf[i]), s2, B)
            if po.hybrid_latency(kb, cq, lut, B, eta) <= bound * (1 + 1e-12):
                need = i / nlist
                break
        out.append(need)
    return min(out)


@pytest.mark.parametrize("zipf_s,slo,kv_mult,mu0", [(1.0, 20e-3, 4.0, 900.0),
                                                    (0.7, 24e-3, 2.0, 1500.0),
                                                    (1.3, 16e-3, 3.0, 1500.0),
                                                    (1.0, 30e-3, 1.5, 1500.0)])
def test_partition_point_is_the_self_consistent_crossing(lib, zipf_s, slo, kv_mult, mu0):
    """Algorithm 1 searches for the coverage rho at which the coverage that the latency bound
    asks for, at the batch size the remaining LLM throughput implies, equals the coverage
    spent.  Brute force over every cluster count i: evaluate the needed coverage need(i) from
    Eq. (1) and Eq. (2) directly (no inversion formula, no bisection) with mu taken at i
    clusters; below the crossing need(i) > i / nlist, from it on need(i) <= i / nlist.  Both
    the oracle's and the library's answers must lie at that crossing, within the search's
    stopping width delta plus the size of the steps need() takes there."""
    nlist = 48
    kb, cq, lut = [1, 4, 16, 64], [1e-3, 1.5e-3, 3e-3, 9e-3], [4e-3, 6e-3, 14e-3, 50e-3]
    hit_cdf, mem = _profile(nlist, zipf_s)
    s2, eps, delta = 0.02, 1.0, 1.0 / 256
    kv = kv_mult * mem[-1]
    tau_s = slo / (1 + eps)
    need = np.empty(nlist + 1)
    for i in range(nlist + 1):
        mu = max(0.0, (kv - mem[i]) / kv) * mu0
        need[i] = _coverage_needed_brute(kb, cq, lut, hit_cdf, s2, tau_s, mu)
    frac = np.arange(nlist + 1) / nlist
    ok = need <= frac
    assert ok.any() and not ok.all(), "scenario has no interior crossing"
    i_star = int(np.argmax(ok))
    assert not ok[:i_star].any() and ok[i_star:].all(), "need(i) - i/nlist changes sign once"
    # the answer is need() at the last midpoint, which lies within delta of the crossing
    near = need[max(0, i_star - 2): i_star + 2]
    lo, hi = near.min() - 1e-12, near.max() + 1e-12
    ref = po.partition_point(kb, cq, lut, hit_cdf, mem, s2, slo, eps, kv, mu0, delta)
    got = lib.ivf_model_partition_point(lib.LatencyModel(kb, cq, lut), hit_cdf, mem, s2, slo, eps,
                                        kv, mu0, delta)
    for name, val in (("oracle", ref), ("library", got)):
        assert lo <= val <= hi, (name, val, i_star / nlist, near)
        assert abs(val - i_star / nlist) <= delta + 2.0 / nlist + (hi - lo), (name, val, i_star)


# ---------------------------------------------------------------------------
# Planted mistakes: each is an exact textual edit of a copy of the oracle's source,
# run as a module of its own under the pins named for it; every named pin must fail.
# ---------------------------------------------------------------------------
def _pin_closed(lib):
    test_oracle_min_hit_rate_closed_forms()


def _pin_monte_carlo(lib):
    test_oracle_min_hit_rate_monte_carlo_and_monotone()


def _pin_latency(lib):
    test_oracle_hybrid_latency_hand_instance()


def _pin_infer(lib):
    test_infer_partition_hand_worked_instances(lib)


def _pin_crossing(lib):
    for args in ((1.0, 20e-3, 4.0, 900.0), (0.7, 24e-3, 2.0, 1500.0), (1.3, 16e-3, 3.0, 1500.0),
                 (1.0, 30e-3, 1.5, 1500.0)):
        test_partition_point_is_the_self_consistent_crossing(lib, *args)


PLANTED = {
    "Eq. (1) adds the hit share of the table time": (
        [("(1.0 - eta) * piecewise_linear", "(1.0 + eta) * piecewise_linear", 1)], [_pin_latency]),
    "variance model with half its factor": (
        [("var = 4.0 * sigma_max2", "var = 2.0 * sigma_max2", 1)], [_pin_closed]),
    "Eq. (2) with the exponent B": (
        [("(1.0 - u) ** (B - 1)", "(1.0 - u) ** B", 1)], [_pin_closed, _pin_monte_carlo]),
    "no extrapolation beyond the last knot": (
        [("0, len(kb) - 2))", "0, len(kb) - 2))\n    b = min(b, kb[-1])", 1)], [_pin_latency]),
    "coverage one cluster too many": (
        [("            return i / nlist\n", "            return (i + 1) / nlist\n", 1)], [_pin_infer]),
    "the larger of the two roundings' coverages": (
        [("return min(out)", "return max(out)", 1)], [_pin_infer]),
    "rounding down held to tau_s instead of B / mu": (
        [("target = tau_s if bound is None else B / mu", "target = tau_s", 1)], [_pin_infer]),
    "bisection moves the wrong end": (
        [("        if rho > mid:\n            lo = mid\n        else:\n            hi = mid",
          "        if rho > mid:\n            hi = mid\n        else:\n            lo = mid", 1)],
        [_pin_crossing]),
    "throughput from the index's share of memory": (
        [("(mem_kvcache - mem) / mem_kvcache", "mem / mem_kvcache", 1)], [_pin_crossing]),
    "latency budget not split with the queue": (
        [("tau_s = slo_search / (1.0 + eps)", "tau_s = slo_search", 1)], [_pin_crossing]),
}


@pytest.mark.parametrize("mistake", sorted(PLANTED))
def test_a_planted_mistake_fails_a_pin(lib, monkeypatch, mistake):
    import sys
    import types
    edits, pins = PLANTED[mistake]
    src = open(po.__file__).read()
    for text, replacement, occurrences in edits:
        assert src.count(text) == occurrences, (mistake, text)
        src = src.replace(text, replacement)
    mutant = types.ModuleType("partition_oracle_mutant")
    exec(compile(src, "partition_oracle_mutant.py", "exec"), mutant.__dict__)
    monkeypatch.setattr(sys.modules[__name__], "po", mutant)
    monkeypatch.setattr(sys.modules[__name__], "_ETA_MEMO", {})
    noticed = []
    for pin in pins:
        try:
            pin(lib)
        except (AssertionError, ArithmeticError):   # a mutant may also divide by zero
            noticed.append(pin.__name__)
    assert noticed == [p.__name__ for p in pins], f"{mistake}: noticed only by {noticed}"
