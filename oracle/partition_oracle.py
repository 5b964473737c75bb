"""Oracle for the latency-bounded partitioning model.  TEST INFRASTRUCTURE ONLY.

Plain numpy/scipy, written from the definitions:
  * piecewise-linear CPU latency models T_CQ(b), T_LUT(b) (Section 4.1.1);
  * hybrid latency, Eq. (1): tau_s(b) = T_CQ(b) + (1 - eta) * T_LUT(b);
  * per-query hit rate ~ Beta with mean eta_bar and variance
    4 * sigma_max^2 * eta_bar * (1 - eta_bar) (Section 4.1.2);
  * expected minimum hit rate in a batch, Eq. (2):
    eta_min(B) = int_0^1 B x f(x) (1 - F(x))^(B-1) dx   (scipy quadrature, in u = F(x));
  * its numerical inverse over the measured hit-rate profile ("HitRate2Coverage");
  * Algorithm 1 (binary search on rho with InferPartition).

Readings of the garbled listing of Algorithm 1: MEM_Index is evaluated at the
midpoint rho_m; t_s is tau_s; the interval update is plain bisection on the sign
of InferPartition(rho_m) - rho_m (rho_low <- rho_m when more coverage is needed);
T_search = T_CQ + T_LUT; a required hit rate <= 0 needs no GPU coverage and a
required hit rate that no coverage reaches maps to rho = 1.  InferPartition
takes both roundings of B = tau_s * mu (Section 4.1.3): rounding up against the
bound tau_s, rounding down against the bound B / mu, and returns the smaller
coverage.

Pins (tests/test_partition_model.py): closed forms (B = 1 gives the mean; the
uniform case gives 1/(B+1)), Monte-Carlo minima of Beta samples, the variance
model at eta_bar = 0.5, monotonicity, a hand-worked instance of Eq. (1); for
InferPartition three instances worked by hand (either rounding deciding the
minimum, and one in which the rounding-down bound B / mu, not tau_s, decides);
for Algorithm 1 a brute-force scan of every cluster count that
evaluates Eq. (1) and Eq. (2) directly and locates the self-consistent
crossing the bisection must find; ten mistakes planted in a copy of this file
each fail the pins named for them.
"""
import math

import numpy as np
from scipy import integrate, stats


def piecewise_linear(knots_b, knots_t, b):
    """Linear interpolation between knots, linear extrapolation beyond them."""
    kb = np.asarray(knots_b, np.float64)
    kt = np.asarray(knots_t, np.float64)
    if len(kb) == 1:
        return float(kt[0])
    i = int(np.clip(np.searchsorted(kb, b, side="right") - 1, 0, len(kb) - 2))
    return float(kt[i] + (kt[i + 1] - kt[i]) * (b - kb[i]) / (kb[i + 1] - kb[i]))


def hybrid_latency(knots_b, t_cq, t_lut, b, eta):
    """Eq. (1)."""
    return piecewise_linear(knots_b, t_cq, b) + (1.0 - eta) * piecewise_linear(knots_b, t_lut, b)


def beta_params(mean, sigma_max2):
    var = 4.0 * sigma_max2 * mean * (1.0 - mean)
    nu = mean * (1.0 - mean) / var - 1.0
    return mean * nu, (1.0 - mean) * nu


def expected_min_hit_rate(mean, sigma_max2, B):
    """Eq. (2) by quadrature of the first-order-statistic density."""
    if mean <= 0.0:
        return 0.0
    if mean >= 1.0:
        return 1.0
    a, b = beta_params(mean, sigma_max2)
    dist = stats.beta(a, b)

    # Eq. (2) in the variable u = F(x) (du = f(x) dx, x = F^-1(u)):
    #   int_0^1 B x f(x) (1 - F(x))^(B-1) dx = int_0^1 B F^-1(u) (1 - u)^(B-1) du,
    # whose integrand is bounded whatever the Beta shape (f itself is singular at an
    # end point when a or b is below 1, which defeats direct quadrature in x).
    def integrand(u):
        return B * float(dist.ppf(u)) * (1.0 - u) ** (B - 1)

    pts = [p for p in (1e-9, 1e-6, 1e-3, 1.0 / (4 * B), 1.0 / B, 4.0 / B, 0.5) if 0.0 < p < 1.0]
    val, _ = integrate.quad(integrand, 0.0, 1.0, limit=800, points=sorted(set(pts)),
                            epsabs=1e-12, epsrel=1e-11)
    return float(val)


def mean_hit_rate_of_coverage(hit_cdf, rho):
    """hit_cdf[i] = share of accesses covered by the hottest i clusters, i = 0..nlist."""
    nlist = len(hit_cdf) - 1
    return float(hit_cdf[int(round(rho * nlist))])


def hitrate_to_coverage(hit_cdf, sigma_max2, B, eta_min):
    """Smallest coverage (in whole clusters) whose expected minimum hit rate in a
    batch of B reaches eta_min; brute-force scan over cluster counts."""
    nlist = len(hit_cdf) - 1
    if eta_min <= 0.0:
        return 0.0
    for i in range(nlist + 1):
        if expected_min_hit_rate(float(hit_cdf[i]), sigma_max2, B) >= eta_min:
            return i / nlist
    return 1.0


def infer_partition(knots_b, t_cq, t_lut, hit_cdf, sigma_max2, tau_s, mu):
    out = []
    for B, bound in ((max(1, math.ceil(tau_s * mu)), None), (max(1, math.floor(tau_s * mu)), "thr")):
        tcq = piecewise_linear(knots_b, t_cq, B)
        tlut = piecewise_linear(knots_b, t_lut, B)
        target = tau_s if bound is None else B / mu
        eta = (tcq + tlut - target) / tlut
        out.append(hitrate_to_coverage(hit_cdf, sigma_max2, B, eta) if eta <= 1.0 else 1.0)
    return min(out)


def partition_point(knots_b, t_cq, t_lut, hit_cdf, mem_index, sigma_max2, slo_search, eps,
                    mem_kvcache, mu_llm0, delta):
    """Algorithm 1.  mem_index[i] = bytes of the hottest i clusters."""
    nlist = len(hit_cdf) - 1
    tau_s = slo_search / (1.0 + eps)
    lo, hi = 0.0, 1.0
    rho = 0.0
    while hi - lo > delta:
        mid = 0.5 * (lo + hi)
        mem = float(mem_index[int(round(mid * nlist))])
        mu = max(0.0, (mem_kvcache - mem) / mem_kvcache) * mu_llm0
        rho = infer_partition(knots_b, t_cq, t_lut, hit_cdf, sigma_max2, tau_s, mu)
        if rho > mid:
            lo = mid
        else:
            hi = mid
    return rho
