// Latency-bounded choice of the partitioning point (Section 4.1): how much of
// the index (which fraction rho of the clusters, hottest first) to keep on the
// GPU so that the hybrid search meets its latency target.  Pure host
// arithmetic; it feeds ivf_index_load_partition.
//
//   * T_CQ(b), T_LUT(b): piecewise-linear CPU latency models from profiled knots
//     (Section 4.1.1), linear beyond the outer knots;
//   * Eq. (1): tau_s(b) = T_CQ(b) + (1 - eta) T_LUT(b), eta = smallest hit rate in the batch;
//   * per-query hit rate ~ Beta(mean eta_bar, variance 4 sigma_max^2 eta_bar (1 - eta_bar))
//     (Section 4.1.2);
//   * Eq. (2), the expected smallest of B draws.  Integrating Eq. (2) by parts,
//     int_0^1 B x f (1-F)^(B-1) dx = int_0^1 (1 - F(x))^B dx, which is the form
//     evaluated here (composite Simpson after an end-flattening substitution; F by
//     the continued fraction of the regularized incomplete beta function);
//   * its inverse over the measured hit-rate profile ("HitRate2Coverage"), by
//     bisection over whole clusters (the expected minimum grows with the mean);
//   * Algorithm 1.  The printed listing is garbled in places; the reading taken:
//     MEM_Index is evaluated at the midpoint rho_m, "t_s" is tau_s,
//     T_search = T_CQ + T_LUT, and the interval is bisected on the sign of
//     InferPartition(rho_m) - rho_m.
#include <math.h>
#include <stdint.h>

#include <algorithm>

#include "../../include/ivfpq_hot.h"

namespace {

double pw_linear(const ivf_latency_model_t *m, const double *t, double b) {
  const int n = m->n_knots;
  if (n == 1) return t[0];
  int i = 0;
  while (i < n - 2 && b >= m->batch[i + 1]) ++i;
  return t[i] + (t[i + 1] - t[i]) * (b - m->batch[i]) / (m->batch[i + 1] - m->batch[i]);
}

// Continued fraction for the incomplete beta function (modified Lentz).
double beta_cf(double a, double b, double x) {
  const double tiny = 1e-300, eps = 1e-15;
  const double qab = a + b, qap = a + 1.0, qam = a - 1.0;
  double c = 1.0, d = 1.0 - qab * x / qap;
  if (fabs(d) < tiny) d = tiny;
  d = 1.0 / d;
  double h = d;
  for (int it = 1; it <= 1000; ++it) {
    const int m2 = 2 * it;
    double aa = it * (b - it) * x / ((qam + m2) * (a + m2));
    d = 1.0 + aa * d;
    if (fabs(d) < tiny) d = tiny;
    c = 1.0 + aa / c;
    if (fabs(c) < tiny) c = tiny;
    d = 1.0 / d;
    h *= d * c;
    aa = -(a + it) * (qab + it) * x / ((a + m2) * (qap + m2));
    d = 1.0 + aa * d;
    if (fabs(d) < tiny) d = tiny;
    c = 1.0 + aa / c;
    if (fabs(c) < tiny) c = tiny;
    d = 1.0 / d;
    const double del = d * c;
    h *= del;
    if (fabs(del - 1.0) < eps) break;
  }
  return h;
}

// Regularized incomplete beta function I_x(a, b) = Beta CDF.
double beta_cdf(double a, double b, double x) {
  if (x <= 0.0) return 0.0;
  if (x >= 1.0) return 1.0;
  const double ln_front =
      lgamma(a + b) - lgamma(a) - lgamma(b) + a * log(x) + b * log1p(-x);
  const double front = exp(ln_front);
  if (x < (a + 1.0) / (a + b + 2.0)) return front * beta_cf(a, b, x) / a;
  return 1.0 - front * beta_cf(b, a, 1.0 - x) / b;
}

double min_hit_rate(double mean, double sigma_max2, int B) {
  if (mean <= 0.0) return 0.0;
  if (mean >= 1.0) return 1.0;
  if (B < 1) B = 1;
  const double var = 4.0 * sigma_max2 * mean * (1.0 - mean);
  const double nu = mean * (1.0 - mean) / var - 1.0;  // = 1 / (4 sigma_max^2) - 1
  const double a = mean * nu, b = (1.0 - mean) * nu;
  // Simpson in t with x = t^6 / (t^6 + (1-t)^6): the substitution flattens the
  // x^a and (1-x)^b behaviour of F at the ends (a or b may be below 1), where the
  // integrand times dx/dt vanishes.
  const int N = 4096;
  double s = 0.0;
  for (int i = 1; i < N; ++i) {
    const double t = (double)i / N, u = 1.0 - t;
    const double t5 = t * t * t * t * t, u5 = u * u * u * u * u;
    const double den = t5 * t + u5 * u;
    const double x = t5 * t / den;
    const double dxdt = 6.0 * t5 * u5 / (den * den);
    s += pow(1.0 - beta_cdf(a, b, x), (double)B) * dxdt * ((i & 1) ? 4.0 : 2.0);
  }
  return s / (3.0 * N);
}

double hitrate_to_coverage(const double *hit_cdf, int nlist, double sigma_max2, int B,
                           double eta_min) {
  if (eta_min <= 0.0) return 0.0;
  if (min_hit_rate(hit_cdf[nlist], sigma_max2, B) < eta_min) return 1.0;
  int lo = 0, hi = nlist;  // invariant: hi reaches the target, lo - 1 ... does not (lo may)
  while (lo < hi) {
    const int mid = (lo + hi) / 2;
    if (min_hit_rate(hit_cdf[mid], sigma_max2, B) >= eta_min) hi = mid;
    else lo = mid + 1;
  }
  return (double)lo / nlist;
}

double infer_partition(const ivf_latency_model_t *m, const double *hit_cdf, int nlist,
                       double sigma_max2, double tau_s, double mu) {
  double best = 1.0;
  for (int pass = 0; pass < 2; ++pass) {
    double Bd = pass == 0 ? ceil(tau_s * mu) : floor(tau_s * mu);
    if (Bd < 1.0) Bd = 1.0;
    const int B = (int)Bd;
    const double tcq = pw_linear(m, m->t_cq, Bd), tlut = pw_linear(m, m->t_lut, Bd);
    const double target = pass == 0 ? tau_s : Bd / mu;  // rounding down: keep the throughput
    const double eta = (tcq + tlut - target) / tlut;
    const double rho = eta <= 1.0 ? hitrate_to_coverage(hit_cdf, nlist, sigma_max2, B, eta) : 1.0;
    best = std::min(best, rho);
  }
  return best;
}

bool model_ok(const ivf_latency_model_t *m) {
  if (!m || m->n_knots < 1 || !m->batch || !m->t_cq || !m->t_lut) return false;
  for (int i = 1; i < m->n_knots; ++i)
    if (!(m->batch[i] > m->batch[i - 1])) return false;
  return true;
}

}  // namespace

extern "C" double ivf_model_hybrid_latency(const ivf_latency_model_t *m, double batch,
                                           double eta) {
  if (!model_ok(m)) return NAN;
  return pw_linear(m, m->t_cq, batch) + (1.0 - eta) * pw_linear(m, m->t_lut, batch);
}

extern "C" double ivf_model_min_hit_rate(double mean_hit_rate, double sigma_max2, int32_t batch) {
  if (!(sigma_max2 > 0.0) || sigma_max2 >= 0.25) return NAN;
  return min_hit_rate(mean_hit_rate, sigma_max2, batch);
}

extern "C" double ivf_model_hitrate_to_coverage(const double *hit_cdf, int32_t nlist,
                                                double sigma_max2, int32_t batch,
                                                double eta_min) {
  if (!hit_cdf || nlist < 1 || !(sigma_max2 > 0.0) || sigma_max2 >= 0.25) return NAN;
  return hitrate_to_coverage(hit_cdf, nlist, sigma_max2, batch, eta_min);
}

extern "C" int ivf_model_partition_point(const ivf_latency_model_t *m, const double *hit_cdf,
                                         const double *mem_index, int32_t nlist,
                                         double sigma_max2, double slo_search, double eps,
                                         double mem_kvcache, double mu_llm0, double delta,
                                         double *rho_out) {
  if (!model_ok(m) || !hit_cdf || !mem_index || !rho_out || nlist < 1 || !(sigma_max2 > 0.0) ||
      sigma_max2 >= 0.25 || !(slo_search > 0.0) || !(eps >= 0.0) || !(mem_kvcache > 0.0) ||
      !(mu_llm0 > 0.0) || !(delta > 0.0))
    return IVF_EINVAL;
  const double tau_s = slo_search / (1.0 + eps);
  double lo = 0.0, hi = 1.0, rho = 0.0;
  while (hi - lo > delta) {
    const double mid = 0.5 * (lo + hi);
    const double mem = mem_index[(int)llround(mid * nlist)];
    const double mu = std::max(0.0, (mem_kvcache - mem) / mem_kvcache) * mu_llm0;
    rho = infer_partition(m, hit_cdf, nlist, sigma_max2, tau_s, mu);
    if (rho > mid) lo = mid;
    else hi = mid;
  }
  *rho_out = rho;
  return IVF_OK;
}
