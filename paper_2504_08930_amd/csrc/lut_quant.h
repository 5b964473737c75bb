// Fixed-point lookup-table arithmetic shared by the GPU kernels and the
// library's CPU scan of cold clusters.
//
// The per-query table of partial distances between the query and the PQ
// codewords (Section 2.2, second stage) is computed in fp32 with one fixed
// operation order, then scaled by a per-query power of two and rounded to
// int32.  A code's distance is the integer sum of its M table entries, so the
// sum is exact and independent of the order in which sub-quantizers are
// visited.  That is what lets the GPU scan visit them in a lane-rotated,
// bank-conflict-free order while the CPU scan visits them in natural order,
// and both return bit-identical distances.  For the inner product the table
// holds the negated partial products, so "smaller is better" everywhere.
//
// Error bound: with B = M * max_{m,j} |T[m][j]| (no code sum can exceed it)
// and e chosen so that B * 2^e <= 2^30, every entry is off by at most
// 2^-(e+1), the sum by at most M * 2^-(e+1) <= M * B / 2^30
// (~ 9e-8 * B at M = 96).
#pragma once
#include <math.h>
#include <stdint.h>
#include <string.h>

#if defined(__HIPCC__)
#define IVF_HD __host__ __device__
#else
#define IVF_HD
#endif

namespace ivf {

constexpr int kKeyInvalid = 0x7fffffff;  // larger than any valid code sum

// One table entry: L2 -> sum_t (q_t - c_t)^2, IP -> -(sum_t q_t * c_t).
// Sequential fused multiply-adds in index order (bit-identical on host and device).
IVF_HD inline float lut_entry(int metric_ip, const float *q, const float *c, int dsub) {
  float acc = 0.0f;
  if (metric_ip) {
    for (int t = 0; t < dsub; ++t) acc = __builtin_fmaf(q[t], c[t], acc);
    return -acc;
  }
  for (int t = 0; t < dsub; ++t) {
    float diff = q[t] - c[t];
    acc = __builtin_fmaf(diff, diff, acc);
  }
  return acc;
}

// Scale exponent from the largest |entry| of the query's table:
// B = M * maxabs = f * 2^x with f in [0.5, 1)  =>  B * 2^(30 - x) <= 2^30.
IVF_HD inline int lut_exponent(float maxabs, int M) {
  const double B = (double)M * (double)maxabs;
  if (!(B > 0.0)) return 0;
  const uint64_t bits = __builtin_bit_cast(uint64_t, B);
  int x = (int)((bits >> 52) & 0x7ff) - 1022;
  int e = 30 - x;
  if (e > 60) e = 60;
  if (e < -60) e = -60;
  return e;
}

IVF_HD inline int lut_quantize(float v, int e) {
  return (int)__builtin_rintf(__builtin_ldexpf(v, e));
}

// Integer code sum -> reported distance.
IVF_HD inline float key_to_dist(int key, int e, int metric_ip) {
  float d = __builtin_ldexpf((float)key, -e);
  return metric_ip ? -d : d;
}

}  // namespace ivf
