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
//
// Residual encoding (codes hold x - centroid of the list): the distance to the
// decoded vector centroid + r splits into
//   IP:  q.c + q.r                      = bias(q, list) + table sum
//   L2:  |q-c|^2 + (|r|^2 + 2 c.r) - 2 q.r = bias(q, list) + pv(vector) + table sum
// with ONE table per query (entries -q_m.cb, resp. -2 q_m.cb); bias and the
// per-vector term pv are quantized with the same scale and added as integers,
// so the sum stays exact and order-independent.  B then also covers the largest
// |bias| among the query's probes and the largest |pv| of the index.
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

// Table kinds
constexpr int kLutL2 = 0;      // entry = sum_t (q_t - c_t)^2
constexpr int kLutIP = 1;      // entry = -(sum_t q_t * c_t)
constexpr int kLutL2Res = 2;   // entry = -2 * (sum_t q_t * c_t)   (residual-encoded L2)

// One table entry.  Sequential fused multiply-adds in index order
// (bit-identical on host and device).
IVF_HD inline float lut_entry(int kind, const float *q, const float *c, int dsub) {
  float acc = 0.0f;
  if (kind != kLutL2) {
    for (int t = 0; t < dsub; ++t) acc = __builtin_fmaf(q[t], c[t], acc);
    return kind == kLutIP ? -acc : -2.0f * acc;
  }
  for (int t = 0; t < dsub; ++t) {
    float diff = q[t] - c[t];
    acc = __builtin_fmaf(diff, diff, acc);
  }
  return acc;
}

// 4-bit codes: entry of a code byte's column = sum of the entries of the two
// sub-quantizers packed in the byte (low half first).  A plain float addition,
// never fused with the producers of a or b, so host and device agree bit for bit.
IVF_HD inline float lut_pair_entry(float a, float b) {
#pragma clang fp contract(off)
  return a + b;
}

// Scale exponent from the largest |entry| of the query's table (plus, with
// residual encoding, the largest |bias| of the query and |pv| of the index):
// B = M * maxabs + max_bias + max_pv = f * 2^x with f in [0.5, 1)
//   =>  B * 2^(30 - x) <= 2^30.
IVF_HD inline int lut_exponent(float maxabs, int M, float max_bias = 0.0f, float max_pv = 0.0f) {
  const double B = (double)M * (double)maxabs + (double)max_bias + (double)max_pv;
  if (!(B > 0.0)) return 0;
  const uint64_t bits = __builtin_bit_cast(uint64_t, B);
  int x = (int)((bits >> 52) & 0x7ff) - 1022;
  int e = 30 - x;
  if (e > 60) e = 60;
  if (e < -60) e = -60;
  return e;
}

// Total: a value that is not finite or does not fit (only possible for a query
// that is itself not finite) quantizes to 0 on host and device alike.
IVF_HD inline int lut_quantize(float v, int e) {
  const float r = __builtin_rintf(__builtin_ldexpf(v, e));
  return __builtin_fabsf(r) < 2147483520.0f ? (int)r : 0;
}

// Residual encoding: the (query, centroid) term is the sum of 64 partial sums,
// combined by a fixed xor-butterfly (residual_bias_combine), the same on host
// and device.  Partial sum `lane` runs over the groups of four consecutive
// elements 4*lane + 256*j (j = 0, 1, ...), each group in index order, so that on
// the device a lane reads 16 bytes at a time and a wavefront 1 KB; d is a
// multiple of 16 (it is a multiple of M, and M of 16).
IVF_HD inline float residual_bias_step(int metric_ip, float q, float c, float acc) {
  if (metric_ip) return __builtin_fmaf(q, c, acc);
  const float diff = q - c;
  return __builtin_fmaf(diff, diff, acc);
}

IVF_HD inline float residual_bias_part(int metric_ip, const float *q, const float *c, int d,
                                       int lane) {
  float acc = 0.0f;
  for (int i = 4 * lane; i < d; i += 256)
    for (int t = 0; t < 4; ++t) acc = residual_bias_step(metric_ip, q[i + t], c[i + t], acc);
  return acc;
}

// Host form of the butterfly: part[64] -> total (every slot ends up equal).
inline float residual_bias_combine(float *part) {
  for (int o = 32; o > 0; o >>= 1) {
    float nxt[64];
    for (int l = 0; l < 64; ++l) nxt[l] = part[l] + part[l ^ o];
    for (int l = 0; l < 64; ++l) part[l] = nxt[l];
  }
  return part[0];
}

// bias(q, list): IP -> -(q.c), L2 -> |q - c|^2.
inline float residual_bias_host(int metric_ip, const float *q, const float *c, int d) {
  float part[64];
  for (int l = 0; l < 64; ++l) part[l] = residual_bias_part(metric_ip, q, c, d, l);
  const float t = residual_bias_combine(part);
  return metric_ip ? -t : t;
}

// Per-vector term of residual-encoded L2: |r|^2 + 2 c.r for the decoded residual r.
IVF_HD inline float residual_pv_accumulate(float acc, const float *r, const float *c, int n) {
  for (int t = 0; t < n; ++t) {
    acc = __builtin_fmaf(r[t], r[t], acc);
    acc = __builtin_fmaf(2.0f * c[t], r[t], acc);
  }
  return acc;
}

// Integer code sum -> reported distance.
IVF_HD inline float key_to_dist(int key, int e, int metric_ip) {
  float d = __builtin_ldexpf((float)key, -e);
  return metric_ip ? -d : d;
}

}  // namespace ivf
