// Two-way fp16 split of one fp32 row by one wavefront (device code shared by the
// stand-alone split kernel and the query-preparation launch).
//
// The row is scaled by a power of two 2^e (exact) that puts its largest magnitude
// in [2^8, 2^9); then x * 2^e = h1 + h2 + rest with h1 = fp16(x * 2^e),
// h2 = fp16(x * 2^e - h1), |rest| <= 2^-22 |x * 2^e| (2 x 11 significand bits of
// fp32's 24; entries 2^12 below the row maximum lose a little more to fp16's
// exponent range, far below anything a dot product with that row can resolve).
// Output layout, chunk-major so that the K = 16 chunk of a row tile is one
// contiguous block: for row r and group g of 8 consecutive k, two 16-byte units
// (h1, h2) at unit index ((g / 2) * rows + r) * 4 + (g % 2) * 2 + part.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

namespace ivf {

typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ void split_row_f16(const float *__restrict__ src, size_t rows,
                                              int groups_per_row, uint4 *__restrict__ dst,
                                              int32_t *__restrict__ row_exp, size_t row,
                                              int lane) {
  const float4 *in = reinterpret_cast<const float4 *>(src + row * (size_t)groups_per_row * 8);
  float mx = 0.0f;
  for (int g = lane; g < groups_per_row; g += 64) {
    const float4 lo = in[g * 2], hi = in[g * 2 + 1];
    mx = fmaxf(mx, fmaxf(fmaxf(fabsf(lo.x), fabsf(lo.y)), fmaxf(fabsf(lo.z), fabsf(lo.w))));
    mx = fmaxf(mx, fmaxf(fmaxf(fabsf(hi.x), fabsf(hi.y)), fmaxf(fabsf(hi.z), fabsf(hi.w))));
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  int e = 0;
  if (mx > 0.0f && mx < INFINITY) {
    int ex;
    (void)frexpf(mx, &ex);  // mx = f * 2^ex, f in [0.5, 1)
    e = 9 - ex;             // mx * 2^e in [2^8, 2^9)
  }
  if (lane == 0) row_exp[row] = e;
  for (int g = lane; g < groups_per_row; g += 64) {
    const float4 lo = in[g * 2], hi = in[g * 2 + 1];
    const float x[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    halfx8 h1, h2;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float v = ldexpf(x[i], e);
      const _Float16 a = (_Float16)v;      // round to nearest even
      h1[i] = a;
      h2[i] = (_Float16)(v - (float)a);    // the difference is exact in fp32
    }
    const size_t out = ((size_t)(g >> 1) * rows + row) * 4 + (size_t)(g & 1) * 2;
    dst[out] = __builtin_bit_cast(uint4, h1);
    dst[out + 1] = __builtin_bit_cast(uint4, h2);
  }
}

// A split job riding along with another launch of 256-thread blocks: block b's
// wavefront w takes rows 4 * b + w, 4 * (b + blocks) + w, ...  rows == 0: none.
struct SplitJob {
  const float *src;
  uint4 *dst;
  int32_t *row_exp;
  int rows;
  int groups_per_row;
};

__device__ __forceinline__ void run_split_job(const SplitJob &job) {
  if (job.rows <= 0) return;  // uniform
  const size_t blocks = (size_t)gridDim.x * gridDim.y * gridDim.z;
  const size_t b = ((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (size_t row = b * 4 + wave; row < (size_t)job.rows; row += blocks * 4)
    split_row_f16(job.src, (size_t)job.rows, job.groups_per_row, job.dst, job.row_exp, row, lane);
}

}  // namespace ivf
