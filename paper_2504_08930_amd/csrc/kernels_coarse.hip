// Stage 1 of IVF search (Section 2.2): coarse quantization.  Every query is
// scored against every centroid as a dense contraction on the fp32 matrix
// cores (v_mfma_f32_32x32x2f32), then the nprobe best clusters per query are
// selected exactly by a radix select over (score, cluster id).
//
// The paper keeps this stage on the CPU to avoid ping-pong between devices
// when several GPU shards are used (Section 4.2.1); with one GPU that concern
// does not arise and the contraction runs on the device.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace ivf {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------
// squared norms of the centroids (L2 metric: score = |c|^2 - 2 q.c, which
// ranks like |q - c|^2 for a fixed query)
// ---------------------------------------------------------------------------
__global__ void k_cent_norms(const float *__restrict__ cent, int nlist, int d,
                             float *__restrict__ out) {
  const int c = blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (c >= nlist) return;
  float s = 0.0f;
  for (int i = lane; i < d; i += 64) {
    float v = cent[(size_t)c * d + i];
    s = __builtin_fmaf(v, v, s);
  }
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (lane == 0) out[c] = s;
}

hipError_t launch_cent_norms(const float *cent, int nlist, int d, float *out, hipStream_t st) {
  hipLaunchKernelGGL(k_cent_norms, dim3((nlist + 3) / 4), dim3(256), 0, st, cent, nlist, d, out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// scores[q][c] = q . c            (IP, larger is better)
//              = |c|^2 - 2 q . c  (L2, smaller is better)
// 128 x 128 block tile, 4 waves in a 2 x 2 arrangement, each wave 64 x 64 as
// 2 x 2 MFMA tiles of 32 x 32; K is consumed 16 at a time through LDS.
// ---------------------------------------------------------------------------
constexpr int kBM = 128, kBN = 128, kBK = 16, kLdk = kBK + 4;

__global__ __launch_bounds__(256) void k_coarse_gemm(const float *__restrict__ Q, int nq,
                                                     const float *__restrict__ C, int nlist, int d,
                                                     const float *__restrict__ cnorm, int metric_ip,
                                                     float *__restrict__ scores) {
  __shared__ __align__(16) float As[2][kBM * kLdk];
  __shared__ __align__(16) float Bs[2][kBN * kLdk];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int row0 = blockIdx.y * kBM;   // queries
  const int col0 = blockIdx.x * kBN;   // centroids

  // global -> LDS assignment: float4 f = tid + 256 * i, row = f / 4, c4 = f % 4
  float4 ga[2], gb[2];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int f = tid + 256 * i;
      const int r = f >> 2, c4 = f & 3;
      const int qa = row0 + r, cb = col0 + r;
      ga[i] = qa < nq ? *reinterpret_cast<const float4 *>(Q + (size_t)qa * d + k0 + c4 * 4)
                      : make_float4(0.f, 0.f, 0.f, 0.f);
      gb[i] = cb < nlist ? *reinterpret_cast<const float4 *>(C + (size_t)cb * d + k0 + c4 * 4)
                         : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int f = tid + 256 * i;
      const int r = f >> 2, c4 = f & 3;
      *reinterpret_cast<float4 *>(&As[buf][r * kLdk + c4 * 4]) = ga[i];
      *reinterpret_cast<float4 *>(&Bs[buf][r * kLdk + c4 * 4]) = gb[i];
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  const int nk = d / kBK;  // d is a multiple of 16
  gload(0);
  sstore(0);
  __syncthreads();
  const int li = lane & 31, kk = lane >> 5;
  for (int kc = 0; kc < nk; ++kc) {
    const int buf = kc & 1;
    if (kc + 1 < nk) gload((kc + 1) * kBK);
    // lane (li, kk) feeds k = kk*8 + s at MFMA step s: A and B use the same
    // permutation of k, so the contraction is unchanged.
    float a[2][8], b[2][8];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const float *pa = &As[buf][(wm * 64 + t * 32 + li) * kLdk + kk * 8];
      const float *pb = &Bs[buf][(wn * 64 + t * 32 + li) * kLdk + kk * 8];
      const float4 a0 = *reinterpret_cast<const float4 *>(pa);
      const float4 a1 = *reinterpret_cast<const float4 *>(pa + 4);
      const float4 b0 = *reinterpret_cast<const float4 *>(pb);
      const float4 b1 = *reinterpret_cast<const float4 *>(pb + 4);
      a[t][0] = a0.x; a[t][1] = a0.y; a[t][2] = a0.z; a[t][3] = a0.w;
      a[t][4] = a1.x; a[t][5] = a1.y; a[t][6] = a1.z; a[t][7] = a1.w;
      b[t][0] = b0.x; b[t][1] = b0.y; b[t][2] = b0.z; b[t][3] = b0.w;
      b[t][4] = b1.x; b[t][5] = b1.y; b[t][6] = b1.z; b[t][7] = b1.w;
    }
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
          acc[mt][nt] =
              __builtin_amdgcn_mfma_f32_32x32x2f32(a[mt][s], b[nt][s], acc[mt][nt], 0, 0, 0);
    if (kc + 1 < nk) sstore(buf ^ 1);
    __syncthreads();
  }

  // D[i][j]: register r of lane l holds i = 8*(r/4) + 4*(l/32) + r%4, j = l%32
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const int c = col0 + wn * 64 + nt * 32 + li;
      const float cn = (!metric_ip && c < nlist) ? cnorm[c] : 0.0f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qi = row0 + wm * 64 + mt * 32 + 8 * (r >> 2) + 4 * kk + (r & 3);
        if (qi < nq && c < nlist) {
          const float dot = acc[mt][nt][r];
          scores[(size_t)qi * nlist + c] = metric_ip ? dot : __builtin_fmaf(-2.0f, dot, cn);
        }
      }
    }
}

hipError_t launch_coarse_gemm(const Shape &sh, const float *q, int nq, const float *cent,
                              const float *cent_norm, float *scores, hipStream_t st) {
  dim3 grid((sh.nlist + kBN - 1) / kBN, (nq + kBM - 1) / kBM);
  hipLaunchKernelGGL(k_coarse_gemm, grid, dim3(256), 0, st, q, nq, cent, sh.nlist, sh.d,
                     cent_norm, sh.metric_ip, scores);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Exact per-query selection of the `keep` best (score, id) pairs, best first,
// ties to the smaller cluster id.  64-bit key = ordered score bits : id; an
// MSB-first radix select finds the keep-th smallest key, a final pass collects
// everything not larger and a bitonic sort orders it.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t score_bits(float s, int metric_ip) {
  uint32_t u = __float_as_uint(s);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending with s
  return metric_ip ? ~u : u;                        // IP: larger score first
}

constexpr int kSelThreads = 512;
constexpr int kSelBins = 2048;  // 11-bit digits
constexpr int kSelBinsPerThread = kSelBins / kSelThreads;

__device__ __forceinline__ unsigned long long sel_key(float s, int metric_ip, int c) {
  return ((unsigned long long)score_bits(s, metric_ip) << 32) | (unsigned)c;
}

__global__ __launch_bounds__(kSelThreads) void k_coarse_select(const float *__restrict__ scores,
                                                               int nlist, int metric_ip, int keep,
                                                               int nprobe, int stride, int n2,
                                                               int32_t *__restrict__ probe) {
  __shared__ unsigned int hist[kSelBins];
  __shared__ unsigned int wsum[kSelThreads / 64];
  __shared__ unsigned long long s_prefix, s_mask;
  __shared__ unsigned int s_need, s_done, s_count;
  extern __shared__ unsigned long long sel[];  // n2 entries
  const int q = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const float *row = scores + (size_t)q * nlist;
  int32_t *out = probe + (size_t)q * stride;

  if (tid == 0) {
    s_prefix = 0ull;
    s_mask = 0ull;
    s_need = (unsigned)keep;
    s_done = 0u;
    s_count = 0u;
  }
  unsigned long long thr = ~0ull;
  if (keep < nlist) {
    // digits of the 64-bit key, most significant first: (shift, bits)
    const int shifts[6] = {53, 42, 32, 21, 10, 0};
    const int widths[6] = {11, 11, 10, 11, 11, 10};
    for (int pass = 0; pass < 6; ++pass) {
      const int shift = shifts[pass];
      const unsigned dmask = (1u << widths[pass]) - 1u;
#pragma unroll
      for (int b = 0; b < kSelBinsPerThread; ++b) hist[tid * kSelBinsPerThread + b] = 0u;
      __syncthreads();
      const unsigned long long prefix = s_prefix, mask = s_mask;
      const unsigned need = s_need;
      if (s_done) break;
      for (int c = tid; c < nlist; c += kSelThreads) {
        const unsigned long long key = sel_key(row[c], metric_ip, c);
        if ((key & mask) == prefix) atomicAdd(&hist[(unsigned)(key >> shift) & dmask], 1u);
      }
      __syncthreads();
      // block-wide exclusive scan of per-thread bin sums
      unsigned loc[kSelBinsPerThread], tsum = 0;
#pragma unroll
      for (int b = 0; b < kSelBinsPerThread; ++b) {
        loc[b] = hist[tid * kSelBinsPerThread + b];
        tsum += loc[b];
      }
      unsigned incl = tsum;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const unsigned v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
      }
      if (lane == 63) wsum[wave] = incl;
      __syncthreads();
      unsigned before = incl - tsum;
      for (int w2 = 0; w2 < wave; ++w2) before += wsum[w2];
      // the thread whose bins straddle rank `need` publishes the bucket
      if (before < need && need <= before + tsum) {
        unsigned cum = before;
        int b = 0;
        for (; b < kSelBinsPerThread - 1; ++b) {
          if (cum + loc[b] >= need) break;
          cum += loc[b];
        }
        const unsigned bucket = (unsigned)(tid * kSelBinsPerThread + b);
        s_need = need - cum;
        s_prefix = prefix | ((unsigned long long)bucket << shift);
        s_mask = mask | ((unsigned long long)dmask << shift);
        if (loc[b] == need - cum || pass == 5) s_done = 1u;  // whole bucket is selected
      }
      __syncthreads();
    }
    __syncthreads();
    // threshold: prefix with all undecided low bits set
    thr = s_prefix | ~s_mask;
  }
  for (int i = tid; i < n2; i += kSelThreads) sel[i] = ~0ull;
  __syncthreads();
  for (int c = tid; c < nlist; c += kSelThreads) {
    const unsigned long long key = sel_key(row[c], metric_ip, c);
    if (key <= thr) {
      const unsigned slot = atomicAdd(&s_count, 1u);
      if (slot < (unsigned)n2) sel[slot] = key;
    }
  }
  __syncthreads();
  for (int size = 2; size <= n2; size <<= 1) {
    for (int st = size >> 1; st > 0; st >>= 1) {
      for (int i = tid; i < n2; i += kSelThreads) {
        const int j = i ^ st;
        if (j > i) {
          const bool asc = (i & size) == 0;
          const unsigned long long a = sel[i], b = sel[j];
          if ((b < a) == asc) {
            sel[i] = b;
            sel[j] = a;
          }
        }
      }
      __syncthreads();
    }
  }
  for (int p = tid; p < nprobe; p += kSelThreads)
    out[p] = p < keep ? (int32_t)(sel[p] & 0xffffffffull) : -1;
}

hipError_t launch_coarse_select(const Shape &sh, const float *scores, int nq, int nprobe,
                                int probe_stride, int32_t *probe, hipStream_t st) {
  const int keep = nprobe < sh.nlist ? nprobe : sh.nlist;
  int n2 = 2;
  while (n2 < keep) n2 <<= 1;
  hipLaunchKernelGGL(k_coarse_select, dim3(nq), dim3(kSelThreads), (size_t)n2 * 8, st, scores,
                     sh.nlist, sh.metric_ip, keep, nprobe, probe_stride, n2, probe);
  return hipGetLastError();
}

}  // namespace ivf
