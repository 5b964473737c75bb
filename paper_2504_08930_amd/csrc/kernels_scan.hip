// Routing, lookup-table construction, ADC scan, top-k merge, and the code-tile
// layout transform, for gfx950 (wave64, 160 KB LDS per CU).
//
// Stage numbering follows Section 2.2 ("Search Operation in IVF Index"):
// stage 2 builds the per-query table of partial distances, stage 3 scans the
// codes of the probed clusters through it and keeps the k best.  Routing of
// probes by the mapping table follows Section 4.2.1.
//
// ADC scan design (what differs from the one-thread-block-per-(query, cluster)
// scheme the paper describes for its GPU tier in Section 3.1):
//  * one block serves one query and walks ALL of that query's resident probes
//    (or a 1/S slice of their tiles), so the table is staged in LDS once per
//    block instead of once per probed cluster;
//  * codes are stored in 64-vector tiles, one lane per vector, 16-byte units
//    interleaved across lanes, so every global load instruction is a fully
//    coalesced 1 KB read;
//  * the table is stored code-major ([code][column], 64 columns per row) and
//    each lane visits the sub-quantizers of a 32-wide group in the order
//    column = lane XOR step.  For a fixed step the 32 lanes of a half-wave hit
//    32 different LDS banks whatever the code values are: lookups are
//    conflict-free by construction.  The codes are stored pre-permuted to match
//    (see src_subq), so no register shuffling is needed at scan time;
//  * the LDS address of a lookup is assembled by one byte-permute instruction
//    (code byte -> address bits 8..15, lane column -> bits 0..7);
//  * table entries are int32 fixed point (lut_quant.h), so the visiting order
//    does not change the sum.
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>

#include "internal.h"
#include "lut_quant.h"
#include "split_f16.h"

namespace ivf {

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool cand_less(int ka, long long ia, int kb, long long ib) {
  return ka < kb || (ka == kb && ia < ib);
}

// Read an int at a raw LDS byte address.  The scan kernel's dynamic LDS block
// is the kernel's only LDS and therefore starts at address 0, so table offsets
// are LDS addresses; going through an address-space-3 pointer keeps the
// compiler from adding a (zero) base to every lookup.
typedef const __attribute__((address_space(3))) int *lds_int_ptr;
__device__ __forceinline__ int lds_read_i32(uint32_t addr) {
  return *reinterpret_cast<lds_int_ptr>(static_cast<uintptr_t>(addr));
}

__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// In-place ascending bitonic sort of n (power of two) candidates held in LDS.
// BLOCK = true: all threads of the block take part, separated by __syncthreads;
// BLOCK = false: one wavefront sorts its own private range.
template <bool BLOCK>
__device__ void bitonic_sort_lds(int *keys, long long *ids, int n, int tid, int nthreads) {
  for (int size = 2; size <= n; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int i = tid; i < n; i += nthreads) {
        int j = i ^ stride;
        if (j > i) {
          bool asc = (i & size) == 0;
          int ka = keys[i], kb = keys[j];
          long long ia = ids[i], ib = ids[j];
          bool b_first = cand_less(kb, ib, ka, ia);
          if (b_first == asc) {
            keys[i] = kb; ids[i] = ib;
            keys[j] = ka; ids[j] = ia;
          }
        }
      }
      if (BLOCK) __syncthreads(); else wave_sync();
    }
  }
}

__global__ void k_fill_u32(uint32_t *p, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t step = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) p[i] = v;
}

hipError_t launch_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t st) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, st, p, n, v);
  return hipGetLastError();
}

// Plain streaming copy of known size: the reference against which hardware
// byte counters are calibrated.
__global__ void k_calib_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t step = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) dst[i] = src[i];
}

// Plain streaming read (each thread folds what it reads into one word and
// stores it once): the achievable read bandwidth of the machine, the practical
// ceiling for the scan.
__global__ void k_calib_read(const uint4 *__restrict__ src, size_t n, uint32_t *__restrict__ sink) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t step = (size_t)gridDim.x * blockDim.x;
  uint32_t acc = 0;
  for (; i + 3 * step < n; i += 4 * step) {
    const uint4 a = src[i], b = src[i + step], c = src[i + 2 * step], d = src[i + 3 * step];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^
           d.z ^ d.w;
  }
  for (; i < n; i += step) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

constexpr int kCalibBlocks = 256 * 8, kCalibThreads = 256;
static_assert((size_t)kCalibBlocks * kCalibThreads * 4 == IVF_CALIB_SINK_BYTES,
              "the read kernel's sink: one word per launched thread");

hipError_t launch_calib_copy(const void *src, void *dst, size_t bytes, hipStream_t st) {
  const size_t n = bytes / 16;
  if (n == 0) return hipSuccess;
  if (src == dst || bytes < (size_t)kCalibBlocks * kCalibThreads * 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_calib_copy, dim3(kCalibBlocks), dim3(kCalibThreads), 0, st,
                     (const uint4 *)src, (uint4 *)dst, n);
  return hipGetLastError();
}

hipError_t launch_calib_read(const void *src, void *sink, size_t bytes, hipStream_t st) {
  const size_t n = bytes / 16;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_calib_read, dim3(kCalibBlocks), dim3(kCalibThreads), 0, st,
                     (const uint4 *)src, n, (uint32_t *)sink);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Residual encoding: bias(q, probe) = -(q.c) (IP) or |q - c|^2 (L2) for every
// probe, one wavefront per (query, probe); partial sums and butterfly order
// as in lut_quant.h so the CPU scan gets the same bits.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_bias(const float *__restrict__ q, int nq, int d,
                                              const int32_t *__restrict__ probe, int nprobe,
                                              int stride, const float *__restrict__ cent,
                                              int metric_ip, float *__restrict__ bias) {
  const long long w = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (w >= (long long)nq * nprobe) return;
  const int qi = (int)(w / nprobe), p = (int)(w % nprobe);
  const int c = probe[(size_t)qi * stride + p];
  float t = 0.0f;
  if (c >= 0) {
    // residual_bias_part with 16-byte loads: the same elements in the same order
    const float4 *q4 = reinterpret_cast<const float4 *>(q + (size_t)qi * d);
    const float4 *c4 = reinterpret_cast<const float4 *>(cent + (size_t)c * d);
    for (int i = lane; i < (d >> 2); i += 64) {
      const float4 a = q4[i], b = c4[i];
      t = residual_bias_step(metric_ip, a.x, b.x, t);
      t = residual_bias_step(metric_ip, a.y, b.y, t);
      t = residual_bias_step(metric_ip, a.z, b.z, t);
      t = residual_bias_step(metric_ip, a.w, b.w, t);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o, 64);
    if (metric_ip) t = -t;
  }
  if (lane == 0) bias[(size_t)qi * stride + p] = t;
}

hipError_t launch_bias(const Shape &sh, const float *q, int nq, const int32_t *probe, int nprobe,
                       int probe_stride, const float *centroids, float *bias, hipStream_t st) {
  const long long waves = (long long)nq * nprobe;
  hipLaunchKernelGGL(k_bias, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, q, nq, sh.d,
                     probe, nprobe, probe_stride, centroids, sh.metric_ip, bias);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Routing (Section 4.2.1): each probe is looked up in the mapping table;
// resident probes form the query's GPU work list, the others its cold list.
// Also the router's counters (Section 4.2.3).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_route(
    const int32_t *__restrict__ probe, int nq, int nprobe, int stride,
    const int32_t *__restrict__ clus_tile, const int32_t *__restrict__ clus_len, int M,
    int32_t *g_base, int32_t *g_len, int32_t *g_prefix, int32_t *g_n, int32_t *cold,
    int32_t *n_cold, int32_t *q_vecs, const float *__restrict__ bias, float *g_bias, float *qbmax,
    unsigned long long *hits, int count_stats, int n2, const uint32_t *__restrict__ lutpart,
    int nparts, uint32_t *__restrict__ lutmax) {
  // One wavefront per query, one lane per probe (64 probes per step).  The
  // probes are first put in cluster-id order (n2 > 0: a bitonic sort of
  // (id, rank) words in LDS), so that the work lists of queries that share
  // lists name them in the same order: such queries, scheduled side by side,
  // then stream the same tiles at about the same time and share them in L2.
  // The result of a query does not depend on the order of its lists.
  extern __shared__ int32_t route_sort[];
  const int q = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (q >= nq) return;
  const int32_t *pr = probe + (size_t)q * stride;
  if (nparts > 0) {
    // largest |entry| of the query's lookup table, from the partial maxima the
    // table kernel left (the tables depend on the queries only and are built first)
    uint32_t mx = 0;
    for (int i = lane; i < nparts; i += 64) mx = max(mx, lutpart[(size_t)q * kLutMaxParts + i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
    if (lane == 0) lutmax[q] = mx;
  }
  int32_t *srt = route_sort + (threadIdx.x >> 6) * n2;
  if (n2 > 0) {
    for (int p = lane; p < n2; p += 64) {
      const int c = p < nprobe ? pr[p] : -1;
      srt[p] = c >= 0 ? ((c << 11) | p) : 0x7fffffff;
    }
    wave_sync();
    for (int size = 2; size <= n2; size <<= 1) {
      for (int st = size >> 1; st > 0; st >>= 1) {
        for (int i = lane; i < n2; i += 64) {
          const int j = i ^ st;
          if (j > i) {
            const bool asc = (i & size) == 0;
            const int a = srt[i], b = srt[j];
            if ((b < a) == asc) {
              srt[i] = b;
              srt[j] = a;
            }
          }
        }
        wave_sync();
      }
    }
  }
  int32_t *gb = g_base + (size_t)q * stride;
  int32_t *gl = g_len + (size_t)q * stride;
  int32_t *gp = g_prefix + (size_t)q * (stride + 1);
  int32_t *cd = cold + (size_t)q * stride;
  const unsigned long long lt = (1ull << lane) - 1ull;
  int ng = 0, nc = 0, tiles = 0, valid_n = 0;
  unsigned long long vecs = 0;
  float bmax = 0.0f;
  for (int base = 0; base < nprobe; base += 64) {
    int p = base + lane;
    int c = p < nprobe ? pr[p] : -1;
    if (n2 > 0) {  // take the probes in cluster-id order; p = rank of the probe
      const int w = p < nprobe ? srt[p] : 0x7fffffff;
      c = w != 0x7fffffff ? (w >> 11) : -1;
      p = w & 2047;
    }
    const bool valid = c >= 0;
    int t = -1, len = 0;
    float b = 0.0f;
    if (valid) {
      if (count_stats) atomicAdd(&hits[c], 1ull);
      t = clus_tile[c];
      len = clus_len[c];
      if (bias) {
        b = bias[(size_t)q * stride + p];
        bmax = fmaxf(bmax, fabsf(b));
      }
    }
    const bool res = valid && t >= 0;
    const bool cld = valid && t < 0;
    const unsigned long long mres = __ballot(res), mcold = __ballot(cld);
    const int nt = res ? (len + kTileVecs - 1) / kTileVecs : 0;
    // inclusive scan of tile counts over lanes
    int incl = nt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o, 64);
      if (lane >= o) incl += v;
    }
    if (res) {
      const int o = ng + __popcll(mres & lt);
      gb[o] = t;
      gl[o] = len;
      gp[o] = tiles + incl - nt;
      if (bias) g_bias[(size_t)q * stride + o] = b;
    }
    if (cld && n2 == 0) cd[nc + __popcll(mcold & lt)] = c;  // n2 > 0: written below
    // wave totals
    long long lv = res ? len : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lv += __shfl_xor(lv, o, 64);
    vecs += (unsigned long long)lv;
    tiles += __shfl(incl, 63, 64);
    ng += __popcll(mres);
    nc += __popcll(mcold);
    valid_n += __popcll(__ballot(valid));
  }
  if (n2 > 0) {
    // The cold list goes to the CPU in the order of the probe list, best cluster
    // first (the cluster-id order above only serves the device's lists): the CPU scan
    // then meets the query's nearest cold lists first and rejects most of the others
    // against what it found there.
    int at = 0;
    for (int base = 0; base < nprobe; base += 64) {
      const int p = base + lane;
      const int c = p < nprobe ? pr[p] : -1;
      const bool cld = c >= 0 && clus_tile[c] < 0;
      const unsigned long long mcold = __ballot(cld);
      if (cld) cd[at + __popcll(mcold & lt)] = c;
      at += __popcll(mcold);
    }
  }
  for (int p = nc + lane; p < nprobe; p += 64) cd[p] = -1;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) bmax = fmaxf(bmax, __shfl_xor(bmax, o, 64));
  if (lane == 0) {
    qbmax[q] = bmax;
    gp[ng] = tiles;
    gp[stride] = tiles;  // also at a fixed place: readable without knowing ng
    g_n[q] = ng;
    n_cold[q] = nc;
    q_vecs[q] = (int32_t)vecs;
  }
}

// The same routing for long probe lists (more than 256 probes, as at the paper's
// own operating point of 2048 probes per query, Section 5.1): one block per query,
// every step spread over all of its threads.
//  A. cluster-id order: without residual encoding a probe needs no memory of its
//     rank, so the probed clusters are marked in a bitmap over the lists and read
//     back in order (a prefix sum over the words' bit counts); otherwise (or when
//     the bitmap would not fit) a block-wide bitonic sort of (id, rank) words;
//  B. mapping table, list length, bias and counters for every probe, all loads in
//     flight together;
//  C. block-wide prefix sums place every probe in the GPU work list or the cold list.
// Outputs are exactly those of k_route.
constexpr int kRouteBigThreads = 512;
constexpr int kRouteBigPer = kMaxNprobe / kRouteBigThreads;  // probes per thread, at most
constexpr int kRouteBitmapLists = 1 << 17;                   // 16 KB of LDS

// exclusive prefix of v over the block's threads (total in *total); s_w: one slot per wavefront
__device__ __forceinline__ int block_excl_scan(int v, int *s_w, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int u = __shfl_up(incl, o, 64);
    if (lane >= o) incl += u;
  }
  if (lane == 63) s_w[wave] = incl;
  __syncthreads();
  int before = 0, all = 0;
  for (int w2 = 0; w2 < kRouteBigThreads / 64; ++w2) {
    const int x = s_w[w2];
    if (w2 < wave) before += x;
    all += x;
  }
  __syncthreads();  // s_w may be reused
  *total = all;
  return before + incl - v;
}

__global__ __launch_bounds__(kRouteBigThreads) void k_route_big(
    const int32_t *__restrict__ probe, int nq, int nprobe, int stride, int nlist,
    const int32_t *__restrict__ clus_tile, const int32_t *__restrict__ clus_len, int32_t *g_base,
    int32_t *g_len, int32_t *g_prefix, int32_t *g_n, int32_t *cold, int32_t *n_cold,
    int32_t *q_vecs, const float *__restrict__ bias, float *g_bias, float *qbmax,
    unsigned long long *hits, int count_stats, int use_bitmap,
    const uint32_t *__restrict__ lutpart, int nparts, uint32_t *__restrict__ lutmax) {
  constexpr int NT = kRouteBigThreads, E = kRouteBigPer, N = NT * E;
  __shared__ int32_t s_c[N];      // cluster of the i-th probe in cluster-id order, or -1
  __shared__ int32_t s_p[N];      // its rank in the query's probe list (bias index)
  __shared__ uint32_t s_bm[kRouteBitmapLists / 32];
  __shared__ int s_w[NT / 64];
  __shared__ unsigned long long s_vecs;
  __shared__ unsigned int s_bmax;
  const int q = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63;
  const int32_t *pr = probe + (size_t)q * stride;
  if (nparts > 0 && tid < 64) {
    uint32_t mx = 0;
    for (int i = lane; i < nparts; i += 64) mx = max(mx, lutpart[(size_t)q * kLutMaxParts + i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
    if (lane == 0) lutmax[q] = mx;
  }
  if (tid == 0) {
    s_vecs = 0ull;
    s_bmax = 0u;
  }
  // ---- A. probes in cluster-id order ----
  int nv = 0;  // valid probes
  if (use_bitmap) {
    const int nwords = (nlist + 31) >> 5;
    for (int w = tid; w < nwords; w += NT) s_bm[w] = 0u;
    __syncthreads();
    for (int p = tid; p < nprobe; p += NT) {
      const int c = pr[p];
      if (c >= 0) atomicOr(&s_bm[c >> 5], 1u << (c & 31));
    }
    __syncthreads();
    const int per = (nwords + NT - 1) / NT;
    const int w0 = min(tid * per, nwords), w1 = min(w0 + per, nwords);
    int cnt = 0;
    for (int w = w0; w < w1; ++w) cnt += __popc(s_bm[w]);
    int pos = block_excl_scan(cnt, s_w, &nv);
    for (int w = w0; w < w1; ++w) {
      uint32_t bits = s_bm[w];
      while (bits) {
        const int b = __ffs((int)bits) - 1;
        bits &= bits - 1;
        s_c[pos] = (w << 5) | b;
        s_p[pos] = 0;
        ++pos;
      }
    }
    for (int i = nv + tid; i < N; i += NT) s_c[i] = -1;
  } else {
    int n2 = 512;
    while (n2 < nprobe) n2 <<= 1;
    for (int p = tid; p < N; p += NT) {
      const int c = p < nprobe ? pr[p] : -1;
      s_c[p] = c >= 0 ? ((c << 11) | p) : 0x7fffffff;
    }
    __syncthreads();
    for (int size = 2; size <= n2; size <<= 1) {
      for (int st = size >> 1; st > 0; st >>= 1) {
        for (int i = tid; i < n2; i += NT) {
          const int j = i ^ st;
          if (j > i) {
            const bool asc = (i & size) == 0;
            const int a = s_c[i], b = s_c[j];
            if ((b < a) == asc) {
              s_c[i] = b;
              s_c[j] = a;
            }
          }
        }
        __syncthreads();
      }
    }
    for (int i = tid; i < N; i += NT) {
      const int w = s_c[i];
      s_c[i] = w != 0x7fffffff ? (w >> 11) : -1;
      s_p[i] = w & 2047;
    }
  }
  __syncthreads();
  // ---- B. look every probe up (thread t owns probes t*E .. t*E+E-1 of the order) ----
  int c[E], t[E], len[E];
  float b[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int i = tid * E + e;
    c[e] = s_c[i];
    t[e] = -1;
    len[e] = 0;
    b[e] = 0.0f;
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    if (c[e] >= 0) {
      if (count_stats) atomicAdd(&hits[c[e]], 1ull);
      t[e] = clus_tile[c[e]];
      len[e] = clus_len[c[e]];
      if (bias) b[e] = bias[(size_t)q * stride + s_p[tid * E + e]];
    }
  }
  // ---- C. place them ----
  int n_res = 0, n_cld = 0, n_tiles = 0;
  unsigned long long vec = 0;
  float bm = 0.0f;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    if (c[e] < 0) continue;
    bm = fmaxf(bm, fabsf(b[e]));
    if (t[e] >= 0) {
      n_res += 1;
      n_tiles += (len[e] + kTileVecs - 1) / kTileVecs;
      vec += (unsigned long long)len[e];
    } else {
      n_cld += 1;
    }
  }
  int ng = 0, nc = 0, tiles = 0, both = 0;
  const int packed = block_excl_scan((n_res << 16) | n_cld, s_w, &both);  // each at most 2048
  int o_res = packed >> 16;
  ng = both >> 16;
  nc = both & 0xffff;
  int o_tile = block_excl_scan(n_tiles, s_w, &tiles);
  int32_t *gb = g_base + (size_t)q * stride;
  int32_t *gl = g_len + (size_t)q * stride;
  int32_t *gp = g_prefix + (size_t)q * (stride + 1);
  int32_t *cd = cold + (size_t)q * stride;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    if (c[e] < 0) continue;
    if (t[e] >= 0) {
      gb[o_res] = t[e];
      gl[o_res] = len[e];
      gp[o_res] = o_tile;
      if (bias) g_bias[(size_t)q * stride + o_res] = b[e];
      o_res += 1;
      o_tile += (len[e] + kTileVecs - 1) / kTileVecs;
    }
  }
  // the cold list in the order of the probe list (see k_route): thread t takes probes
  // t*E .. t*E+E-1 of that list
  {
    int cc[E], n_mine = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int p = tid * E + e;
      const int c0 = p < nprobe ? pr[p] : -1;
      cc[e] = (c0 >= 0 && clus_tile[c0] < 0) ? c0 : -1;
      n_mine += cc[e] >= 0 ? 1 : 0;
    }
    int total_cold = 0;
    int o = block_excl_scan(n_mine, s_w, &total_cold);
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (cc[e] >= 0) cd[o++] = cc[e];
  }
  for (int p = nc + tid; p < nprobe; p += NT) cd[p] = -1;
  if (vec) atomicAdd(&s_vecs, vec);
  if (bm > 0.0f) atomicMax(&s_bmax, __float_as_uint(bm));  // non-negative floats order like their bits
  __syncthreads();
  if (tid == 0) {
    qbmax[q] = __uint_as_float(s_bmax);
    gp[ng] = tiles;
    gp[stride] = tiles;
    g_n[q] = ng;
    n_cold[q] = nc;
    q_vecs[q] = (int32_t)s_vecs;
  }
}

// One single-block kernel for the small per-batch steps between the router and
// the scan:
//  * batch totals of the router counters (same-address atomics from every
//    query's wavefront would serialize);
//  * the visiting order of the scan: queries grouped by their best cluster (a
//    counting sort on the cluster id folded into kOrderBins bins; the order
//    inside a group does not matter), histogram and offsets in LDS;
//  * for small batches whose scan blocks would leave the last round of the chip
//    part-full: the `extra` queries with the most resident vectors, which the
//    scan cuts into one block more than the others.
constexpr int kOrderBins = 4096;

__global__ __launch_bounds__(1024) void k_order(const int32_t *__restrict__ probe, int nq,
                                                int stride, int32_t *__restrict__ order,
                                                const int32_t *__restrict__ g_n,
                                                const int32_t *__restrict__ n_cold,
                                                const int32_t *__restrict__ q_vecs, int M,
                                                unsigned long long *qstats, int count_stats,
                                                int extra, int32_t *__restrict__ heavy,
                                                int32_t *__restrict__ hslot) {
  __shared__ unsigned int bins[kOrderBins];
  __shared__ unsigned int wsum[16];
  __shared__ unsigned long long s_res[16], s_all[16], s_vec[16], s_r1[16], s_r2[16];
  __shared__ unsigned int s_min[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < kOrderBins; i += 1024) bins[i] = 0u;

  // ---- router counters ----
  // (first and second moment of the per-query hit rate as integers in units of 2^-32:
  // the sums do not depend on the order in which they are formed)
  unsigned long long res = 0, all = 0, vec = 0, r1 = 0, r2 = 0;
  unsigned int mn = 0x3f800000u;  // 1.0f
  for (int q = tid; q < nq; q += 1024) {
    const int ng = g_n[q], valid = ng + n_cold[q];
    res += (unsigned long long)ng;
    all += (unsigned long long)valid;
    vec += (unsigned long long)q_vecs[q];
    const float rate = valid ? (float)ng / (float)valid : 0.0f;
    mn = min(mn, __float_as_uint(rate));
    if (valid) {  // ng <= valid <= 2048
      r1 += ((unsigned long long)ng << 32) / (unsigned long long)valid;
      r2 += (((unsigned long long)ng * (unsigned long long)ng) << 32) /
            ((unsigned long long)valid * (unsigned long long)valid);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    res += __shfl_xor((long long)res, o, 64);
    all += __shfl_xor((long long)all, o, 64);
    vec += __shfl_xor((long long)vec, o, 64);
    r1 += __shfl_xor((long long)r1, o, 64);
    r2 += __shfl_xor((long long)r2, o, 64);
    mn = min(mn, (unsigned int)__shfl_xor((int)mn, o, 64));
  }
  if (lane == 0) {
    s_res[wave] = res;
    s_all[wave] = all;
    s_vec[wave] = vec;
    s_r1[wave] = r1;
    s_r2[wave] = r2;
    s_min[wave] = mn;
  }
  __syncthreads();  // also: bins are zero
  if (tid == 0) {
    for (int w2 = 1; w2 < 16; ++w2) {
      res += s_res[w2];
      all += s_all[w2];
      vec += s_vec[w2];
      r1 += s_r1[w2];
      r2 += s_r2[w2];
      mn = min(mn, s_min[w2]);
    }
    atomicAdd(&qstats[QS_SCAN_BYTES], vec * (unsigned long long)M);
    if (count_stats) {
      atomicAdd(&qstats[QS_RESIDENT_PROBES], res);
      atomicAdd(&qstats[QS_PROBES], all);
      atomicAdd(&qstats[QS_QUERIES], (unsigned long long)nq);
      atomicAdd(&qstats[QS_RATE_SUM], r1);
      atomicAdd(&qstats[QS_RATE_SQ], r2);
      atomicMin(reinterpret_cast<unsigned int *>(&qstats[QS_MIN_RATE_BITS]), mn);
    }
  }

  // ---- visiting order ----
  for (int q = tid; q < nq; q += 1024)
    atomicAdd(&bins[(unsigned)probe[(size_t)q * stride] % kOrderBins], 1u);
  __syncthreads();
  // exclusive scan: thread t owns bins [4t, 4t+4)
  unsigned loc[4], tsum = 0;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    loc[b] = bins[tid * 4 + b];
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
  unsigned run = incl - tsum;
  for (int w2 = 0; w2 < wave; ++w2) run += wsum[w2];
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    bins[tid * 4 + b] = run;
    run += loc[b];
  }
  __syncthreads();
  for (int q = tid; q < nq; q += 1024) {
    const unsigned pos = atomicAdd(&bins[(unsigned)probe[(size_t)q * stride] % kOrderBins], 1u);
    order[pos] = q;
  }
  // ---- the `extra` queries with the most resident vectors get one more scan block ----
  // (small batches only: every thread ranks its queries by counting those that come
  // before them, larger first and the smaller query number first among equals)
  if (extra > 0) {
    for (int q = tid; q < nq; q += 1024) {
      const int mine = q_vecs[q];
      int rank = 0;
      for (int o = 0; o < nq; ++o) {
        const int v = q_vecs[o];
        rank += (v > mine || (v == mine && o < q)) ? 1 : 0;
      }
      hslot[q] = rank < extra ? rank : -1;
      if (rank < extra) heavy[rank] = q;
    }
  }
}

hipError_t launch_order(const BatchWs &W, int nq, int probe_stride, int M,
                        unsigned long long *qstats, int count_stats, int extra, hipStream_t st) {
  if (extra < 0 || extra > nq) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_order, dim3(1), dim3(1024), 0, st, W.probe, nq, probe_stride, W.order,
                     W.g_n, W.n_cold, W.q_vecs, M, qstats, count_stats, extra, W.heavy, W.hslot);
  return hipGetLastError();
}

hipError_t launch_route(const int32_t *probe, int nq, int nprobe, int probe_stride, int nlist,
                        const int32_t *clus_tile, const int32_t *clus_len, int M, int32_t *g_base,
                        int32_t *g_len, int32_t *g_prefix, int32_t *g_n, int32_t *cold,
                        int32_t *n_cold, int32_t *q_vecs, const float *bias, float *g_bias,
                        float *qbmax, unsigned long long *hits, int count_stats,
                        const uint32_t *lutpart, int lut_parts, uint32_t *lutmax, hipStream_t st) {
  // (id << 11 | rank) must fit a positive int: nprobe <= 2048 holds, ids need < 2^20
  int n2 = 0;
  if (nlist < (1 << 20)) {
    n2 = 64;
    while (n2 < nprobe) n2 <<= 1;
  }
  if (nprobe > 256 && nlist < (1 << 20)) {  // long lists: a block per query
    const int use_bitmap = (!bias && nlist <= kRouteBitmapLists) ? 1 : 0;
    hipLaunchKernelGGL(k_route_big, dim3(nq), dim3(kRouteBigThreads), 0, st, probe, nq, nprobe,
                       probe_stride, nlist, clus_tile, clus_len, g_base, g_len, g_prefix, g_n, cold,
                       n_cold, q_vecs, bias, g_bias, qbmax, hits, count_stats, use_bitmap, lutpart,
                       lut_parts, lutmax);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(k_route, dim3((nq + 3) / 4), dim3(256), (size_t)4 * n2 * sizeof(int32_t), st,
                     probe, nq, nprobe, probe_stride, clus_tile, clus_len, M, g_base, g_len,
                     g_prefix, g_n, cold, n_cold, q_vecs, bias, g_bias, qbmax, hits, count_stats,
                     n2, lutpart, lut_parts, lutmax);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Stage 2: per-query lookup table, fp32, layout [query][code j][sub-quantizer m],
// plus the largest |entry| per query for the fixed-point scale.
// Thread (ml, jl) owns JPT codewords of sub-quantizer m in registers (eight for
// sub-vectors of up to 16 elements, fewer for longer ones so that they still
// fit) and strides over the queries, so a block reads its codewords once and each
// query sub-vector once per JPT entries.  Lanes run along
// m: table stores are contiguous in m.  Sub-vector lengths without an
// instantiation take DSUB = 0: nothing is held in registers and every entry
// re-reads its codeword (correct, and an order of magnitude slower).
// ---------------------------------------------------------------------------
template <int DSUB, int JPT, int NT>
__global__ __launch_bounds__(256) void k_lut(const float *__restrict__ queries, int nq, int d,
                                             int M, int dsub_rt, int MW,
                                             const float *__restrict__ cbT, int kind,
                                             float *__restrict__ lut,
                                             uint32_t *__restrict__ lutpart, SplitJob split) {
  run_split_job(split);  // the queries' fp16 split for the coarse GEMM, if asked for
  const int dsub = DSUB > 0 ? DSUB : dsub_rt;
  const int tid = threadIdx.x;
  const int JL = 256 / MW;  // j lanes per block
  const int ml = tid % MW, jl = tid / MW;
  const int m = blockIdx.y * MW + ml;
  const int j0 = blockIdx.x * (JL * JPT) + jl;  // this thread's codes: j0 + t * JL
  float creg[JPT][DSUB > 0 ? DSUB : 1];
  if (DSUB > 0) {
#pragma unroll
    for (int t = 0; t < JPT; ++t) {
      const float *cw = cbT + ((size_t)(j0 + t * JL) * M + m) * DSUB;
#pragma unroll
      for (int i = 0; i < DSUB; ++i) creg[t][i] = cw[i];
    }
  }
  for (int qi = blockIdx.z; qi < nq; qi += gridDim.z) {
    const float *qv = queries + (size_t)qi * d + (size_t)m * dsub;
    float qreg[DSUB > 0 ? DSUB : 1];
    if (DSUB > 0) {
#pragma unroll
      for (int i = 0; i < DSUB; ++i) qreg[i] = qv[i];
    }
    float mxf = 0.0f;
#pragma unroll
    for (int t = 0; t < JPT; ++t) {
      const int j = j0 + t * JL;
      const float v = DSUB > 0 ? lut_entry(kind, qreg, creg[t], DSUB)
                               : lut_entry(kind, qv, cbT + ((size_t)j * M + m) * dsub, dsub);
      float *dst = &lut[((size_t)qi * 256 + j) * M + m];
      if (NT) __builtin_nontemporal_store(v, dst);
      else *dst = v;
      mxf = fmaxf(mxf, fabsf(v));
    }
    // largest |entry| seen by this wave for the query: a plain store into the
    // wave's own slot (atomics on one word per query would serialize)
    uint32_t mx = __float_as_uint(mxf);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
    if ((tid & 63) == 0) {
      const int part = ((blockIdx.y * gridDim.x + blockIdx.x) << 2) | (tid >> 6);
      lutpart[(size_t)qi * kLutMaxParts + part] = mx;
    }
  }
}

// Query strides of the table kernel: as many (x, y, z) blocks as the chip's 256
// compute units hold at once, so the launch is one even round of blocks.
template <int DSUB, int JPT>
static int lut_zblocks(unsigned xy, int nq) {
  static const int per_cu = [] {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_lut<DSUB, JPT, 0>, 256, 0) != hipSuccess || n < 1)
      n = 1;
    return n;
  }();
  int z = (int)(256u * (unsigned)per_cu / xy);
  if (z < 1) z = 1;
  if (z > nq) z = nq;
  return z;
}

// 4-bit codes: the table the scan reads has one column per code BYTE; entry j of
// column m is the sum of the entries of the two sub-quantizers packed in the
// byte (sub-quantizer 2m from the low half of j, 2m+1 from the high half).  A
// block first builds the query's msub x 16 entries in LDS (even and odd
// sub-quantizers apart, so the second phase reads consecutive words), then its
// waves write rows of the 256 x M sums, lanes along m.
template <int DSUB>
__global__ __launch_bounds__(256) void k_lut4(const float *__restrict__ queries, int d, int M,
                                              int dsub_rt, const float *__restrict__ cbT, int kind,
                                              int rows_per_block, float *__restrict__ lut,
                                              uint32_t *__restrict__ lutpart, SplitJob split) {
  run_split_job(split);
  __shared__ float t_even[16 * 128];  // [j][m]: sub-quantizer 2m
  __shared__ float t_odd[16 * 128];   //         sub-quantizer 2m + 1
  __shared__ float qs[2048];          // the query (d <= 2048 is checked by the launcher)
  const int dsub = DSUB > 0 ? DSUB : dsub_rt;
  const int msub = 2 * M;
  const int tid = threadIdx.x;
  const int qi = blockIdx.x;
  for (int i = tid; i < d; i += 256) qs[i] = queries[(size_t)qi * d + i];
  __syncthreads();
  for (int idx = tid; idx < 16 * msub; idx += 256) {
    const int j = idx / msub, s = idx - j * msub;
    const float *cw = cbT + ((size_t)j * msub + s) * dsub;
    float v;
    if (DSUB > 0) {
      float c[DSUB > 0 ? DSUB : 1];
#pragma unroll
      for (int i = 0; i < DSUB; ++i) c[i] = cw[i];
      v = lut_entry(kind, qs + s * DSUB, c, DSUB);
    } else {
      v = lut_entry(kind, qs + s * dsub, cw, dsub);
    }
    ((s & 1) ? t_odd : t_even)[j * M + (s >> 1)] = v;
  }
  __syncthreads();
  const int lane = tid & 63, w = tid >> 6;
  const int j_begin = blockIdx.y * rows_per_block;
  float mxf = 0.0f;
  for (int j = j_begin + w; j < j_begin + rows_per_block; j += 4) {
    const float *lo = t_even + (j & 15) * M;
    const float *hi = t_odd + (j >> 4) * M;
    float *row = lut + ((size_t)qi * 256 + j) * M;
    for (int m = lane; m < M; m += 64) {
      const float v = lut_pair_entry(lo[m], hi[m]);
      row[m] = v;
      mxf = fmaxf(mxf, fabsf(v));
    }
  }
  uint32_t mx = __float_as_uint(mxf);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
  if (lane == 0) lutpart[(size_t)qi * kLutMaxParts + ((blockIdx.y << 2) | w)] = mx;
}

hipError_t launch_lut(const Shape &sh, const float *q, int nq, const float *cbT, float *lut,
                      uint32_t *lutpart, int *n_parts, void *q_parts, int32_t *q_exp,
                      hipStream_t st) {
  // q_parts != NULL: the same launch also splits the queries into fp16 parts for
  // the coarse GEMM (both depend on the queries only)
  const SplitJob job{q, (uint4 *)q_parts, q_exp, q_parts ? nq : 0, sh.d / 8};
  if (sh.nbits == 4) {
    if (sh.d > 2048 || sh.M > 128) return hipErrorInvalidValue;
    const int split = nq >= 512 ? 1 : (nq >= 128 ? 4 : 16);  // blocks per query
    const dim3 grid(nq, split);
    const int rows = 256 / split;
#define IVF_LUT4_CASE(DS)                                                                  \
  case DS:                                                                                 \
    hipLaunchKernelGGL(k_lut4<DS>, grid, dim3(256), 0, st, q, sh.d, sh.M, sh.dsub, cbT,    \
                       sh.lut_kind(), rows, lut, lutpart, job);                            \
    break;
    switch (sh.dsub) {
      IVF_LUT4_CASE(1)
      IVF_LUT4_CASE(2)
      IVF_LUT4_CASE(4)
      IVF_LUT4_CASE(8)
      default:
        hipLaunchKernelGGL(k_lut4<0>, grid, dim3(256), 0, st, q, sh.d, sh.M, sh.dsub, cbT,
                           sh.lut_kind(), rows, lut, lutpart, job);
    }
#undef IVF_LUT4_CASE
    *n_parts = split * 4;
    return hipGetLastError();
  }
  const int MW = (sh.M % 32 == 0) ? 32 : 16;
  const int JL = 256 / MW;
  // Tables of more than 32 MB per batch are stored past the caches: the scan reads
  // them several kernels later, and what they leave dirty in the last-level cache
  // is written back under the scan (measured: the scan of a batch of 512 or more
  // queries at 96 code bytes runs 2 % faster this way; smaller tables, and the
  // 4-bit kernel's at any size, gain nothing).
  const bool stream_out = (size_t)nq * 256 * sh.M * sizeof(float) > ((size_t)32 << 20);
#define IVF_LUT_CASE(DS, JPT_)                                                                  \
  case DS:                                                                                     \
    grid = dim3(256 / (JL * JPT_), sh.M / MW, 1);                                              \
    grid.z = lut_zblocks<DS, JPT_>(grid.x * grid.y, nq);                                       \
    if (stream_out)                                                                            \
      hipLaunchKernelGGL((k_lut<DS, JPT_, 1>), grid, dim3(256), 0, st, q, nq, sh.d, sh.M,      \
                         sh.dsub, MW, cbT, sh.lut_kind(), lut, lutpart, job);                       \
    else                                                                                       \
      hipLaunchKernelGGL((k_lut<DS, JPT_, 0>), grid, dim3(256), 0, st, q, nq, sh.d, sh.M,      \
                         sh.dsub, MW, cbT, sh.lut_kind(), lut, lutpart, job);                       \
    break;
  dim3 grid;
  switch (sh.dsub) {
    IVF_LUT_CASE(1, 8)
    IVF_LUT_CASE(2, 8)
    IVF_LUT_CASE(3, 8)
    IVF_LUT_CASE(4, 8)
    IVF_LUT_CASE(6, 8)
    IVF_LUT_CASE(8, 8)
    IVF_LUT_CASE(12, 8)
    IVF_LUT_CASE(16, 8)
    IVF_LUT_CASE(24, 2)
    IVF_LUT_CASE(32, 2)
    IVF_LUT_CASE(48, 1)
    IVF_LUT_CASE(64, 1)
    default:
      grid = dim3(256 / (JL * 8), sh.M / MW, 1);
      grid.z = lut_zblocks<0, 8>(grid.x * grid.y, nq);
      hipLaunchKernelGGL((k_lut<0, 8, 0>), grid, dim3(256), 0, st, q, nq, sh.d, sh.M, sh.dsub, MW,
                         cbT, sh.lut_kind(), lut, lutpart, job);
  }
#undef IVF_LUT_CASE
  *n_parts = (int)(grid.x * grid.y * 4);
  if (*n_parts > kLutMaxParts) return hipErrorInvalidValue;  // cannot happen for M <= 128
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Code-tile layout.
//
// Sub-quantizers are split into groups of 32 (a trailing group of 16 when M is
// not a multiple of 32).  Byte i of a lane's M stored bytes belongs to group
// gi = i / 32 (position ip inside the group) and holds the code of
// sub-quantizer  32*gi + ((lane XOR ip) & (W-1)),  W the group width.
// A tile holds 64 vectors: 16-byte unit u of lane l sits at
// ((u * 64) + l) * 16 bytes from the start of the tile.
// ---------------------------------------------------------------------------
__host__ __device__ inline int src_subq(int lane, int i, int M) {
  const int n_full = M / 32;
  int gi = i / 32;
  int ip = i % 32;
  int W = 32;
  if (gi >= n_full) {  // trailing 16-wide group
    gi = n_full;
    ip = i - 32 * n_full;
    W = 16;
  }
  return 32 * gi + ((lane ^ ip) & (W - 1));
}

__global__ __launch_bounds__(512) void k_interleave(const uint8_t *__restrict__ stage_codes,
                                                    const int64_t *__restrict__ stage_ids,
                                                    const float *__restrict__ stage_pv,
                                                    const TileDesc *__restrict__ descs, int M,
                                                    uint8_t *__restrict__ tile_codes,
                                                    int64_t *__restrict__ tile_ids,
                                                    float *__restrict__ tile_pv) {
  const TileDesc td = descs[blockIdx.x];
  const int units = M / 16;
  const int lane = threadIdx.x & 63;
  const int u = threadIdx.x >> 6;
  const bool valid = lane < td.n_valid;
  const size_t src = (size_t)(td.src_vec + lane);
  if (u < units) {
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (valid) {
      const uint8_t *row = stage_codes + src * M;
#pragma unroll
      for (int b = 0; b < 16; ++b) {
        int m = src_subq(lane, 16 * u + b, M);
        w[b >> 2] |= (uint32_t)row[m] << (8 * (b & 3));
      }
    }
    uint4 *dst = reinterpret_cast<uint4 *>(tile_codes + (size_t)td.dst_tile * kTileVecs * M);
    dst[(size_t)u * 64 + lane] = make_uint4(w[0], w[1], w[2], w[3]);
  }
  if (u == 0) {
    tile_ids[(size_t)td.dst_tile * kTileVecs + lane] = valid ? stage_ids[src] : -1;
    if (tile_pv) tile_pv[(size_t)td.dst_tile * kTileVecs + lane] = valid ? stage_pv[src] : 0.0f;
  }
}

// The same from PINNED HOST memory that the device can address: a tile's source
// (up to 64 vectors x M bytes, contiguous in the caller's array) crosses the bus
// as 16-byte loads, 1 KB per wavefront instruction, into LDS; the bytes are then
// gathered from LDS (rows padded by one word: lane l's row starts in bank
// l * (M/4 + 1), so the 64 lanes of a gather spread over the banks).
// td.src_vec is the vector's index in the caller's arrays.
__global__ __launch_bounds__(512) void k_interleave_direct(
    const uint8_t *__restrict__ host_codes, const int64_t *__restrict__ host_ids,
    const float *__restrict__ host_pv, const TileDesc *__restrict__ descs, int M,
    uint8_t *__restrict__ tile_codes, int64_t *__restrict__ tile_ids,
    float *__restrict__ tile_pv) {
  __shared__ uint32_t rows[64 * (128 / 4 + 1)];
  const TileDesc td = descs[blockIdx.x];
  const int units = M / 16;
  const int lane = threadIdx.x & 63;
  const int u = threadIdx.x >> 6;
  const int pitch = M / 4 + 1;  // words per padded row
  const uint4 *g = reinterpret_cast<const uint4 *>(host_codes + (size_t)td.src_vec * M);
  for (int i = threadIdx.x; i < td.n_valid * units; i += 512) {
    const uint4 v = g[i];
    const int r = i / units, c = (i - r * units) * 4;
    uint32_t *d = rows + r * pitch + c;
    d[0] = v.x;
    d[1] = v.y;
    d[2] = v.z;
    d[3] = v.w;
  }
  __syncthreads();
  const bool valid = lane < td.n_valid;
  if (u < units) {
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (valid) {
      const uint8_t *row = reinterpret_cast<const uint8_t *>(rows + lane * pitch);
#pragma unroll
      for (int b = 0; b < 16; ++b) {
        int m = src_subq(lane, 16 * u + b, M);
        w[b >> 2] |= (uint32_t)row[m] << (8 * (b & 3));
      }
    }
    uint4 *dst = reinterpret_cast<uint4 *>(tile_codes + (size_t)td.dst_tile * kTileVecs * M);
    dst[(size_t)u * 64 + lane] = make_uint4(w[0], w[1], w[2], w[3]);
  }
  if (u == 0) {
    const size_t src = (size_t)td.src_vec + lane;
    tile_ids[(size_t)td.dst_tile * kTileVecs + lane] = valid ? host_ids[src] : -1;
    if (tile_pv) tile_pv[(size_t)td.dst_tile * kTileVecs + lane] = valid ? host_pv[src] : 0.0f;
  }
}

hipError_t launch_interleave_direct(const uint8_t *host_codes, const int64_t *host_ids,
                                    const float *host_pv, const TileDesc *descs, int n_tiles, int M,
                                    uint8_t *tile_codes, int64_t *tile_ids, float *tile_pv,
                                    hipStream_t st) {
  if (n_tiles <= 0) return hipSuccess;
  if (M > 128 || M % 16 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_interleave_direct, dim3(n_tiles), dim3(512), 0, st, host_codes, host_ids,
                     host_pv, descs, M, tile_codes, tile_ids, tile_pv);
  return hipGetLastError();
}

hipError_t launch_interleave(const uint8_t *stage_codes, const int64_t *stage_ids,
                             const float *stage_pv, const TileDesc *descs, int n_tiles, int M,
                             uint8_t *tile_codes, int64_t *tile_ids, float *tile_pv,
                             hipStream_t st) {
  if (n_tiles <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_interleave, dim3(n_tiles), dim3(512), 0, st, stage_codes, stage_ids,
                     stage_pv, descs, M, tile_codes, tile_ids, tile_pv);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Stage 3: ADC scan with in-block top-k.
// ---------------------------------------------------------------------------
constexpr int kScanChunk = 32;  // consecutive scan units kept on one XCD

struct ScanParams {
  const uint8_t *tile_codes;
  const int64_t *tile_ids;
  const float *lut;
  const uint32_t *lutmax;
  const float *qbmax;
  const float *g_bias;
  const float *tile_pv;
  float pv_max;
  const int32_t *g_base;
  const int32_t *g_len;
  const int32_t *g_prefix;
  const int32_t *g_n;
  const int32_t *order;
  int32_t *part_key;
  int64_t *part_id;
  // slices == 1: the block's result is the query's result and is written here
  // directly (ids and distances if out_ids != NULL, else keys and ids)
  int32_t *res_key;
  int64_t *res_id;
  int64_t *out_ids;
  float *out_dists;
  int metric_ip;
  int nq;
  int probe_stride;
  int slices;
  // `extra` queries (heavy[0 .. extra), hslot[q] = position there or -1) are cut into
  // slices + 1 blocks instead of slices: their last block is unit nq * slices + hslot
  int extra;
  const int32_t *heavy;
  const int32_t *hslot;
  int k;
};

template <int M>
struct ScanGeom {
  static constexpr int kFull = M / 32;
  static constexpr int kRem = M % 32;
  static constexpr int kGroups = kFull + (kRem ? 1 : 0);
  static constexpr int kTables = (kGroups + 1) / 2;
  static constexpr int kTableBytes = 65536;  // 256 rows x 64 columns x 4 B
};

// A located tile: where its codes are and which vectors of it are real.
struct TileRef {
  int gtile;   // tile index in the cluster region
  int first;   // position of lane 0 inside its list
  int len;     // list length
  int bias;    // quantized bias(q, list) (residual encoding), else 0
};

// RES: 0 = codes encode the vector; 1 = residual, inner product (bias per
// list); 2 = residual, L2 (bias per list + one float per vector).
template <int M, int NW, int CAP, int RES>
__global__ __launch_bounds__(NW * 64) void k_scan(ScanParams P) {
  using G = ScanGeom<M>;
  extern __shared__ __align__(16) unsigned char smem[];
  int *tab = reinterpret_cast<int *>(smem);
  // a candidate is (key, position): position = tile * 64 + lane in the cluster
  // region; its 64-bit id is read only when ids decide (ties) and for the k winners
  int *buf_pos_all = reinterpret_cast<int *>(smem + G::kTables * G::kTableBytes);
  int *buf_key_all = reinterpret_cast<int *>(smem + G::kTables * G::kTableBytes +
                                             (size_t)NW * CAP * sizeof(int));
  int *s_thr = buf_key_all + NW * CAP;
  int *s_total = s_thr + 1;
  int *s_next = s_thr + 2;  // next tile (position in the block's range) nobody has taken yet

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Block -> (query, slice).  Queries are visited in `order` (sorted by their
  // best cluster, so queries drawn around the same hot centre, which probe
  // nearly the same lists, run at the same time and share those lists through
  // L2 / Infinity Cache).  Consecutive block ids go to different XCDs, so runs
  // of kScanChunk consecutive units are mapped to one XCD.
  int u;
  {
    const int b = blockIdx.x;
    const int x = b & 7, jj = b >> 3;
    const int within = jj % kScanChunk, cc = jj / kScanChunk;
    u = (cc * 8 + x) * kScanChunk + within;
  }
  const int base_units = P.nq * P.slices;
  if (u >= base_units + P.extra) return;
  const int q = u < base_units ? P.order[u / P.slices] : P.heavy[u - base_units];
  const int s = u < base_units ? u % P.slices : P.slices;
  const int hs = P.extra ? P.hslot[q] : -1;
  const int n_slices = P.slices + (hs >= 0 ? 1 : 0);  // blocks this query is cut into
  const int k = P.k;

  // scale of the query's fixed-point table
  const int e = lut_exponent(__uint_as_float(P.lutmax[q]), M, RES ? P.qbmax[q] : 0.0f,
                             RES == 2 ? P.pv_max : 0.0f);
  int *bkey = buf_key_all + w * CAP;
  int *bpos = buf_pos_all + w * CAP;

  // per-lane column offsets: x[ip] = ((lane ^ ip) & 31) * 4, with 1 in byte 2
  // (selected by the permute only for lookups in the second table).
  uint32_t x[32];
#pragma unroll
  for (int ip = 0; ip < 32; ++ip) x[ip] = ((uint32_t)((lane ^ ip) & 31) << 2) | 0x00010000u;

  const int ng = P.g_n[q];
  const int32_t *gpre = P.g_prefix + (size_t)q * (P.probe_stride + 1);
  const int32_t *gbase = P.g_base + (size_t)q * P.probe_stride;
  const int32_t *glen = P.g_len + (size_t)q * P.probe_stride;
  const int T = gpre[P.probe_stride];  // total tiles (the router keeps a copy in the last slot)
  const int t_begin = (int)((long long)T * s / n_slices);
  const int t_end = (int)((long long)T * (s + 1) / n_slices);

  // window of 64 probes held one per lane
  int win_base = -64, win_end = 0;  // win_end: first tile index beyond the window
  int w_pre = 0, w_tile = 0, w_len = 0, w_bias = 0;
  const float *gbias = P.g_bias + (size_t)q * P.probe_stride;

  auto locate = [&](int t) -> TileRef {
    while (t >= win_end) {  // wave-uniform
      win_base += 64;
      const int p = win_base + lane;
      // the loads only need p inside the row, not the number of entries: they go
      // out together with the load of ng, whose value then masks them
      const bool can = p < P.probe_stride;
      const int l_pre = can ? gpre[p] : 0, l_tile = can ? gbase[p] : 0, l_len = can ? glen[p] : 0;
      const float l_bias = (RES && can) ? gbias[p] : 0.0f;
      const bool in = p < ng;
      w_pre = in ? l_pre : 0x7fffffff;
      w_tile = in ? l_tile : 0;
      w_len = in ? l_len : 0;
      if (RES) w_bias = in ? lut_quantize(l_bias, e) : 0;
      const int last = min(win_base + 64, ng);
      win_end = last == ng ? T : gpre[last];
    }
    const unsigned long long mask = __ballot(w_pre <= t);
    const int pl = max(__popcll(mask) - 1, 0);  // last probe of the window starting at or before t
    const int pre = __builtin_amdgcn_readlane(w_pre, pl);
    TileRef r;
    r.gtile = __builtin_amdgcn_readlane(w_tile, pl) + (t - pre);
    r.first = (t - pre) * kTileVecs;
    r.len = __builtin_amdgcn_readlane(w_len, pl);
    r.bias = RES ? __builtin_amdgcn_readlane(w_bias, pl) : 0;
    return r;
  };

  auto load_tile = [&](const TileRef &tr, uint4 (&c)[M / 16], float &pv) {
    const uint4 *src =
        reinterpret_cast<const uint4 *>(P.tile_codes + (size_t)tr.gtile * (kTileVecs * M));
#pragma unroll
    for (int u = 0; u < M / 16; ++u) c[u] = src[u * 64 + lane];
    if (RES == 2) pv = P.tile_pv[(size_t)tr.gtile * kTileVecs + lane];
  };

  int cnt = 0;            // candidates in this wave's (unsorted) buffer
  int tk = kKeyInvalid;   // a key above this can no longer reach the block's top k
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  constexpr int E = CAP / 64;

  // Shrink the buffer to the candidates whose key is not above its k-th smallest
  // key.  The k-th smallest key is found by a bitwise search with ballots (no
  // sorting, no ids); ties on that key all stay - the exact (key, id) order is
  // settled once, in the block merge.
  auto compact = [&]() {
    wave_sync();
    int kk[E];
    int pp[E];
    uint32_t uk[E];
    bool vv[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int idx = lane + 64 * e;
      vv[e] = idx < cnt;
      kk[e] = vv[e] ? bkey[idx] : kKeyInvalid;
      pp[e] = vv[e] ? bpos[idx] : 0;
      uk[e] = (uint32_t)kk[e] ^ 0x80000000u;  // order-preserving unsigned form
    }
    uint32_t prefix = 0;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = prefix | (1u << bit);
      int c = 0;
#pragma unroll
      for (int e = 0; e < E; ++e) c += __popcll(__ballot(vv[e] && uk[e] < cand));
      if (c < k) prefix = cand;  // fewer than k keys below cand: the k-th smallest is >= cand
    }
    const int T = (int)(prefix ^ 0x80000000u);
    int kept = 0, below = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      kept += __popcll(__ballot(vv[e] && kk[e] <= T));
      below += __popcll(__ballot(vv[e] && kk[e] < T));
    }
    // Usually all keys up to T stay.  Only with a mass of keys equal to T (more than
    // the buffer can carry along) the ties are cut exactly: their ids are read and
    // the (k - below) smallest ids stay, found by the same bitwise search on the
    // order-preserving unsigned form of the id.
    unsigned long long id_cut = ~0ull;
    unsigned long long uid[E];
    const bool cut_ties = kept > CAP - 64;  // wave-uniform
    if (cut_ties) {
      const int need = k - below;  // >= 1: fewer than k keys lie below the k-th smallest
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const bool tie = vv[e] && kk[e] == T;
        uid[e] = tie ? ((unsigned long long)P.tile_ids[pp[e]] ^ 0x8000000000000000ull) : ~0ull;
      }
      unsigned long long pre = 0;
      for (int bit = 63; bit >= 0; --bit) {
        const unsigned long long cand = pre | (1ull << bit);
        int c = 0;
#pragma unroll
        for (int e = 0; e < E; ++e)
          c += __popcll(__ballot(vv[e] && kk[e] == T && uid[e] < cand));
        if (c < need) pre = cand;
      }
      id_cut = pre;
    }
    wave_sync();
    int base = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      bool keep = vv[e] && kk[e] <= T;
      if (cut_ties && keep && kk[e] == T) keep = uid[e] <= id_cut;
      const unsigned long long mask = __ballot(keep);
      if (keep) {
        const int o = base + __popcll(mask & lt_mask);
        bkey[o] = kk[e];
        bpos[o] = pp[e];
      }
      base += __popcll(mask);
    }
    cnt = base;
    tk = min(tk, T);
    if (lane == 0) atomicMin(s_thr, T);
  };

  auto process = [&](const TileRef &tr, const uint4 (&c)[M / 16], float pv) {
    int acc = tr.bias;
    if (RES == 2) acc += lut_quantize(pv, e);
#pragma unroll
    for (int u = 0; u < M / 16; ++u) {
      const uint32_t dw[4] = {c[u].x, c[u].y, c[u].z, c[u].w};
#pragma unroll
      for (int ww = 0; ww < 4; ++ww) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int i = 16 * u + 4 * ww + b;
          int gi = i / 32, ip = i % 32;
          if (G::kRem && gi >= G::kFull) { gi = G::kFull; ip = i - 32 * G::kFull; }
          // result byte0 = x.byte0, byte1 = code byte b, byte2 = x.byte2 or 0, byte3 = 0
          const uint32_t sel = 0x0c000000u | ((gi >> 1) ? 0x00020000u : 0x000c0000u) |
                               ((uint32_t)(4 + b) << 8);
          const uint32_t off = __builtin_amdgcn_perm(dw[ww], x[ip], sel);
          acc += lds_read_i32(off + (gi & 1) * 128);
        }
      }
    }
    const int pos = tr.first + lane;
    const bool valid = pos < tr.len;
    const int key = valid ? acc : kKeyInvalid;
    const int thr = min(tk, __atomic_load_n(s_thr, __ATOMIC_RELAXED));
    const bool pass = valid && key <= thr;
    const unsigned long long mask = __ballot(pass);
    if (mask) {  // rare after the first tiles
      if (pass) {
        const int off = cnt + __popcll(mask & lt_mask);
        bkey[off] = key;
        bpos[off] = tr.gtile * kTileVecs + lane;
      }
      cnt += __popcll(mask);
      if (cnt > CAP - 64) compact();
    }
  };

  {
    // The first two tiles of every wave are fixed (positions w and w + NW of the
    // block's range); after that a wave takes the next position nobody has taken
    // from a counter in LDS, so all waves run out of work at about the same time
    // whatever their tiles cost (waves of a SIMD do not get equal issue time, and
    // a tile that feeds the candidate buffer costs more than one that does not).
    const int span = t_end - t_begin;
    const float4 *lut_src = reinterpret_cast<const float4 *>(P.lut + (size_t)q * 256 * M);
    constexpr int kVec = 256 * M / 4;
    constexpr int kIter = (kVec + NW * 64 - 1) / (NW * 64);
    // table loads in flight per thread (one round trip per batch): all of them if few
    constexpr int kBatch = kIter <= 6 ? kIter : 4;
    // the first batch of table loads goes out before the (dependent) work-list loads
    float4 lv[kBatch];
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      const int idx = tid + b * (NW * 64);
      if (b < kIter && idx < kVec) lv[b] = lut_src[idx];
    }
    int t = w;  // position of the current tile in the block's range
    TileRef cur{0, 0, 0, 0};
    uint4 ca[M / 16];
    float pa = 0.0f;
    if (t < span) {
      cur = locate(t_begin + t);
      load_tile(cur, ca, pa);
    }
    // ---- stage the query's table in LDS as fixed point, code-major (the first
    // tile's loads are already in flight) ----
    {
#pragma unroll
      for (int i0 = 0; i0 < kIter; i0 += kBatch) {
        if (i0 > 0) {
#pragma unroll
          for (int b = 0; b < kBatch; ++b) {
            const int idx = tid + (i0 + b) * (NW * 64);
            if (i0 + b < kIter && idx < kVec) lv[b] = lut_src[idx];
          }
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
          const int idx = tid + (i0 + b) * (NW * 64);
          if (i0 + b < kIter && idx < kVec) {
            const int flat = idx * 4;
            const int j = flat / M;
            const int m0 = flat % M;  // 4 consecutive sub-quantizers of one code (M % 4 == 0)
            const int4 keys = make_int4(lut_quantize(lv[b].x, e), lut_quantize(lv[b].y, e),
                                        lut_quantize(lv[b].z, e), lut_quantize(lv[b].w, e));
            const int gi = m0 / 32, r = m0 % 32;  // the four share a 32-wide group
            int *row = tab + (gi >> 1) * (G::kTableBytes / 4) + j * 64 + (gi & 1) * 32;
            *reinterpret_cast<int4 *>(row + r) = keys;
            if (G::kRem && gi == G::kFull)  // 16-wide group: second replica
              *reinterpret_cast<int4 *>(row + r + 16) = keys;
          }
        }
      }
      if (tid == 0) {
        *s_thr = kKeyInvalid;
        *s_total = 0;
        *s_next = 2 * NW;
      }
    }
    __syncthreads();
    int tn = t + NW;  // the wave's second tile
    while (t < span) {
      TileRef nxt{0, 0, 0, 0};
      uint4 cb[M / 16];
      float pb = 0.0f;
      if (tn < span) {
        nxt = locate(t_begin + tn);
        load_tile(nxt, cb, pb);
      } else {
#pragma unroll
        for (int u = 0; u < M / 16; ++u) cb[u] = make_uint4(0, 0, 0, 0);
      }
      // take the position after that; the answer is only needed after this tile's work
      int taken = 0;
      if (lane == 0) taken = atomicAdd(s_next, 1);
      process(cur, ca, pa);
#pragma unroll
      for (int u = 0; u < M / 16; ++u) ca[u] = cb[u];
      pa = pb;
      cur = nxt;
      t = tn;
      tn = __builtin_amdgcn_readfirstlane(taken);
    }
  }

  // ---- block merge.  Each wave trims its buffer to about k candidates, all of
  // them are gathered in the (now idle) table region, and one wave selects the
  // k best by (key, id): bitwise search for the k-th smallest key, then a rank
  // sort of the few candidates at or below it. ----
  if (cnt > k) compact();
  wave_sync();
  __syncthreads();
  constexpr int kMaxCand = NW * (CAP - 64);        // every wave holds at most CAP - 64
  constexpr int kFin = kMaxCand <= 1024 ? 1024 : 2048;  // power of two >= kMaxCand
  static_assert(kMaxCand <= kFin && kMaxCand * 8 + kFin * 12 <= 65536, "merge arrays fit");
  int *mpos = reinterpret_cast<int *>(smem);
  int *mkey = reinterpret_cast<int *>(smem + (size_t)kMaxCand * 4);
  long long *fid = reinterpret_cast<long long *>(smem + (size_t)kMaxCand * 8);
  int *fkey = reinterpret_cast<int *>(smem + (size_t)kMaxCand * 8 + (size_t)kFin * 8);
  {
    // Some wave holds k candidates at or below s_thr (the smallest k-th key any wave
    // found), so nothing above it can be among the block's k best: only the
    // candidates at or below it are gathered, a few more than k in all.
    const int thr = *s_thr;
    int kk[E];
    int pp[E];
    bool keep[E];
    int mine = 0;
#pragma unroll
    for (int e2 = 0; e2 < E; ++e2) {
      const int idx = lane + 64 * e2;
      const bool v = idx < cnt;
      kk[e2] = v ? bkey[idx] : kKeyInvalid;
      pp[e2] = v ? bpos[idx] : 0;
      keep[e2] = v && kk[e2] <= thr;
      mine += __popcll(__ballot(keep[e2]));
    }
    int base = 0;
    if (lane == 0) base = atomicAdd(s_total, mine);
    base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
    for (int e2 = 0; e2 < E; ++e2) {
      const unsigned long long mask = __ballot(keep[e2]);
      if (keep[e2]) {
        const int o = base + __popcll(mask & lt_mask);
        mkey[o] = kk[e2];
        mpos[o] = pp[e2];
      }
      base += __popcll(mask);
    }
  }
  __syncthreads();
  if (w != 0) return;
  const int n = *s_total;
  // Keys of the gathered candidates in registers (order-preserving unsigned form), RR
  // per lane: bitwise search for the k-th smallest key, then everything at or below
  // it moves to (fkey, fid), its id read from the cluster region.  Usually only a few
  // more than k candidates arrive here.
  constexpr int R = kMaxCand / 64;
  int nf = 0;
  auto select_kth = [&](auto rr_tag) {
    constexpr int RR = decltype(rr_tag)::value;
    uint32_t rk[RR];
#pragma unroll
    for (int e2 = 0; e2 < RR; ++e2) {
      const int i = e2 * 64 + lane;
      rk[e2] = i < n ? ((uint32_t)mkey[i] ^ 0x80000000u) : 0xffffffffu;
    }
    uint32_t kth_u = 0xffffffffu;
    if (n > k) {
      uint32_t prefix = 0;
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = prefix | (1u << bit);
        int c = 0;
#pragma unroll
        for (int e2 = 0; e2 < RR; ++e2) c += __popcll(__ballot(rk[e2] < cand));
        if (c < k) prefix = cand;
      }
      kth_u = prefix;
    }
#pragma unroll
    for (int e2 = 0; e2 < RR; ++e2) {
      const int i = e2 * 64 + lane;
      const bool keep = i < n && rk[e2] <= kth_u;
      const unsigned long long mask = __ballot(keep);
      if (keep) {
        const int o = nf + __popcll(mask & lt_mask);
        fkey[o] = (int)(rk[e2] ^ 0x80000000u);
        fid[o] = P.tile_ids[mpos[i]];  // the finalists' ids, for the exact (key, id) order
      }
      nf += __popcll(mask);
    }
  };
  if (n <= 128) select_kth(std::integral_constant<int, 2>{});
  else select_kth(std::integral_constant<int, R>{});
  wave_sync();
  const size_t obase = (s < P.slices ? (size_t)q * P.slices + s : (size_t)base_units + hs) * k;
  // rank-th best of this block: a partial result for k_merge, or, with one
  // slice per query, the query's result itself
  auto emit = [&](int rank, int key, long long id) {
    if (n_slices > 1) {
      P.part_key[obase + rank] = key;
      P.part_id[obase + rank] = id;
      return;
    }
    const bool ok = key != kKeyInvalid;
    const size_t o = (size_t)q * k + rank;
    if (P.out_ids) {
      P.out_ids[o] = ok ? id : -1;
      P.out_dists[o] =
          ok ? key_to_dist(key, e, P.metric_ip) : (P.metric_ip ? -INFINITY : INFINITY);
    } else {
      P.res_key[o] = key;
      P.res_id[o] = ok ? id : -1;
    }
  };
  if (nf <= 192) {
    for (int i = lane; i < nf; i += 64) {
      const int ki = fkey[i];
      const long long idi = fid[i];
      int rank = 0;
      for (int j = 0; j < nf; ++j) rank += cand_less(fkey[j], fid[j], ki, idi) ? 1 : 0;
      if (rank < k) emit(rank, ki, idi);
    }
    for (int r = nf + lane; r < k; r += 64) emit(r, kKeyInvalid, 0x7fffffffffffffffll);
  } else {  // a mass of equal keys: sort them all
    int n2 = 256;
    while (n2 < nf) n2 <<= 1;
    for (int i = nf + lane; i < n2; i += 64) {
      fkey[i] = kKeyInvalid;
      fid[i] = 0x7fffffffffffffffll;
    }
    wave_sync();
    bitonic_sort_lds<false>(fkey, fid, n2, lane, 64);
    for (int r = lane; r < k; r += 64) emit(r, fkey[r], fid[r]);
  }
}

template <int M, int NW, int CAP, int RES>
static hipError_t launch_scan_t(const ScanParams &P, int nq, hipStream_t st) {
  using G = ScanGeom<M>;
  const size_t lds = (size_t)G::kTables * G::kTableBytes + (size_t)NW * CAP * 8 + 64;
  static std::atomic<bool> attr_done{false};  // setting it twice is harmless
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_scan<M, NW, CAP, RES>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done.store(true, std::memory_order_release);
  }
  const int total = nq * P.slices + P.extra;
  const int grid = (total + 8 * kScanChunk - 1) / (8 * kScanChunk) * (8 * kScanChunk);
  hipLaunchKernelGGL((k_scan<M, NW, CAP, RES>), dim3(grid), dim3(NW * 64), lds, st, P);
  return hipGetLastError();
}

int scan_blocks_per_cu(int M, int k) { return (M <= 64 && k <= 64) ? 2 : 1; }

bool scan_supports(int M, int k) {
  if (k < 1 || k > kMaxK) return false;
  return M == 16 || M == 32 || M == 48 || M == 64 || M == 96 || M == 128;
}

hipError_t launch_scan(const Shape &sh, const DevLayout &L, const BatchWs &W, int nq,
                       int probe_stride, int slices, int extra, int k, int64_t *out_ids,
                       float *out_dists, hipStream_t st) {
  if (!scan_supports(sh.M, k)) return hipErrorInvalidValue;
  if (slices < 1 || extra < 0 || extra > nq) return hipErrorInvalidValue;
  ScanParams P;
  P.tile_codes = L.tile_codes;
  P.tile_ids = L.tile_ids;
  P.lut = W.lut;
  P.lutmax = W.lutmax;
  P.g_base = W.g_base;
  P.g_len = W.g_len;
  P.g_prefix = W.g_prefix;
  P.g_n = W.g_n;
  P.order = W.order;
  P.nq = nq;
  P.part_key = W.part_key;
  P.part_id = W.part_id;
  P.res_key = W.res_key;
  P.res_id = W.res_id;
  P.out_ids = out_ids;
  P.out_dists = out_dists;
  P.metric_ip = sh.metric_ip;
  P.probe_stride = probe_stride;
  P.slices = slices;
  P.extra = extra;
  P.heavy = W.heavy;
  P.hslot = W.hslot;
  P.k = k;
  P.qbmax = W.qbmax;
  P.g_bias = W.g_bias;
  P.tile_pv = L.tile_pv;
  P.pv_max = sh.pv_max;
  const int res = sh.scan_res();
#define IVF_SCAN_RES(MM, NW_, CAP_)                                               \
  (res == 0 ? launch_scan_t<MM, NW_, CAP_, 0>(P, nq, st)                          \
            : res == 1 ? launch_scan_t<MM, NW_, CAP_, 1>(P, nq, st)               \
                       : launch_scan_t<MM, NW_, CAP_, 2>(P, nq, st))
  // Wavefronts per block and candidate slots (8 bytes each) per wavefront: at
  // least k + 64 slots; 128 up to k = 48, 192 above (at k near 64 a buffer of 128
  // would be trimmed after every 64 insertions).  Two tables (96 or 128 code
  // bytes) leave 32 KB of LDS for the buffers of 16 wavefronts.  One table leaves
  // room for two blocks of eight wavefronts per CU up to k = 64 (one stages its
  // table while the other streams), one block of 16 above.
#define IVF_SCAN_CASE(MM) \
  case MM:                \
    return k <= 48 ? IVF_SCAN_RES(MM, 16, 128) : IVF_SCAN_RES(MM, 16, 192);
#define IVF_SCAN_CASE_SMALL(MM) \
  case MM:                      \
    return k <= 48 ? IVF_SCAN_RES(MM, 8, 128) : (k <= 64 ? IVF_SCAN_RES(MM, 8, 192) : IVF_SCAN_RES(MM, 16, 192));
  switch (sh.M) {
    IVF_SCAN_CASE_SMALL(16)
    IVF_SCAN_CASE_SMALL(32)
    IVF_SCAN_CASE_SMALL(48)
    IVF_SCAN_CASE_SMALL(64)
    IVF_SCAN_CASE(96)
    IVF_SCAN_CASE(128)
  }
#undef IVF_SCAN_CASE_SMALL
#undef IVF_SCAN_CASE
#undef IVF_SCAN_RES
  return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------
// Per-query merge of the scan blocks' partial lists; emits the GPU result.
// One block per query.  The k-th smallest key of the slices * k candidates is found
// by a radix search over the keys' bytes (four passes of a 256-bin histogram in LDS),
// the few candidates at or below it are ranked exactly by (key, id) by counting, and
// ranks below k are written: the cost does not grow with the number of slices a
// small batch was split into.
// ---------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(NT) void k_merge(const int32_t *__restrict__ part_key,
                                              const int64_t *__restrict__ part_id, int slices,
                                              int nq, const int32_t *__restrict__ hslot, int k,
                                              const uint32_t *__restrict__ lutmax,
                                              const float *__restrict__ qbmax, float pv_max,
                                              int M, int metric_ip, int32_t *res_key, int64_t *res_id,
                                              int64_t *out_ids, float *out_dists) {
  extern __shared__ __align__(16) unsigned char merge_smem[];
  const int q = blockIdx.x;
  const int tid = threadIdx.x;
  // the query's `slices` partial lists, plus one more (stored after those of all the
  // queries) if it is one of the batch's heavy queries (hslot, optional)
  const int hs = hslot ? hslot[q] : -1;
  const int n_base = slices * k;
  const int n_in = n_base + (hs >= 0 ? k : 0);
  if (n_in == k) return;  // a single block scanned this query and wrote its result itself
  long long *mid = reinterpret_cast<long long *>(merge_smem);          // [n_in]
  int *mkey = reinterpret_cast<int *>(merge_smem + (size_t)n_in * 8);  // [n_in]
  int *fin = mkey + n_in;                                              // [n_in] finalists' indices
  __shared__ unsigned int hist[256];
  __shared__ unsigned int s_prefix, s_mask, s_need, s_nf;
  for (int i = tid; i < n_in; i += NT) {
    const size_t src = i < n_base ? (size_t)q * n_base + i
                                  : ((size_t)nq * slices + hs) * k + (i - n_base);
    mkey[i] = part_key[src];
    mid[i] = (long long)part_id[src];
  }
  if (tid == 0) {
    s_prefix = 0u;
    s_mask = 0u;
    s_need = (unsigned)k;  // n_in >= k
    s_nf = 0u;
  }
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int b = tid; b < 256; b += NT) hist[b] = 0u;
    __syncthreads();
    const unsigned prefix = s_prefix, mask = s_mask, need = s_need;
    for (int i = tid; i < n_in; i += NT) {
      const unsigned u = (unsigned)mkey[i] ^ 0x80000000u;  // order-preserving unsigned form
      if ((u & mask) == prefix) atomicAdd(&hist[(u >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid < 64) {  // one wavefront finds the byte value that holds rank `need`
      unsigned loc[4], tsum = 0;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        loc[b] = hist[tid * 4 + b];
        tsum += loc[b];
      }
      unsigned incl = tsum;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const unsigned u = __shfl_up(incl, o, 64);
        if (tid >= o) incl += u;
      }
      const unsigned before = incl - tsum;
      if (before < need && need <= before + tsum) {
        unsigned cum = before;
        int b = 0;
        for (; b < 3; ++b) {
          if (cum + loc[b] >= need) break;
          cum += loc[b];
        }
        s_need = need - cum;
        s_prefix = prefix | ((unsigned)(tid * 4 + b) << shift);
        s_mask = mask | (0xffu << shift);
      }
    }
    __syncthreads();
  }
  const int kth = (int)(s_prefix ^ 0x80000000u);  // the k-th smallest key
  for (int i = tid; i < n_in; i += NT) {
    const int key = mkey[i];
    if (key <= kth && key != kKeyInvalid) fin[atomicAdd(&s_nf, 1u)] = i;
  }
  __syncthreads();
  const int nf = (int)s_nf;  // k or a few more (ties on the k-th key), fewer if fewer candidates exist
  const int e = lut_exponent(__uint_as_float(lutmax[q]), M, qbmax[q], pv_max);
  auto emit = [&](int rank, int key, long long id) {
    const bool ok = key != kKeyInvalid;
    if (out_ids) {
      out_ids[(size_t)q * k + rank] = ok ? (int64_t)id : -1;
      out_dists[(size_t)q * k + rank] =
          ok ? key_to_dist(key, e, metric_ip) : (metric_ip ? -INFINITY : INFINITY);
    } else {
      res_key[(size_t)q * k + rank] = key;
      res_id[(size_t)q * k + rank] = ok ? (int64_t)id : -1;
    }
  };
  for (int f = tid; f < nf; f += NT) {
    const int i = fin[f];
    const int key = mkey[i];
    const long long id = mid[i];
    int rank = 0;
    for (int g = 0; g < nf; ++g) {
      const int j = fin[g];
      rank += cand_less(mkey[j], mid[j], key, id) ? 1 : 0;
    }
    if (rank < k) emit(rank, key, id);
  }
  for (int r = nf + tid; r < k; r += NT) emit(r, kKeyInvalid, -1);
}

hipError_t launch_merge(const Shape &sh, const BatchWs &W, int nq, int slices, int extra, int k,
                        int64_t *out_ids, float *out_dists, hipStream_t st) {
  const int most = slices + (extra > 0 ? 1 : 0);  // partial lists of one query, at most
  if (slices < 1 || most > kMaxSlices + 1 || k > kMaxK || most * k > kMaxMergeCand + kMaxK)
    return hipErrorInvalidValue;
  const size_t lds = (size_t)most * k * 16;  // at most 130 KB
  const float pvm = sh.scan_res() == 2 ? sh.pv_max : 0.0f;
  const int32_t *hslot = extra > 0 ? W.hslot : nullptr;
  if (most * k <= 1024) {
    hipLaunchKernelGGL(k_merge<256>, dim3(nq), dim3(256), lds, st, W.part_key, W.part_id, slices, nq,
                       hslot, k, W.lutmax, W.qbmax, pvm, sh.M, sh.metric_ip, W.res_key, W.res_id,
                       out_ids, out_dists);
  } else {
    static std::atomic<bool> attr_done{false};  // setting it twice is harmless
    if (!attr_done.load(std::memory_order_acquire)) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_merge<1024>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (kMaxMergeCand + kMaxK) * 16);
      if (e != hipSuccess) return e;
      attr_done.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(k_merge<1024>, dim3(nq), dim3(1024), lds, st, W.part_key, W.part_id, slices,
                       nq, hslot, k, W.lutmax, W.qbmax, pvm, sh.M, sh.metric_ip, W.res_key, W.res_id,
                       out_ids, out_dists);
  }
  return hipGetLastError();
}

}  // namespace ivf
