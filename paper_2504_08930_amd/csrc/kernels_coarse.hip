// Stage 1 of IVF search (Section 2.2): coarse quantization.  Every query is
// scored against every centroid as a dense contraction on the matrix cores
// (split-fp16 MFMA at close to fp32 accuracy), then the nprobe best clusters per query
// are selected exactly by a radix select over (score, cluster id).
//
// The paper keeps this stage on the CPU to avoid ping-pong between devices
// when several GPU shards are used (Section 4.1.1); with one GPU that concern
// does not arise and the contraction runs on the device.
#include <hip/hip_runtime.h>
#include <math.h>

#include <algorithm>
#include <atomic>

#include "internal.h"
#include "split_f16.h"

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
// Two-way fp16 split of an fp32 matrix (split_f16.h), one wavefront per row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_split_f16(const float *__restrict__ src, size_t rows,
                                                   int groups_per_row, uint4 *__restrict__ dst,
                                                   int32_t *__restrict__ row_exp) {
  const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  split_row_f16(src, rows, groups_per_row, dst, row_exp, row, threadIdx.x & 63);
}

hipError_t launch_split_f16(const float *src, size_t rows, int d, void *dst, int32_t *row_exp,
                            hipStream_t st) {
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(k_split_f16, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, src, rows,
                     d / 8, (uint4 *)dst, row_exp);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// scores[q][c] = q . c            (IP, larger is better)
//              = |c|^2 - 2 q . c  (L2, smaller is better)
//
// The contraction runs on the fp16 matrix cores at close to fp32 accuracy:
// with q 2^eq = q1 + q2 and c 2^ec = c1 + c2 (two-way fp16 splits of the scaled
// rows), q.c 2^(eq+ec) is accumulated in fp32 from the three products q2c1,
// q1c2, q1c1; the dropped product and the split remainders are below 2^-21
// relative per term.  The power-of-two scales are taken out exactly in the
// epilogue.  Three v_mfma_f32_32x32x16_f16 cost 3/16 of the fp32 MFMA work
// for the same K.
//
// Block tile of WM x WN waves, each wave TM x TN MFMA tiles of 32 x 32; K is
// consumed 16 at a time through LDS (per row: 2 groups x 2 parts x 16 B).
// Blocks are numbered so that the row tiles sharing a centroid tile run next
// to each other on one XCD (block id mod 8 picks the XCD), which keeps each
// centroid tile in that XCD's L2.
// ---------------------------------------------------------------------------
static_assert(kSplitPadBytes >= 256 * 64, "padding covers one row tile of the last chunk");
// LDS image of a K = 16 chunk: 64 B per row (two groups x two parts x 16 B), unpadded.
// The 16-byte unit u of row r sits at unit position u ^ swz(r), swz a 2-bit function of
// the row chosen so that both access patterns are conflict-free whether the LDS serves
// 8 lanes x 16 B per cycle over 32 banks or 16 lanes over 64: the fragment reads (32
// consecutive rows, one unit each) and the stores of the staged chunk (four
// consecutive units of consecutive rows).  A padded layout (80 B per row) makes the
// reads conflict-free too, but every group of 8 or 16 storing lanes then hits one
// 16-byte bank group twice.
constexpr int kRowBytes = 64;
__device__ __forceinline__ int lds_swz(int row) {
  return (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1);
}

// <1,4,1,2> / <1,2,1,2>: 32 x 256 / 32 x 128 block, 4 / 2 waves of 32 x 64 (up to 64 queries);
// <4,2,1,2>: 128 x 128 block, 8 waves of 32 x 64 (batches that leave big tiles too few
// blocks; twice the waves of a 4-wave block of 64 x 64 tiles hide more of the K loop's
// latency: 29 instead of 36 us at 256 queries x 16384 centroids);
// <4,4,2,2>: 256 x 256 block, 16 waves of 64 x 64 (half the L2 traffic per MFMA of the
// small tile; 120 registers, so four waves per SIMD hide one another's LDS and
// barrier waits - measured 10 % faster than 8 waves of 64 x 128 at two per SIMD).
template <int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(WM *WN * 64) void k_coarse_gemm(
    const uint4 *__restrict__ Qp, const int32_t *__restrict__ q_exp, int nq,
    const uint4 *__restrict__ Cp, const int32_t *__restrict__ c_exp, int nlist, int d,
    const float *__restrict__ cnorm, int metric_ip, int row_tiles, int col_tiles,
    float *__restrict__ scores) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32, NT = WM * WN * 64;
  // rows of the query operand staged per chunk: the tile's, or (a tile of 32 queries
  // under 128 or 256 threads) as many as give every thread one unit to load; the
  // extra rows are read like any rows beyond the matrix and never used
  constexpr int BMA = BM * 4 >= NT ? BM : NT / 4;
  constexpr int LA = BMA * 4 / NT, LB = BN * 4 / NT;  // 16-byte units per thread and chunk
  static_assert(BMA * 4 % NT == 0 && BN * 4 % NT == 0, "tile loads divide evenly");
  static_assert(BMA * 64 <= kSplitPadBytes, "staged rows beyond the matrix stay inside the padding");
  extern __shared__ __align__(16) unsigned char gsm[];
  auto a_tile = [&](int buf) { return gsm + buf * ((BMA + BN) * kRowBytes); };
  auto b_tile = [&](int buf) { return gsm + buf * ((BMA + BN) * kRowBytes) + BMA * kRowBytes; };
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  // XCD-aware tile assignment
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  const int ct = (j / row_tiles) * 8 + xcd, rt = j % row_tiles;
  if (ct >= col_tiles) return;
  const int row0 = rt * BM;   // queries
  const int col0 = ct * BN;   // centroids

  // global -> LDS: unit f = tid + NT * i, row = f / 4, u = f % 4; loads run two
  // chunks ahead of the MFMAs in registers, LDS is double buffered.  The loads
  // carry no bounds check (straight-line code lets the compiler wait for exactly
  // the older of the two stages): rows of a tile beyond the matrix read the
  // following chunk or, for the last chunk, the kSplitPadBytes of padding that
  // both operand arrays carry; whatever they hold only reaches rows and columns
  // of the product that the epilogue never stores.
  // Two register stages.  Each is named in the code that touches it (no stage
  // index, no reference passed around), so both stay in registers.
  typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
  uintx4 ga0[LA], gb0[LB], ga1[LA], gb1[LB];
  // per-thread unit offsets inside a chunk (32-bit), added to a uniform chunk base
  unsigned offa[LA], offb[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) offa[i] = (unsigned)(row0 * 4 + tid + NT * i);
#pragma unroll
  for (int i = 0; i < LB; ++i) offb[i] = (unsigned)(col0 * 4 + tid + NT * i);
#define IVF_GLOAD(kc, GA, GB)                                       \
  do {                                                              \
    const uintx4 *qb_ = reinterpret_cast<const uintx4 *>(Qp) + (size_t)(kc) * nq * 4;    \
    const uintx4 *cb_ = reinterpret_cast<const uintx4 *>(Cp) + (size_t)(kc) * nlist * 4; \
    _Pragma("unroll") for (int i = 0; i < LA; ++i) GA[i] = qb_[offa[i]]; \
    _Pragma("unroll") for (int i = 0; i < LB; ++i) GB[i] = cb_[offb[i]]; \
  } while (0)
#define IVF_SSTORE(buf, GA, GB)                                                              \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < LA; ++i) {                                         \
      const int f = tid + NT * i;                                                            \
      *reinterpret_cast<uintx4 *>(a_tile(buf) + (f >> 2) * kRowBytes + (((f & 3) ^ swz_st) << 4)) = GA[i]; \
    }                                                                                        \
    _Pragma("unroll") for (int i = 0; i < LB; ++i) {                                         \
      const int f = tid + NT * i;                                                            \
      *reinterpret_cast<uintx4 *>(b_tile(buf) + (f >> 2) * kRowBytes + (((f & 3) ^ swz_st) << 4)) = GB[i]; \
    }                                                                                        \
  } while (0)

  // a thread's stored rows are (tid >> 2) + a multiple of 64: one swizzle for all of them
  const int swz_st = lds_swz(tid >> 2);
  floatx16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  const int nk = d / 16;  // d is a multiple of 16
  IVF_GLOAD(0, ga0, gb0);
  IVF_SSTORE(0, ga0, gb0);
  if (nk > 1) IVF_GLOAD(1, ga1, gb1);
  __syncthreads();
  const int li = lane & 31, kk = lane >> 5;
  const int swz_ld = lds_swz(li);  // fragment rows are li + a multiple of 32
  // the MFMA work of one K chunk held in LDS buffer `buf`
  auto mma = [&](int buf) {
    // lane (li, kk) holds k = 8*kk .. 8*kk+7 of the chunk for row li of a tile
    halfx8 a[TM][2], b[TN][2];
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
      for (int p = 0; p < 2; ++p)
        a[t][p] = __builtin_bit_cast(
            halfx8,
            *reinterpret_cast<const uint4 *>(
                a_tile(buf) + (wm * TM * 32 + t * 32 + li) * kRowBytes + (((kk * 2 + p) ^ swz_ld) << 4)));
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
      for (int p = 0; p < 2; ++p)
        b[t][p] = __builtin_bit_cast(
            halfx8,
            *reinterpret_cast<const uint4 *>(
                b_tile(buf) + (wn * TN * 32 + t * 32 + li) * kRowBytes + (((kk * 2 + p) ^ swz_ld) << 4)));
    // small products first; consecutive MFMAs go to different accumulators
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
      for (int nt = 0; nt < TN; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mt][1], b[nt][0], acc[mt][nt], 0, 0, 0);
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
      for (int nt = 0; nt < TN; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mt][0], b[nt][1], acc[mt][nt], 0, 0, 0);
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
      for (int nt = 0; nt < TN; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mt][0], b[nt][0], acc[mt][nt], 0, 0, 0);
  };
  // chunk kc is computed from LDS while chunk kc+2 is loaded into the stage that
  // chunk kc's own data left free, and chunk kc+1 (loaded one step earlier) moves
  // from its stage to the other LDS buffer; unrolled by two, the stages alternate
  int kc = 0;
  for (; kc + 3 < nk; kc += 2) {  // steady state: straight-line, so waits can be exact
    IVF_GLOAD(kc + 2, ga0, gb0);
    mma(0);
    IVF_SSTORE(1, ga1, gb1);
    __syncthreads();
    IVF_GLOAD(kc + 3, ga1, gb1);
    mma(1);
    IVF_SSTORE(0, ga0, gb0);
    __syncthreads();
  }
  for (; kc < nk; kc += 2) {  // the last one to three chunks
    if (kc + 2 < nk) IVF_GLOAD(kc + 2, ga0, gb0);
    mma(0);
    if (kc + 1 < nk) IVF_SSTORE(1, ga1, gb1);
    __syncthreads();
    if (kc + 1 < nk) {
      if (kc + 3 < nk) IVF_GLOAD(kc + 3, ga1, gb1);
      mma(1);
      if (kc + 2 < nk) IVF_SSTORE(0, ga0, gb0);
      __syncthreads();
    }
  }
#undef IVF_GLOAD
#undef IVF_SSTORE

  // D[i][j]: register r of lane l holds i = 8*(r/4) + 4*(l/32) + r%4, j = l%32
#pragma unroll
  for (int mt = 0; mt < TM; ++mt)
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) {
      const int c = col0 + wn * TN * 32 + nt * 32 + li;
      const float cn = (!metric_ip && c < nlist) ? cnorm[c] : 0.0f;
      const int ce = c < nlist ? c_exp[c] : 0;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qi = row0 + wm * TM * 32 + mt * 32 + 8 * (r >> 2) + 4 * kk + (r & 3);
        if (qi < nq && c < nlist) {
          const float dot = ldexpf(acc[mt][nt][r], -(ce + q_exp[qi]));
          scores[(size_t)qi * nlist + c] = metric_ip ? dot : __builtin_fmaf(-2.0f, dot, cn);
        }
      }
    }
}

template <int WM, int WN, int TM, int TN>
static hipError_t launch_gemm_t(const Shape &sh, const void *q_parts, const int32_t *q_exp, int nq,
                                const void *cent_parts, const int32_t *cent_exp,
                                const float *cent_norm, float *scores, hipStream_t st) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32, NT = WM * WN * 64;
  constexpr int BMA = BM * 4 >= NT ? BM : NT / 4;
  const size_t lds = (size_t)2 * (BMA + BN) * kRowBytes;
  static std::atomic<bool> attr_done{false};  // setting it twice is harmless
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e =
        hipFuncSetAttribute(reinterpret_cast<const void *>(&k_coarse_gemm<WM, WN, TM, TN>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done.store(true, std::memory_order_release);
  }
  const int row_tiles = (nq + BM - 1) / BM;
  const int col_tiles = (sh.nlist + BN - 1) / BN;
  const int grid = 8 * ((col_tiles + 7) / 8) * row_tiles;
  hipLaunchKernelGGL((k_coarse_gemm<WM, WN, TM, TN>), dim3(grid), dim3(WM * WN * 64), lds, st,
                     (const uint4 *)q_parts, q_exp, nq, (const uint4 *)cent_parts, cent_exp, sh.nlist,
                     sh.d, cent_norm, sh.metric_ip, row_tiles, col_tiles, scores);
  return hipGetLastError();
}

hipError_t launch_coarse_gemm(const Shape &sh, const void *q_parts, const int32_t *q_exp, int nq,
                              const void *cent_parts, const int32_t *cent_exp,
                              const float *cent_norm, float *scores, hipStream_t st) {
  // A handful of queries (the paper's batches run from a few to a few dozen): tiles
  // of 32 queries, so that the matrix cores are not fed 256 rows of which 8 are real
  // and the kernel is bound by reading the centroids once; 256 centroids wide when
  // that still gives the chip enough blocks.
  if (nq <= 64) {
    const long long wide_blocks = (long long)((nq + 31) / 32) * ((sh.nlist + 255) / 256);
    if (wide_blocks >= 192)
      return launch_gemm_t<1, 4, 1, 2>(sh, q_parts, q_exp, nq, cent_parts, cent_exp, cent_norm,
                                       scores, st);
    return launch_gemm_t<1, 2, 1, 2>(sh, q_parts, q_exp, nq, cent_parts, cent_exp, cent_norm, scores,
                                     st);
  }
  // 256 x 256 tiles of 16 waves or 128 x 128 tiles of 8 waves (two blocks per CU): the
  // one that a fit to measured launches expects to finish first (us).  A launch of
  // small tiles lasts 25 us however little it does (its K loop of d / 16 chunks),
  // then grows with its blocks, 0.1 us each beyond two per CU; a round of big tiles on
  // all 256 CUs lasts 85 us, a part-full last round 55 us plus 0.11 us per block.
  const long long big_blocks = (long long)((nq + 255) / 256) * ((sh.nlist + 255) / 256);
  const long long mid_blocks = (long long)((nq + 127) / 128) * ((sh.nlist + 127) / 128);
  const double t_mid = mid_blocks <= 512
                           ? 25.0 + 0.0625 * (double)std::max<long long>(0, mid_blocks - 128)
                           : 0.1 * (double)mid_blocks;
  const long long rem = big_blocks % 256;
  const double t_big = 85.0 * (double)(big_blocks / 256) + (rem ? 55.0 + 0.11 * (double)rem : 0.0);
  if (t_big <= t_mid)
    return launch_gemm_t<4, 4, 2, 2>(sh, q_parts, q_exp, nq, cent_parts, cent_exp, cent_norm,
                                     scores, st);
  return launch_gemm_t<4, 2, 1, 2>(sh, q_parts, q_exp, nq, cent_parts, cent_exp, cent_norm, scores,
                                   st);
}

// ---------------------------------------------------------------------------
// Exact per-query selection of the `keep` best (score, id) pairs, best first,
// ties to the smaller cluster id.  64-bit key = ordered score bits : id; an
// MSB-first radix select finds the keep-th smallest key, a final pass collects
// everything not larger and a counting pass ranks it.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t score_bits(float s, int metric_ip) {
  uint32_t u = __float_as_uint(s);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending with s
  return metric_ip ? ~u : u;                        // IP: larger score first
}

constexpr int kSelBins = 2048;  // 11-bit digits

__device__ __forceinline__ unsigned long long sel_key(float s, int metric_ip, int c) {
  return ((unsigned long long)score_bits(s, metric_ip) << 32) | (unsigned)c;
}

// Exact order of `filled` collected candidates (64-bit keys in sel[0..cap), slots
// beyond `filled` hold ~0; cap a power of two): the `keep` best go to out[], best
// first, entries from there up to nprobe become -1.  Keys are distinct (the id is part
// of them), so the number of keys that come before a candidate's is its rank.  Up to
// NT candidates: every thread counts, for one candidate, one stretch of the others,
// and the stretches' counts are added up in LDS (lanes of a wavefront compare against
// the same key at a time, one LDS broadcast); more (nprobe in the thousands): counting
// would cost filled^2 / NT comparisons per thread, so the block sorts them.
// rank: NT words of LDS.  Called by every thread of the block.
// ordered == 0 (the search path, which routes probes in cluster-id order anyway): a
// large candidate set is not sorted; the keep-th smallest key is found by a radix
// search over the keys' bytes and the keys up to it are written in no particular
// order, except that the best cluster still comes first (the scan's visiting order
// groups queries by it).
template <int NT>
__device__ __forceinline__ void sel_rank_emit(unsigned long long *sel, int filled, int cap, int keep,
                                              int nprobe, int32_t *out, unsigned int *rank,
                                              int ordered) {
  const int tid = threadIdx.x;
  int n2 = 64;
  while (n2 < filled) n2 <<= 1;
  __syncthreads();
  if (n2 > NT && !ordered && filled > keep) {
    __shared__ unsigned long long s_prefix2, s_mask2, s_best;
    __shared__ unsigned int s_need2, s_slot;
    unsigned int *hist = rank;  // 256 bins
    if (tid == 0) {
      s_prefix2 = 0ull;
      s_mask2 = 0ull;
      s_need2 = (unsigned)keep;
      s_slot = 1u;
      s_best = ~0ull;
    }
    for (int pass = 0; pass < 8; ++pass) {
      const int shift = 56 - 8 * pass;
      if (tid < 256) hist[tid] = 0u;
      __syncthreads();
      const unsigned long long prefix = s_prefix2, mask = s_mask2;
      const unsigned need = s_need2;
      for (int i = tid; i < filled; i += NT) {
        const unsigned long long key = sel[i];
        if ((key & mask) == prefix) atomicAdd(&hist[(unsigned)(key >> shift) & 255u], 1u);
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
          s_need2 = need - cum;
          s_prefix2 = prefix | ((unsigned long long)(tid * 4 + b) << shift);
          s_mask2 = mask | (0xffull << shift);
        }
      }
      __syncthreads();
    }
    const unsigned long long thr = s_prefix2;  // the keep-th smallest key itself
    unsigned long long mine_best = ~0ull;
    for (int i = tid; i < filled; i += NT) mine_best = min(mine_best, sel[i]);
    atomicMin(&s_best, mine_best);
    __syncthreads();
    const unsigned long long best = s_best;
    for (int i = tid; i < filled; i += NT) {
      const unsigned long long key = sel[i];
      if (key > thr) continue;
      const unsigned slot = key == best ? 0u : atomicAdd(&s_slot, 1u);
      out[slot] = (int32_t)(key & 0xffffffffull);
    }
    for (int p = keep + tid; p < nprobe; p += NT) out[p] = -1;
    return;
  }
  if (n2 <= NT) {
    if (tid < n2) rank[tid] = 0u;
    __syncthreads();
    const int i = tid & (n2 - 1), part = tid / n2, n_parts = NT / n2;
    const int per = (filled + n_parts - 1) / n_parts;
    if (i < filled) {
      const unsigned long long mine = sel[i];
      const int j1 = min(filled, (part + 1) * per);
      unsigned cnt = 0;
      for (int j = part * per; j < j1; ++j) cnt += sel[j] < mine ? 1u : 0u;
      if (cnt) atomicAdd(&rank[i], cnt);
    }
    __syncthreads();
    if (tid < filled) {
      const unsigned r = rank[tid];
      if (r < (unsigned)keep) out[r] = (int32_t)(sel[tid] & 0xffffffffull);
    }
  } else {
    for (int size = 2; size <= cap; size <<= 1) {
      for (int st = size >> 1; st > 0; st >>= 1) {
        for (int i = tid; i < cap; i += NT) {
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
    for (int r = tid; r < min(filled, keep); r += NT) out[r] = (int32_t)(sel[r] & 0xffffffffull);
  }
  for (int p = min(filled, keep) + tid; p < nprobe; p += NT) out[p] = -1;
}

// PER > 0: the query's row of scores is read once and held in registers (PER per
// thread, nlist <= PER * kSelThreads); PER == 0: every pass re-reads the row.
//
// Fast path: one histogram over 2048 equal-width bins of the score range
// [best, worst] of the row.  Binning is monotone in the score, so every cluster
// in a bin before the one that contains rank `keep` beats every cluster after
// it; all clusters up to and including that bin are collected (a few more than
// `keep`) and sorted exactly by (score bits, id).  If that set does not fit the
// `cap` LDS slots (heavy ties, a degenerate range, non-finite scores), the exact
// MSB-first radix select over the 64-bit keys below does the work instead.
// Two blocks of sixteen wavefronts per CU (eight wavefronts per SIMD) need the kernel
// within 64 vector registers; at 66 the compiler leaves one block per CU and a batch of
// thousands of queries takes a third longer.
template <int PER, int kSelThreads>
__global__ __launch_bounds__(kSelThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_coarse_select(const float *__restrict__ scores,
                                                               int nlist, int metric_ip, int keep,
                                                               int nprobe, int stride, int cap,
                                                               float stash_z,
                                                               int32_t *__restrict__ probe,
                                                               const int32_t *__restrict__ only_flagged,
                                                               int ordered) {
  // only_flagged: the split selection below has served every query but those it flagged
  if (only_flagged && !only_flagged[blockIdx.x]) return;
  constexpr int kSelBinsPerThread = kSelBins / kSelThreads;
  __shared__ unsigned int hist[kSelBins];
  __shared__ unsigned int wsum[kSelThreads / 64];
  __shared__ float wmin[kSelThreads / 64], wmax[kSelThreads / 64];
  __shared__ float wmom[kSelThreads / 64][3];
  __shared__ unsigned long long s_prefix, s_mask;
  __shared__ unsigned int s_need, s_done, s_count, s_bin, s_total;
  extern __shared__ unsigned long long sel[];  // cap entries (+ the stash when PER == 0)
  // PER == 0: clusters met in the low bins during the histogram pass are kept
  // aside (score and id), so that when the bin that holds rank `keep` turns out
  // to lie among them the row need not be read again to collect them
  constexpr int kStash = 1024;
  float *stash_s = reinterpret_cast<float *>(sel + cap);
  int *stash_c = reinterpret_cast<int *>(stash_s + kStash);
  __shared__ unsigned int s_stash;
  const int q = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const float *row = scores + (size_t)q * nlist;
  int32_t *out = probe + (size_t)q * stride;

  float sc[PER > 0 ? PER : 1];
  if (PER > 0) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid + i * kSelThreads;
      sc[i] = c < nlist ? row[c] : 0.0f;
    }
  }
  // body(score, cluster) for every cluster of the row this thread owns
  auto visit = [&](auto body) {
    if (PER > 0) {
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int c = tid + i * kSelThreads;
        if (c < nlist) body(sc[i], c);
      }
    } else {
      // eight loads in flight per thread before their values are used
      int c = tid;
      for (; c + 7 * kSelThreads < nlist; c += 8 * kSelThreads) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = row[c + i * kSelThreads];
#pragma unroll
        for (int i = 0; i < 8; ++i) body(v[i], c + i * kSelThreads);
      }
      for (; c < nlist; c += kSelThreads) body(row[c], c);
    }
  };

  // the same from memory (the rarely taken radix passes do not hold the row in registers)
  auto visit_mem = [&](auto body) {
    for (int c = tid; c < nlist; c += kSelThreads) body(row[c], c);
  };

  if (tid == 0) {
    s_prefix = 0ull;
    s_mask = 0ull;
    s_need = (unsigned)keep;
    s_done = 0u;
    s_count = 0u;
    s_bin = 0xffffffffu;
    s_total = 0u;
    s_stash = 0u;
  }
#pragma unroll
  for (int b = 0; b < kSelBinsPerThread; ++b) hist[tid * kSelBinsPerThread + b] = 0u;

  // ---- fast path ----
  bool fast_ok = false;
  if (keep < nlist) {
    // v = score (L2) or -score (IP): smaller is better
    float vmin = INFINITY, vmax = -INFINITY;
    float ssum = 0.0f, ssq = 0.0f, scnt = 0.0f;  // PER == 0: moments of the sample
    if (PER > 0) {
      visit([&](float s0, int) {
        const float v = metric_ip ? -s0 : s0;
        vmin = fminf(vmin, v);
        vmax = fmaxf(vmax, v);
      });
    } else {
      // the row is not held in registers: take the range from every 16th stretch of
      // it and leave room below (binning clamps, so it stays monotone whatever
      // the range is; a range that turns out too narrow only sends the block to
      // the exact fall-back)
      for (int c = tid; c < nlist; c += kSelThreads * 16) {
        const float v = metric_ip ? -row[c] : row[c];
        vmin = fminf(vmin, v);
        vmax = fmaxf(vmax, v);
        ssum += v;
        ssq += v * v;
        scnt += 1.0f;
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      vmin = fminf(vmin, __shfl_xor(vmin, o, 64));
      vmax = fmaxf(vmax, __shfl_xor(vmax, o, 64));
      if (PER == 0) {
        ssum += __shfl_xor(ssum, o, 64);
        ssq += __shfl_xor(ssq, o, 64);
        scnt += __shfl_xor(scnt, o, 64);
      }
    }
    if (lane == 0) {
      wmin[wave] = vmin;
      wmax[wave] = vmax;
      if (PER == 0) {
        wmom[wave][0] = ssum;
        wmom[wave][1] = ssq;
        wmom[wave][2] = scnt;
      }
    }
    __syncthreads();
    ssum = ssq = scnt = 0.0f;
#pragma unroll
    for (int w2 = 0; w2 < kSelThreads / 64; ++w2) {
      vmin = fminf(vmin, wmin[w2]);
      vmax = fmaxf(vmax, wmax[w2]);
      if (PER == 0) {
        ssum += wmom[w2][0];
        ssq += wmom[w2][1];
        scnt += wmom[w2][2];
      }
    }
    if (PER == 0) vmin -= 0.5f * (vmax - vmin);
    const float scale = (float)(kSelBins - 1) / (vmax - vmin);
    const bool usable = scale > 0.0f && scale < INFINITY;  // block-uniform
    if (usable) {
      auto bin_of = [&](float s0) -> unsigned {
        const float v = metric_ip ? -s0 : s0;
        const unsigned b = (unsigned)(int)fmaxf((v - vmin) * scale, 0.0f);
        return b < (unsigned)kSelBins ? b : (unsigned)(kSelBins - 1);
      };
      // bins up to this one are stashed: stash_z standard deviations of the sample
      // on the good side of its mean (the launcher picks stash_z so that a
      // bell-shaped row sends two to three times `keep` clusters there, whatever
      // outliers the sample caught).  The stash holds 1024 clusters; if it
      // overflows or ends before the bin of rank `keep`, the row is read again.
      unsigned stash_bin = 0u;
      if (PER == 0 && stash_z > 0.0f) {
        const float mean = ssum / scnt;
        const float sd = sqrtf(fmaxf(ssq / scnt - mean * mean, 0.0f));
        const float lim =
            fminf(fmaxf((mean - stash_z * sd - vmin) * scale, 0.0f), (float)(kSelBins - 1));
        stash_bin = lim == lim ? (unsigned)(int)lim : 0u;
      }
      if (PER > 0) {
        visit([&](float s0, int) { atomicAdd(&hist[bin_of(s0)], 1u); });
      } else {
        // with a stash only its bins are counted at first: rank `keep` lies among
        // them whenever they hold at least `keep` clusters, and the bins above
        // (nearly all of the row, and the crowded ones) then cost no atomics
        const bool partial = stash_z > 0.0f;  // block-uniform
        visit([&](float s0, int c) {
          const unsigned b = bin_of(s0);
          if (!partial) {
            atomicAdd(&hist[b], 1u);
          } else if (b <= stash_bin) {
            atomicAdd(&hist[b], 1u);
            const unsigned slot = atomicAdd(&s_stash, 1u);
            if (slot < (unsigned)kStash) {
              stash_s[slot] = s0;
              stash_c[slot] = c;
            }
          }
        });
        __syncthreads();
        if (partial && s_stash < (unsigned)keep) {  // too few below the limit: count the rest too
          visit([&](float s0, int) {
            const unsigned b = bin_of(s0);
            if (b > stash_bin) atomicAdd(&hist[b], 1u);
          });
        }
      }
      __syncthreads();
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
      if (before < (unsigned)keep && (unsigned)keep <= before + tsum) {
        unsigned cum = before;
        int b = 0;
        for (; b < kSelBinsPerThread - 1; ++b) {
          if (cum + loc[b] >= (unsigned)keep) break;
          cum += loc[b];
        }
        s_bin = (unsigned)(tid * kSelBinsPerThread + b);
        s_total = cum + loc[b];  // clusters in bins up to and including this one
      }
      __syncthreads();
      const unsigned tbin = s_bin, total = s_total;
      if (total >= (unsigned)keep && total <= (unsigned)cap) {  // block-uniform
        fast_ok = true;
        for (int i = tid; i < cap; i += kSelThreads) sel[i] = ~0ull;
        __syncthreads();
        auto take = [&](float s0, int c) {
          if (bin_of(s0) <= tbin) {
            const unsigned slot = atomicAdd(&s_count, 1u);
            if (slot < (unsigned)cap) sel[slot] = sel_key(s0, metric_ip, c);
          }
        };
        const unsigned n_stash = PER == 0 ? s_stash : 0u;
        if (PER == 0 && tbin <= stash_bin && n_stash <= (unsigned)kStash) {
          for (unsigned i = tid; i < n_stash; i += kSelThreads) take(stash_s[i], stash_c[i]);
        } else {
          visit(take);
        }
      }
    }
  }

  if (!fast_ok) {
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
        visit_mem([&](float s0, int c) {
          const unsigned long long key = sel_key(s0, metric_ip, c);
          if ((key & mask) == prefix) atomicAdd(&hist[(unsigned)(key >> shift) & dmask], 1u);
        });
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
    for (int i = tid; i < cap; i += kSelThreads) sel[i] = ~0ull;
    __syncthreads();
    visit_mem([&](float s0, int c) {
      const unsigned long long key = sel_key(s0, metric_ip, c);
      if (key <= thr) {
        const unsigned slot = atomicAdd(&s_count, 1u);
        if (slot < (unsigned)cap) sel[slot] = key;
      }
    });
    __syncthreads();
  }
  __syncthreads();
  sel_rank_emit<kSelThreads>(sel, (int)min(s_count, (unsigned)cap), cap, keep, nprobe, out, hist,
                             ordered);
}

// ---------------------------------------------------------------------------
// The same selection for a handful of queries over many clusters (the paper's
// batches of a few to a few dozen queries against tens of thousands of lists): one
// block per query would leave the chip idle and spend its time on the latency of
// three passes over a long row, so the row is cut into kSelParts parts with a block
// each, and the passes become small kernels: range of each part; histogram of each
// part over the query's common range, added into one histogram per query; the
// clusters up to the bin that holds rank `keep` appended to one candidate list per
// query; exact ranking of the candidates.  Everything that made the one-block fast
// path give up (candidates that do not fit, a degenerate range) flags the query,
// and the one-block kernel then runs for the flagged queries only.  The result is
// the exact selection either way.
// Workspace per query: SelSplitWs below.
// ---------------------------------------------------------------------------
constexpr int kSelParts = 32;
constexpr int kSelPartThreads = 256;
constexpr int kSelPartPer = 8;  // scores per thread: parts of up to 2048 clusters
constexpr int kSelSplitCap = 4096;

struct SelSplitWs {
  float minmax[kSelParts][2];
  unsigned int hist[kSelBins];
  unsigned int count;   // candidates appended
  int flag;             // 1: leave the query to the one-block kernel
  unsigned int pad[62];
  unsigned long long cand[kSelSplitCap];
};
static_assert(sizeof(SelSplitWs) % 256 == 0, "workspace entries stay aligned");

// one entry per query, then one flag word per query
static size_t coarse_select_split_entries_bytes() { return sizeof(SelSplitWs) * (size_t)kSelSplitMaxNq; }
size_t coarse_select_split_bytes() {
  return coarse_select_split_entries_bytes() + (size_t)kSelSplitMaxNq * sizeof(int32_t);
}

__device__ __forceinline__ void sel_part_load(const float *__restrict__ row, int nlist, int part_len,
                                              int metric_ip, float (&v)[kSelPartPer],
                                              int (&c)[kSelPartPer]) {
  const int base = blockIdx.x * part_len;
#pragma unroll
  for (int i = 0; i < kSelPartPer; ++i) {
    const int o = threadIdx.x + i * kSelPartThreads;
    c[i] = (o < part_len && base + o < nlist) ? base + o : -1;
    const float s0 = c[i] >= 0 ? row[c[i]] : 0.0f;
    v[i] = metric_ip ? -s0 : s0;  // smaller is better
  }
}

__global__ __launch_bounds__(kSelPartThreads) void k_sel_part_range(
    const float *__restrict__ scores, int nlist, int part_len, int metric_ip, SelSplitWs *ws) {
  __shared__ float wmin[kSelPartThreads / 64], wmax[kSelPartThreads / 64];
  const int q = blockIdx.y, tid = threadIdx.x;
  SelSplitWs &W = ws[q];
  float v[kSelPartPer];
  int c[kSelPartPer];
  sel_part_load(scores + (size_t)q * nlist, nlist, part_len, metric_ip, v, c);
  float vmin = INFINITY, vmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < kSelPartPer; ++i)
    if (c[i] >= 0) {
      vmin = fminf(vmin, v[i]);
      vmax = fmaxf(vmax, v[i]);
    }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    vmin = fminf(vmin, __shfl_xor(vmin, o, 64));
    vmax = fmaxf(vmax, __shfl_xor(vmax, o, 64));
  }
  if ((tid & 63) == 0) {
    wmin[tid >> 6] = vmin;
    wmax[tid >> 6] = vmax;
  }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < kSelPartThreads / 64; ++w) {
      vmin = fminf(vmin, wmin[w]);
      vmax = fmaxf(vmax, wmax[w]);
    }
    W.minmax[blockIdx.x][0] = vmin;
    W.minmax[blockIdx.x][1] = vmax;
  }
  // the query's histogram and counters start from zero (this kernel precedes their use)
  if (blockIdx.x == 0) {
    for (int b = tid; b < kSelBins; b += kSelPartThreads) W.hist[b] = 0u;
    if (tid == 0) {
      W.count = 0u;
      W.flag = 0;
    }
  }
}

// common range of a query's parts -> (vmin, scale); false if the range cannot be binned
__device__ __forceinline__ bool sel_part_scale(const SelSplitWs &W, int parts, float *vmin_out,
                                               float *scale_out) {
  float vmin = INFINITY, vmax = -INFINITY;
  for (int p = 0; p < parts; ++p) {
    vmin = fminf(vmin, W.minmax[p][0]);
    vmax = fmaxf(vmax, W.minmax[p][1]);
  }
  const float scale = (float)(kSelBins - 1) / (vmax - vmin);
  *vmin_out = vmin;
  *scale_out = scale;
  return scale > 0.0f && scale < INFINITY;
}

__device__ __forceinline__ unsigned sel_part_bin(float v, float vmin, float scale) {
  const unsigned b = (unsigned)(int)fmaxf((v - vmin) * scale, 0.0f);
  return b < (unsigned)kSelBins ? b : (unsigned)(kSelBins - 1);
}

__global__ __launch_bounds__(kSelPartThreads) void k_sel_part_hist(
    const float *__restrict__ scores, int nlist, int part_len, int metric_ip, SelSplitWs *ws) {
  __shared__ unsigned int hist[kSelBins];
  const int q = blockIdx.y, tid = threadIdx.x;
  SelSplitWs &W = ws[q];
  float vmin, scale;
  if (!sel_part_scale(W, gridDim.x, &vmin, &scale)) return;  // uniform over the query's blocks
  for (int b = tid; b < kSelBins; b += kSelPartThreads) hist[b] = 0u;
  float v[kSelPartPer];
  int c[kSelPartPer];
  sel_part_load(scores + (size_t)q * nlist, nlist, part_len, metric_ip, v, c);
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSelPartPer; ++i)
    if (c[i] >= 0) atomicAdd(&hist[sel_part_bin(v[i], vmin, scale)], 1u);
  __syncthreads();
  for (int b = tid; b < kSelBins; b += kSelPartThreads) {
    const unsigned n = hist[b];
    if (n) atomicAdd(&W.hist[b], n);
  }
}

__global__ __launch_bounds__(kSelPartThreads) void k_sel_part_collect(
    const float *__restrict__ scores, int nlist, int part_len, int metric_ip, int keep, int cap,
    SelSplitWs *ws) {
  constexpr int kPerThread = kSelBins / kSelPartThreads;
  __shared__ unsigned int wsum[kSelPartThreads / 64];
  __shared__ unsigned int s_bin, s_total, s_n, s_base;
  const int q = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  SelSplitWs &W = ws[q];
  float vmin, scale;
  if (!sel_part_scale(W, gridDim.x, &vmin, &scale)) {
    if (blockIdx.x == 0 && tid == 0) W.flag = 1;
    return;
  }
  if (tid == 0) {
    s_bin = 0xffffffffu;
    s_total = 0u;
    s_n = 0u;
  }
  // the bin that holds rank `keep` (every block of the query finds the same one)
  unsigned loc[kPerThread], tsum = 0;
#pragma unroll
  for (int b = 0; b < kPerThread; ++b) {
    loc[b] = W.hist[tid * kPerThread + b];
    tsum += loc[b];
  }
  unsigned incl = tsum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned u = __shfl_up(incl, o, 64);
    if (lane >= o) incl += u;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  unsigned before = incl - tsum;
  for (int w2 = 0; w2 < wave; ++w2) before += wsum[w2];
  if (before < (unsigned)keep && (unsigned)keep <= before + tsum) {
    unsigned cum = before;
    int b = 0;
    for (; b < kPerThread - 1; ++b) {
      if (cum + loc[b] >= (unsigned)keep) break;
      cum += loc[b];
    }
    s_bin = (unsigned)(tid * kPerThread + b);
    s_total = cum + loc[b];
  }
  __syncthreads();
  const unsigned tbin = s_bin, total = s_total;
  if (total < (unsigned)keep || total > (unsigned)cap) {  // uniform over the query's blocks
    if (blockIdx.x == 0 && tid == 0) W.flag = 1;
    return;
  }
  float v[kSelPartPer];
  int c[kSelPartPer];
  sel_part_load(scores + (size_t)q * nlist, nlist, part_len, metric_ip, v, c);
  bool take[kSelPartPer];
  unsigned slot[kSelPartPer];
#pragma unroll
  for (int i = 0; i < kSelPartPer; ++i) {
    take[i] = c[i] >= 0 && sel_part_bin(v[i], vmin, scale) <= tbin;
    slot[i] = take[i] ? atomicAdd(&s_n, 1u) : 0u;
  }
  __syncthreads();
  if (tid == 0) s_base = s_n ? atomicAdd(&W.count, s_n) : 0u;
  __syncthreads();
  const unsigned base = s_base;
#pragma unroll
  for (int i = 0; i < kSelPartPer; ++i)
    if (take[i]) {
      const float s0 = metric_ip ? -v[i] : v[i];
      W.cand[base + slot[i]] = sel_key(s0, metric_ip, c[i]);  // base + slot < total <= cap
    }
}

__global__ __launch_bounds__(1024) void k_sel_part_rank(SelSplitWs *ws, int keep, int nprobe,
                                                        int stride, int cap, int ordered,
                                                        int32_t *__restrict__ probe,
                                                        int32_t *__restrict__ flags) {
  extern __shared__ unsigned long long sel[];  // cap entries
  __shared__ unsigned int rank[1024];
  const int q = blockIdx.x, tid = threadIdx.x;
  SelSplitWs &W = ws[q];
  const int flag = W.flag;  // uniform
  if (tid == 0) flags[q] = flag;
  if (flag) return;
  const int filled = (int)min(W.count, (unsigned)cap);
  for (int i = tid; i < cap; i += 1024) sel[i] = i < filled ? W.cand[i] : ~0ull;
  sel_rank_emit<1024>(sel, filled, cap, keep, nprobe, probe + (size_t)q * stride, rank, ordered);
}

hipError_t launch_coarse_select(const Shape &sh, const float *scores, int nq, int nprobe,
                                int probe_stride, int32_t *probe, void *split_ws, int ordered,
                                hipStream_t st) {
  const int keep = nprobe < sh.nlist ? nprobe : sh.nlist;
  int cap = 128;  // LDS slots for collected candidates: a power of two >= 2 * keep
  while (cap < 2 * keep) cap <<= 1;
  const int32_t *only_flagged = nullptr;
  // few queries, long rows, more probes than the one-block kernel's side buffer of low-bin
  // clusters serves (it then reads the row three times): the split selection first, the
  // one-block kernel for what it flags
  if (split_ws && nq <= kSelSplitMaxNq && sh.nlist > 16 * 1024 && keep < sh.nlist && keep > 533 &&
      cap <= kSelSplitCap) {
    int parts = kSelParts;
    int part_len = (sh.nlist + parts - 1) / parts;
    if (part_len > kSelPartThreads * kSelPartPer) {  // more than 65536 lists: more parts would be
      part_len = 0;                                  // needed than the workspace holds
    }
    if (part_len > 0) {
      SelSplitWs *ws = static_cast<SelSplitWs *>(split_ws);
      const dim3 grid(parts, nq);
      hipLaunchKernelGGL(k_sel_part_range, grid, dim3(kSelPartThreads), 0, st, scores, sh.nlist,
                         part_len, sh.metric_ip, ws);
      hipLaunchKernelGGL(k_sel_part_hist, grid, dim3(kSelPartThreads), 0, st, scores, sh.nlist,
                         part_len, sh.metric_ip, ws);
      hipLaunchKernelGGL(k_sel_part_collect, grid, dim3(kSelPartThreads), 0, st, scores, sh.nlist,
                         part_len, sh.metric_ip, keep, cap, ws);
      int32_t *flag_arr = reinterpret_cast<int32_t *>(reinterpret_cast<unsigned char *>(split_ws) +
                                                      coarse_select_split_entries_bytes());
      hipLaunchKernelGGL(k_sel_part_rank, dim3(nq), dim3(1024), (size_t)cap * 8, st, ws, keep,
                         nprobe, probe_stride, cap, ordered, probe, flag_arr);
      only_flagged = flag_arr;
    }
  }
  // PER == 0 only: how far from the mean the stash reaches.  For a bell-shaped row
  // the stash should catch about 2.4 * keep clusters (never more than 800 of its
  // 1024 slots); P(z < -stash_z) = that share of the row.  Solved by bisection
  // on erfc; 0 (no stash) when even 1.5 * keep clusters would not fit.
  float stash_z = 0.0f;
  if (sh.nlist > 16 * 1024 && keep * 3 / 2 <= 800) {
    const double want = std::min(800.0, 2.4 * keep) / (double)sh.nlist;
    double lo = 0.0, hi = 8.0;
    for (int it = 0; it < 60; ++it) {
      const double mid = 0.5 * (lo + hi);
      if (0.5 * erfc(mid / sqrt(2.0)) > want) lo = mid; else hi = mid;
    }
    stash_z = (float)lo;
  }
#define IVF_SEL_LAUNCH(PER, THREADS)                                                          \
  hipLaunchKernelGGL((k_coarse_select<PER, THREADS>), dim3(nq), dim3(THREADS),                   \
                     (size_t)cap * 8 + (PER == 0 ? 1024 * 8 : 0),                                \
                     st, scores, sh.nlist, sh.metric_ip, keep, nprobe, probe_stride, cap, stash_z, probe, \
                     only_flagged, ordered)
  // the row of scores in registers (4 or 16 per thread) up to 16384 clusters, re-read above
  if (sh.nlist <= 4 * 1024) IVF_SEL_LAUNCH(4, 1024);
  else if (sh.nlist <= 16 * 1024) IVF_SEL_LAUNCH(16, 1024);
  else IVF_SEL_LAUNCH(0, 1024);
#undef IVF_SEL_LAUNCH
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Coarse quantizer for callers that cannot allocate or bring a workspace: the
// split queries, their scales and the score matrix live in a file-scope device
// array instead of the index's per-batch workspace.  The array's name is only a
// host-side handle; its device address is looked up once per device
// (static_scratch_for_device) and that pointer is what the kernels get.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];

hipError_t static_scratch_for_device(int device, void **ptr) {
  *ptr = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  void *p = g_scratch_ptr[device].load(std::memory_order_acquire);
  if (!p) {
    // every device holds its own copy of the array at its own address: ask with that
    // device current (two threads asking at once get the same answer)
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return e;
    if (cur != device) return hipErrorInvalidDevice;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[device].store(p, std::memory_order_release);
  }
  *ptr = p;
  return hipSuccess;
}

static size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t coarse_static_bytes(const Shape &sh, int64_t nq) {
  return round256((size_t)nq * sh.d * 4 + kSplitPadBytes) + round256((size_t)nq * 4) +
         round256((size_t)nq * sh.nlist * 4);
}

hipError_t launch_coarse_probe_static(const Shape &sh, const float *queries, int nq, int nprobe,
                                      const void *cent_parts, const int32_t *cent_exp,
                                      const float *cent_norm, void *scratch_ptr, int32_t *out_probe,
                                      hipStream_t st) {
  if (!scratch_ptr || coarse_static_bytes(sh, nq) > (size_t)kStaticScratchBytes)
    return hipErrorInvalidValue;
  unsigned char *base = static_cast<unsigned char *>(scratch_ptr);
  void *q_parts = base;
  int32_t *q_exp = reinterpret_cast<int32_t *>(base + round256((size_t)nq * sh.d * 4 + kSplitPadBytes));
  float *scores = reinterpret_cast<float *>(reinterpret_cast<unsigned char *>(q_exp) +
                                            round256((size_t)nq * 4));
  // Nothing in the array has to start at zero: every word the kernels read for a row
  // or column they store was written earlier in this call; the operand padding the
  // GEMM reads unchecked only feeds rows of the product that are never stored.
  hipError_t e = launch_split_f16(queries, (size_t)nq, sh.d, q_parts, q_exp, st);
  if (e != hipSuccess) return e;
  e = launch_coarse_gemm(sh, q_parts, q_exp, nq, cent_parts, cent_exp, cent_norm, scores, st);
  if (e != hipSuccess) return e;
  return launch_coarse_select(sh, scores, nq, nprobe, nprobe, out_probe, nullptr, 1, st);
}

}  // namespace ivf
