#include "host_scan.h"

#include <immintrin.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <mutex>
#include <thread>

#include "lut_quant.h"

namespace ivf {

int cpu_threads() {
  static int n = [] {
    int v = 0;
    if (const char *e = getenv("IVF_CPU_THREADS")) v = atoi(e);
    if (v <= 0) {
      if (const char *e = getenv("OMP_NUM_THREADS")) v = atoi(e);
    }
    if (v <= 0) v = (int)std::thread::hardware_concurrency();
    if (v <= 0) v = 1;
    return std::min(v, 256);
  }();
  return n;
}

struct WorkerPool::Impl {
  std::mutex mu;
  std::condition_variable cv_work, cv_done;
  std::vector<std::thread> threads;
  std::function<void()> job;
  uint64_t generation = 0;
  int want = 0, started = 0, finished = 0;
  bool busy = false, stop = false;
};

WorkerPool &WorkerPool::get() {
  static WorkerPool pool;
  return pool;
}

WorkerPool::WorkerPool() : impl_(new Impl()), n_threads_(cpu_threads()) {
  impl_->threads.reserve((size_t)n_threads_);
  for (int i = 0; i < n_threads_; ++i) impl_->threads.emplace_back([this] { worker(); });
}

WorkerPool::~WorkerPool() {
  {
    std::lock_guard<std::mutex> lk(impl_->mu);
    impl_->stop = true;
  }
  impl_->cv_work.notify_all();
  for (auto &t : impl_->threads) t.join();
  delete impl_;
}

void WorkerPool::worker() {
  Impl &p = *impl_;
  uint64_t seen = 0;
  std::unique_lock<std::mutex> lk(p.mu);
  for (;;) {
    p.cv_work.wait(lk, [&] { return p.stop || (p.generation != seen && p.started < p.want); });
    if (p.stop) return;
    seen = p.generation;
    p.started += 1;
    std::function<void()> job = p.job;
    lk.unlock();
    job();
    lk.lock();
    p.finished += 1;
    if (p.finished == p.want) p.cv_done.notify_all();
  }
}

bool WorkerPool::start(int n, std::function<void()> fn) {
  Impl &p = *impl_;
  n = std::min(n, n_threads_);
  if (n <= 0) return false;
  {
    std::lock_guard<std::mutex> lk(p.mu);
    if (p.busy) return false;
    p.busy = true;
    p.job = std::move(fn);
    p.want = n;
    p.started = 0;
    p.finished = 0;
    p.generation += 1;
  }
  p.cv_work.notify_all();
  return true;
}

void WorkerPool::wait() {
  Impl &p = *impl_;
  std::unique_lock<std::mutex> lk(p.mu);
  p.cv_done.wait(lk, [&] { return p.finished == p.want; });
  p.job = nullptr;
  p.busy = false;
}

void parallel_for(int64_t n, const std::function<void(int64_t)> &fn,
                  const std::function<void()> *caller_first) {
  if (n <= 0) {
    if (caller_first) (*caller_first)();
    return;
  }
  int nt = (int)std::min<int64_t>(cpu_threads(), n);
  if (nt <= 1) {
    if (caller_first) (*caller_first)();
    for (int64_t i = 0; i < n; ++i) fn(i);
    return;
  }
  std::atomic<int64_t> next(0);
  auto work = [&]() {
    for (;;) {
      int64_t i = next.fetch_add(1, std::memory_order_relaxed);
      if (i >= n) break;
      fn(i);
    }
  };
  // the caller is one of the nt threads
  WorkerPool &pool = WorkerPool::get();
  if (pool.start(nt - 1, work)) {
    if (caller_first) (*caller_first)();
    work();
    pool.wait();
    return;
  }
  std::vector<std::thread> th;  // the pool is taken: threads of our own
  th.reserve(nt - 1);
  for (int t = 1; t < nt; ++t) th.emplace_back(work);
  if (caller_first) (*caller_first)();
  work();
  for (auto &t : th) t.join();
}

float cpu_residual_pv(const HostIndexView &ix, int64_t n_total, float *pv) {
  (void)n_total;
  std::vector<float> list_max((size_t)ix.nlist, 0.0f);
  parallel_for(ix.nlist, [&](int64_t c) {
    const float *cen = ix.centroids + (size_t)c * ix.d;
    float mx = 0.0f;
    for (int64_t v = ix.list_offsets[c]; v < ix.list_offsets[c + 1]; ++v) {
      const uint8_t *code = ix.codes + (size_t)v * ix.M;
      const int ksub = 1 << ix.nbits;
      float acc = 0.0f;
      for (int m = 0; m < ix.msub; ++m) {
        const int j = ix.nbits == 8 ? code[m] : (code[m >> 1] >> (4 * (m & 1))) & 15;
        acc = residual_pv_accumulate(acc, ix.codebooks + ((size_t)m * ksub + j) * ix.dsub,
                                     cen + (size_t)m * ix.dsub, ix.dsub);
      }
      pv[v] = acc;
      mx = std::max(mx, fabsf(acc));
    }
    list_max[(size_t)c] = mx;
  });
  float mx = 0.0f;
  for (float v : list_max) mx = std::max(mx, v);
  return mx;
}

float cpu_max_bias(const HostIndexView &ix, const float *q, const int32_t *clusters, int n) {
  if (!ix.by_residual) return 0.0f;
  float mx = 0.0f;
  for (int i = 0; i < n; ++i) {
    if (clusters[i] < 0) continue;
    mx = std::max(mx, fabsf(residual_bias_host(ix.metric_ip, q,
                                               ix.centroids + (size_t)clusters[i] * ix.d, ix.d)));
  }
  return mx;
}

void cpu_transpose_codebooks(const HostIndexView &ix, float *out) {
  const int ksub = 1 << ix.nbits;
  for (int s = 0; s < ix.msub; ++s)
    for (int j = 0; j < ksub; ++j)
      for (int t = 0; t < ix.dsub; ++t)
        out[((size_t)s * ix.dsub + t) * ksub + j] =
            ix.codebooks[((size_t)s * ksub + j) * ix.dsub + t];
}

// out[j] = lut_entry(kind, q, codeword j) for the n codewords of one
// sub-quantizer, ct = its codewords element-major ([dsub][n]).  The loop over j
// is innermost and independent, so the compiler turns it into vector fused
// multiply-adds; every j still takes lut_entry's operations in lut_entry's order,
// hence the same bits.
template <int NB>
static inline void lut_column_block(int kind, const float *__restrict__ q,
                                    const float *__restrict__ ct, int dsub, int n,
                                    float *__restrict__ out) {
  float acc[NB];
  for (int j = 0; j < NB; ++j) acc[j] = 0.0f;
  if (kind != kLutL2) {
    for (int t = 0; t < dsub; ++t) {
      const float qt = q[t];
      const float *c = ct + (size_t)t * n;
      for (int j = 0; j < NB; ++j) acc[j] = __builtin_fmaf(qt, c[j], acc[j]);
    }
    const float sc = kind == kLutIP ? -1.0f : -2.0f;  // exact either way
    for (int j = 0; j < NB; ++j) out[j] = sc * acc[j];
  } else {
    for (int t = 0; t < dsub; ++t) {
      const float qt = q[t];
      const float *c = ct + (size_t)t * n;
      for (int j = 0; j < NB; ++j) {
        const float diff = qt - c[j];
        acc[j] = __builtin_fmaf(diff, diff, acc[j]);
      }
    }
    for (int j = 0; j < NB; ++j) out[j] = acc[j];
  }
}

static void lut_column(int kind, const float *q, const float *ct, int dsub, int n, float *out) {
  if (n == 16) return lut_column_block<16>(kind, q, ct, dsub, n, out);
  for (int j0 = 0; j0 < n; j0 += 64) lut_column_block<64>(kind, q, ct + j0, dsub, n, out + j0);
}

// The 256 entries of one column for NQ queries at once, with 512-bit vectors: the
// codewords (the larger operand: 256 x dsub floats per column, 786 KB per table at
// 768 dimensions) are read once for all of them.  Every lane does lut_entry's
// operations in lut_entry's order, hence the same bits.
// mx[b]: sixteen running maxima of |entry| per query (a NaN entry is skipped, as fmaxf
// skips it on the device).
template <int NQ>
__attribute__((target("avx512f"))) static void lut_column_wide(int kind, const float *const *q,
                                                               const float *ct, int dsub,
                                                               float *const *out, __m512 *mx) {
  const __m512 sc = _mm512_set1_ps(kind == kLutIP ? -1.0f : -2.0f);  // exact either way
  for (int j0 = 0; j0 < 256; j0 += 64) {
    __m512 acc[NQ][4];
#pragma unroll
    for (int b = 0; b < NQ; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[b][i] = _mm512_setzero_ps();
    for (int t = 0; t < dsub; ++t) {
      __m512 c[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) c[i] = _mm512_loadu_ps(ct + (size_t)t * 256 + j0 + 16 * i);
#pragma unroll
      for (int b = 0; b < NQ; ++b) {
        const __m512 qt = _mm512_set1_ps(q[b][t]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (kind != kLutL2) {
            acc[b][i] = _mm512_fmadd_ps(qt, c[i], acc[b][i]);
          } else {
            const __m512 diff = _mm512_sub_ps(qt, c[i]);
            acc[b][i] = _mm512_fmadd_ps(diff, diff, acc[b][i]);
          }
        }
      }
    }
#pragma unroll
    for (int b = 0; b < NQ; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const __m512 v = kind != kLutL2 ? _mm512_mul_ps(sc, acc[b][i]) : acc[b][i];
        _mm512_storeu_ps(out[b] + j0 + 16 * i, v);
        mx[b] = _mm512_max_ps(_mm512_abs_ps(v), mx[b]);  // (a > mx) ? a : mx, lane by lane
      }
  }
}

// The float table in fixed point with exponent e, 512 bits at a time (lut_quantize
// lane by lane: the scaling as an exact product, round to nearest even, 0 for what
// does not fit).
__attribute__((target("avx512f"))) static void lut_quantize_wide(const float *f, size_t n, int e,
                                                                 int32_t *lut) {
  const __m512 scale = _mm512_set1_ps(ldexpf(1.0f, e));
  const __m512 lim = _mm512_set1_ps(2147483520.0f);
  for (size_t i = 0; i < n; i += 16) {
    const __m512 r = _mm512_roundscale_ps(_mm512_mul_ps(_mm512_loadu_ps(f + i), scale),
                                          _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
    const __mmask16 ok = _mm512_cmp_ps_mask(_mm512_abs_ps(r), lim, _CMP_LT_OQ);
    _mm512_storeu_si512((void *)(lut + i), _mm512_maskz_cvttps_epi32(ok, r));
  }
}

// Largest |entry| of the float table f, the scale exponent it gives, and the table in
// fixed point.
static int lut_finish(const HostIndexView &ix, const float *f, float max_bias, int32_t *lut) {
  const size_t n = (size_t)ix.M * 256;
  // sixteen running maxima so that the loop vectorizes (a NaN entry is skipped, as
  // fmaxf skips it on the device)
  float lane_mx[16];
  for (int l = 0; l < 16; ++l) lane_mx[l] = 0.0f;
  for (size_t i = 0; i < n; i += 16)
    for (int l = 0; l < 16; ++l) {
      const float a = fabsf(f[i + l]);
      lane_mx[l] = a > lane_mx[l] ? a : lane_mx[l];
    }
  float mx = 0.0f;
  for (int l = 0; l < 16; ++l) mx = std::max(mx, lane_mx[l]);
  const int e = lut_exponent(mx, ix.M, max_bias, ix.pv ? ix.pv_max : 0.0f);
  // lut_quantize with the scaling written as a product: |e| <= 60, so 2^e is a
  // normal float and v * 2^e rounds exactly as ldexpf(v, e) does
  const float scale = ldexpf(1.0f, e);
  for (size_t i = 0; i < n; ++i) {
    const float r = __builtin_rintf(f[i] * scale);
    lut[i] = __builtin_fabsf(r) < 2147483520.0f ? (int)r : 0;
  }
  return e;
}

// 8-bit codes on a CPU with AVX-512: columns, largest |entry| and fixed point, for one
// query (q1 == NULL) or two.  f: 2 * M * 256 floats of scratch.
__attribute__((target("avx512f"))) static void lut_pair_wide(
    const HostIndexView &ix, int kind, const float *q0, const float *q1, float max_bias0,
    float max_bias1, float *f, int32_t *lut0, int32_t *lut1, int *e0, int *e1) {
  const int M = ix.M, dsub = ix.dsub;
  const size_t n = (size_t)M * 256;
  __m512 mx[2] = {_mm512_setzero_ps(), _mm512_setzero_ps()};
  for (int m = 0; m < M; ++m) {
    const float *qm[2] = {q0 + (size_t)m * dsub, q1 ? q1 + (size_t)m * dsub : nullptr};
    float *om[2] = {f + (size_t)m * 256, f + n + (size_t)m * 256};
    const float *ct = ix.codebooks_t + (size_t)m * dsub * 256;
    if (q1) lut_column_wide<2>(kind, qm, ct, dsub, om, mx);
    else lut_column_wide<1>(kind, qm, ct, dsub, om, mx);
  }
  const float pvm = ix.pv ? ix.pv_max : 0.0f;
  *e0 = lut_exponent(_mm512_reduce_max_ps(mx[0]), M, max_bias0, pvm);
  lut_quantize_wide(f, n, *e0, lut0);
  if (q1) {
    *e1 = lut_exponent(_mm512_reduce_max_ps(mx[1]), M, max_bias1, pvm);
    lut_quantize_wide(f + n, n, *e1, lut1);
  }
}

void cpu_build_lut_pair(const HostIndexView &ix, const float *q0, const float *q1, float max_bias0,
                        float max_bias1, int32_t *lut0, int32_t *lut1, int *e0, int *e1) {
  const int M = ix.M, dsub = ix.dsub;
  const int kind = ix.metric_ip ? kLutIP : (ix.by_residual ? kLutL2Res : kLutL2);
  const size_t n = (size_t)M * 256;
  static const bool wide = __builtin_cpu_supports("avx512f");
  thread_local std::vector<float> f, t;
  f.resize(2 * n);
  const float *qs[2] = {q0, q1};
  const int nb = q1 ? 2 : 1;
  if (ix.nbits == 8 && wide) {
    lut_pair_wide(ix, kind, q0, q1, max_bias0, max_bias1, f.data(), lut0, lut1, e0, e1);
    return;
  } else {
    for (int b = 0; b < nb; ++b) {
      const float *q = qs[b];
      float *fb = &f[(size_t)b * n];
      if (ix.nbits == 8) {
        for (int m = 0; m < M; ++m)
          lut_column(kind, q + (size_t)m * dsub, ix.codebooks_t + (size_t)m * dsub * 256, dsub, 256,
                     fb + (size_t)m * 256);
      } else {
        // 16 entries per sub-quantizer, then one 256-entry column per code byte
        t.resize((size_t)ix.msub * 16);
        for (int s2 = 0; s2 < ix.msub; ++s2)
          lut_column(kind, q + (size_t)s2 * dsub, ix.codebooks_t + (size_t)s2 * dsub * 16, dsub, 16,
                     &t[(size_t)s2 * 16]);
        for (int m = 0; m < M; ++m) {
          const float *lo = &t[(size_t)(2 * m) * 16], *hi = &t[(size_t)(2 * m + 1) * 16];
          float *col = fb + (size_t)m * 256;
          for (int jh = 0; jh < 16; ++jh)
            for (int jl = 0; jl < 16; ++jl) col[jh * 16 + jl] = lut_pair_entry(lo[jl], hi[jh]);
        }
      }
    }
  }
  *e0 = lut_finish(ix, &f[0], max_bias0, lut0);
  if (q1) *e1 = lut_finish(ix, &f[n], max_bias1, lut1);
}

int cpu_build_lut(const HostIndexView &ix, const float *q, float max_bias, int32_t *lut) {
  int e = 0;
  cpu_build_lut_pair(ix, q, nullptr, max_bias, 0.0f, lut, nullptr, &e, nullptr);
  return e;
}

// Sum of a vector's M table entries by plain lookups: eight code bytes per 64-bit
// load, two independent accumulators (integer sums: the order does not matter); M is
// a multiple of 8.
static inline int32_t code_sum(const int32_t *lut, const uint8_t *code, int M) {
  int32_t s0 = 0, s1 = 0;
  for (int m = 0; m < M; m += 8) {
    uint64_t w;
    memcpy(&w, code + m, 8);
    const int32_t *t = lut + m * 256;
    s0 += t[w & 255] + t[512 + ((w >> 16) & 255)] + t[1024 + ((w >> 32) & 255)] +
          t[1536 + ((w >> 48) & 255)];
    s1 += t[256 + ((w >> 8) & 255)] + t[768 + ((w >> 24) & 255)] +
          t[1280 + ((w >> 40) & 255)] + t[1792 + (w >> 56)];
  }
  return (int32_t)((uint32_t)s0 + (uint32_t)s1);
}

static inline bool cand_less(const HostCand &a, const HostCand &b) {
  return a.key < b.key || (a.key == b.key && a.id < b.id);
}

// ---------------------------------------------------------------------------
// Byte-plane scan (CPUs with AVX-512 VBMI).
//
// A table entry is an int32; split into its four bytes, a column of the table
// becomes four 256-entry BYTE tables, each of which fits four 512-bit registers.
// With the codes of a list stored column-major (row m = byte m of every vector
// of the list), one register of 64 code bytes indexes those tables with two
// two-register byte permutes and a blend per plane: 64 lookups of one column in
// twelve instructions, no memory access.  The planes' bytes are summed apart in
// 16-bit lanes (at most 128 columns x 255 < 2^16) and put together at the end:
// sum_p 2^(8p) * (sum over columns of byte p) = the int32 sum of the entries
// modulo 2^32, and the true sum fits an int32 by the choice of the table's
// scale.  So the result is the very integer the plain loop below and the GPU
// scan produce.
// ---------------------------------------------------------------------------
constexpr int kPlaneSegGroups = 32;  // 64-vector groups per pass: 16 KB of partial sums

bool cpu_has_plane_scan() {
  static const bool ok = __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") &&
                         __builtin_cpu_supports("avx512vbmi");
  if (const char *e = getenv("IVF_HOST_SCAN"))
    if (!strcmp(e, "scalar")) return false;
  return ok;
}

int64_t cpu_transposed_bytes(const HostIndexView &ix, int64_t *list_toff) {
  int64_t at = 0;
  for (int c = 0; c < ix.nlist; ++c) {
    if (list_toff) list_toff[c] = at;
    const int64_t len = ix.list_offsets[c + 1] - ix.list_offsets[c];
    at += (int64_t)ix.M * ((len + 63) / 64 * 64);
  }
  if (list_toff) list_toff[ix.nlist] = at;
  return at;
}

void cpu_transpose_codes(const HostIndexView &ix, const int64_t *list_toff, uint8_t *out) {
  const int M = ix.M;
  parallel_for(ix.nlist, [&](int64_t c) {
    const int64_t v0 = ix.list_offsets[c], len = ix.list_offsets[c + 1] - v0;
    const int64_t lpad = (len + 63) / 64 * 64;
    uint8_t *dst = out + list_toff[c];
    for (int64_t b = 0; b < lpad; b += 64) {
      const int64_t nv = std::min<int64_t>(64, len - b);
      for (int m = 0; m < M; ++m) {
        uint8_t *row = dst + (size_t)m * lpad + b;
        const uint8_t *src = ix.codes + (size_t)(v0 + b) * M + m;
        for (int64_t i = 0; i < nv; ++i) row[i] = src[(size_t)i * M];
        for (int64_t i = nv; i < 64; ++i) row[i] = 0;
      }
    }
  });
}

// planes[(m * 4 + p) * 256 + j] = byte p of lut[m * 256 + j]
static void build_planes(const int32_t *lut, int M, uint8_t *planes) {
  for (int m = 0; m < M; ++m) {
    const int32_t *col = lut + (size_t)m * 256;
    uint8_t *pl = planes + (size_t)m * 1024;
    for (int p = 0; p < 4; ++p)
      for (int j = 0; j < 256; ++j) pl[p * 256 + j] = (uint8_t)((uint32_t)col[j] >> (8 * p));
  }
}

// Partial sums of `ng` groups of 64 vectors: acc[g][p][h] holds, for plane p, the
// sums of the group's even (h = 0) and odd (h = 1) vectors as 32 uint16 lanes.
// VARIANT 0 looks a byte up with two two-register permutes and a blend (the
// quicker form on AMD cores), VARIANT 1 with four one-register permutes merged
// under masks (quicker where the two-register permute is split into several
// operations, as on Intel cores).
template <int VARIANT>
__attribute__((target("avx512f,avx512bw,avx512vbmi"))) static void plane_accumulate(
    const uint8_t *rows, size_t stride, int M, int ng, const uint8_t *planes, uint16_t *acc) {
  const __m512i lo8 = _mm512_set1_epi16(0x00ff);
  const __m512i bit6 = _mm512_set1_epi8(0x40);
  memset(acc, 0, (size_t)ng * 512);
  for (int m = 0; m < M; ++m) {
    __m512i T[16];
    for (int r = 0; r < 16; ++r)
      T[r] = _mm512_loadu_si512((const void *)(planes + (size_t)m * 1024 + r * 64));
    const uint8_t *row = rows + (size_t)m * stride;
    for (int g = 0; g < ng; ++g) {
      const __m512i c = _mm512_loadu_si512((const void *)(row + (size_t)g * 64));
      const __mmask64 b7 = _mm512_movepi8_mask(c);  // codes 128..255
      __m512i *a = (__m512i *)(acc + (size_t)g * 256);
      __mmask64 k1 = 0, k2 = 0, k3 = 0;
      if (VARIANT == 1) {
        const __mmask64 b6 = _mm512_test_epi8_mask(c, bit6);
        k1 = b6 & ~b7;
        k2 = ~b6 & b7;
        k3 = b6 & b7;
      }
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        __m512i v;
        if (VARIANT == 0) {
          const __m512i lo = _mm512_permutex2var_epi8(T[4 * p + 0], c, T[4 * p + 1]);
          const __m512i hi = _mm512_permutex2var_epi8(T[4 * p + 2], c, T[4 * p + 3]);
          v = _mm512_mask_blend_epi8(b7, lo, hi);
        } else {
          v = _mm512_permutexvar_epi8(c, T[4 * p + 0]);
          v = _mm512_mask_permutexvar_epi8(v, k1, c, T[4 * p + 1]);
          v = _mm512_mask_permutexvar_epi8(v, k2, c, T[4 * p + 2]);
          v = _mm512_mask_permutexvar_epi8(v, k3, c, T[4 * p + 3]);
        }
        const __m512i ev = _mm512_and_si512(v, lo8);
        const __m512i od = _mm512_srli_epi16(v, 8);
        _mm512_storeu_si512(a + 2 * p, _mm512_add_epi16(_mm512_loadu_si512(a + 2 * p), ev));
        _mm512_storeu_si512(a + 2 * p + 1, _mm512_add_epi16(_mm512_loadu_si512(a + 2 * p + 1), od));
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Filter pass.  Once the query's result list is full, nearly every vector of a
// list is rejected, and a lower bound of its sum is enough to reject it.  With
// mn_m the smallest entry of column m, the entry less mn_m is non-negative, and
// h = min((entry - mn_m) >> 8, 65535) satisfies 256 * h <= entry - mn_m.  So
//   sum_m mn_m + 256 * sum_m h_m(code_m)  <=  the vector's true sum,
// short of it by less than 256 per column unless an entry saturates (only the
// largest entries of a column whose range passes 2^24 do, and they belong to
// vectors far from the query).  h has two bytes, so the bound costs two byte
// planes per column instead of four; a vector whose bound exceeds the worst kept
// key is done, the few others get their exact sum by plain lookups in the row-major
// codes.  Every key that is compared with the result list's is therefore exact,
// and results are the same with or without the filter.
// The inequality also holds with the sum over any subset of the columns (a column
// left out adds nothing below its mn_m, which the base already counts), so the pass
// adds the columns in stretches and drops a group of 64 vectors as soon as all of
// its bounds exceed the worst kept key: for the cold lists of a hybrid batch, which
// mostly lie far from the query, the first eighth of the columns settles nearly
// every group, and the rows of the other columns are never read.
// ---------------------------------------------------------------------------
// filt[(m * 2 + p) * 256 + j] = byte p of h_m(j); returns sum_m mn_m (mod 2^32).
// Only called on CPUs that run the byte-plane scan.
__attribute__((target("avx512f,avx512bw"))) static int32_t build_filter(const int32_t *lut, int M,
                                                                        uint8_t *filt) {
  uint32_t base = 0;
  const __m512i cap = _mm512_set1_epi32(65535);
  for (int m = 0; m < M; ++m) {
    const int32_t *col = lut + (size_t)m * 256;
    __m512i x[16];
    __m512i vmn = _mm512_loadu_si512((const void *)col);
    x[0] = vmn;
    for (int r = 1; r < 16; ++r) {
      x[r] = _mm512_loadu_si512((const void *)(col + 16 * r));
      vmn = _mm512_min_epi32(vmn, x[r]);
    }
    const int32_t mn = _mm512_reduce_min_epi32(vmn);
    base += (uint32_t)mn;
    const __m512i bmn = _mm512_set1_epi32(mn);
    uint8_t *f = filt + (size_t)m * 512;
    for (int r = 0; r < 16; ++r) {
      // (entry - mn) as an unsigned 32-bit value, its bits 8..23 saturated to 16 bits
      const __m512i h = _mm512_min_epu32(_mm512_srli_epi32(_mm512_sub_epi32(x[r], bmn), 8), cap);
      _mm_storeu_si128((__m128i *)(f + 16 * r), _mm512_cvtepi32_epi8(h));
      _mm_storeu_si128((__m128i *)(f + 256 + 16 * r), _mm512_cvtepi32_epi8(_mm512_srli_epi32(h, 8)));
    }
  }
  return (int32_t)base;
}

// acc[group][p][h]: for byte plane p of the filter values, the sums over the columns
// seen so far of the group's even (h = 0) and odd (h = 1) vectors as 32 uint16 lanes
// (at most 128 columns x 255).  A block of up to four groups (numbers in gsel, groups
// of 64 vectors counted from `rows`) keeps its sixteen partial sums in registers while
// the columns m0 .. m1 - 1 go by (a column's two byte tables are reloaded per block of
// groups instead: eight loads from the cache per column against sixteen loads and
// sixteen stores of partial sums); with m0 > 0 the sums continue from what acc holds.
// pf (optional): a cursor through memory that will be read next (the head of the next
// list); one line of it is requested per line of codes read here, so the requests are
// spread over the scan instead of arriving in one burst.
struct PrefetchCursor {
  const uint8_t *at = nullptr, *end = nullptr;
};

template <int VARIANT, int GB>
__attribute__((target("avx512f,avx512bw,avx512vbmi"))) static inline void filter_block(
    const uint8_t *rows, size_t stride, int m0, int m1, const int *gsel, const uint8_t *filt,
    uint16_t *acc, PrefetchCursor *pf) {
  const __m512i lo8 = _mm512_set1_epi16(0x00ff);
  const __m512i bit6 = _mm512_set1_epi8(0x40);
  __m512i s[GB][4];
#pragma unroll
  for (int g = 0; g < GB; ++g)
#pragma unroll
    for (int r = 0; r < 4; ++r)
      s[g][r] = m0 > 0 ? _mm512_loadu_si512((const void *)(acc + (size_t)gsel[g] * 128 + r * 32))
                       : _mm512_setzero_si512();
  for (int m = m0; m < m1; ++m) {
    __m512i T[8];
#pragma unroll
    for (int r = 0; r < 8; ++r)
      T[r] = _mm512_loadu_si512((const void *)(filt + (size_t)m * 512 + r * 64));
    const uint8_t *row = rows + (size_t)m * stride;
    if (pf->at < pf->end) {
#pragma unroll
      for (int g = 0; g < GB; ++g) __builtin_prefetch(pf->at + 64 * g, 0, 2);
      pf->at += 64 * GB;
    }
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      const __m512i c = _mm512_loadu_si512((const void *)(row + (size_t)gsel[g] * 64));
      const __mmask64 b7 = _mm512_movepi8_mask(c);  // codes 128..255
      __mmask64 k1 = 0, k2 = 0, k3 = 0;
      if (VARIANT == 1) {
        const __mmask64 b6 = _mm512_test_epi8_mask(c, bit6);
        k1 = b6 & ~b7;
        k2 = ~b6 & b7;
        k3 = b6 & b7;
      }
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        __m512i v;
        if (VARIANT == 0) {
          const __m512i lo = _mm512_permutex2var_epi8(T[4 * p + 0], c, T[4 * p + 1]);
          const __m512i hi = _mm512_permutex2var_epi8(T[4 * p + 2], c, T[4 * p + 3]);
          v = _mm512_mask_blend_epi8(b7, lo, hi);
        } else {
          v = _mm512_permutexvar_epi8(c, T[4 * p + 0]);
          v = _mm512_mask_permutexvar_epi8(v, k1, c, T[4 * p + 1]);
          v = _mm512_mask_permutexvar_epi8(v, k2, c, T[4 * p + 2]);
          v = _mm512_mask_permutexvar_epi8(v, k3, c, T[4 * p + 3]);
        }
        s[g][2 * p] = _mm512_add_epi16(s[g][2 * p], _mm512_and_si512(v, lo8));
        s[g][2 * p + 1] = _mm512_add_epi16(s[g][2 * p + 1], _mm512_srli_epi16(v, 8));
      }
    }
  }
#pragma unroll
  for (int g = 0; g < GB; ++g)
#pragma unroll
    for (int r = 0; r < 4; ++r)
      _mm512_storeu_si512((void *)(acc + (size_t)gsel[g] * 128 + r * 32), s[g][r]);
}

// Columns m0 .. m1 - 1 for the n listed groups.
template <int VARIANT>
__attribute__((target("avx512f,avx512bw,avx512vbmi"))) static void filter_accumulate(
    const uint8_t *rows, size_t stride, int m0, int m1, const int *gsel, int n,
    const uint8_t *filt, uint16_t *acc, PrefetchCursor *pf) {
  int g = 0;
  for (; g + 4 <= n; g += 4)
    filter_block<VARIANT, 4>(rows, stride, m0, m1, gsel + g, filt, acc, pf);
  switch (n - g) {
    case 3: filter_block<VARIANT, 3>(rows, stride, m0, m1, gsel + g, filt, acc, pf); break;
    case 2: filter_block<VARIANT, 2>(rows, stride, m0, m1, gsel + g, filt, acc, pf); break;
    case 1: filter_block<VARIANT, 1>(rows, stride, m0, m1, gsel + g, filt, acc, pf); break;
    default: break;
  }
}

// Of the n groups listed in gsel, those in which some vector's lower bound (256 x the
// partial sums in acc, plus add: the table's base and the list's bias, plus the
// vector's own term pvq, or NULL) does not exceed bound; nv = vectors from `rows` on
// (the last group may be ragged).  The list is compacted in place; per remaining group
// the vectors in question come back as a bit mask (bit i = vector i of the group) in
// gmask.  Returns how many remain.  The bound is valid whichever columns acc covers so
// far: the base counts every column's smallest entry, and a column not yet seen adds
// nothing below that.
__attribute__((target("avx512f,avx512bw,avx512vbmi,bmi2"))) static int filter_survivors(
    const uint16_t *acc, int *gsel, int n, int64_t nv, uint32_t add, const int32_t *pvq,
    int32_t bound, uint64_t *gmask) {
  const __m512i vadd = _mm512_set1_epi32((int)add);
  const __m512i vbound = _mm512_set1_epi32(bound);
  const __m512i lane = _mm512_set_epi32(15, 14, 13, 12, 11, 10, 9, 8, 7, 6, 5, 4, 3, 2, 1, 0);
  const __m512i idx_even = _mm512_slli_epi32(lane, 1);                       // 0, 2, ..., 30
  const __m512i idx_odd = _mm512_add_epi32(idx_even, _mm512_set1_epi32(1));  // 1, 3, ..., 31
  int kept = 0;
  for (int j = 0; j < n; ++j) {
    const int g = gsel[j];
    const uint16_t *a = acc + (size_t)g * 128;
    const int left = (int)std::min<int64_t>(64, nv - (int64_t)g * 64);  // vectors of this group
    uint64_t any = 0;
    for (int h2 = 0; h2 < 2; ++h2) {  // words 16 * h2 .. + 15 of the even and of the odd vectors
      const __m512i e0 = _mm512_cvtepu16_epi32(_mm256_loadu_si256((const __m256i *)(a + 16 * h2)));
      const __m512i o0 = _mm512_cvtepu16_epi32(_mm256_loadu_si256((const __m256i *)(a + 32 + 16 * h2)));
      const __m512i e1 = _mm512_cvtepu16_epi32(_mm256_loadu_si256((const __m256i *)(a + 64 + 16 * h2)));
      const __m512i o1 = _mm512_cvtepu16_epi32(_mm256_loadu_si256((const __m256i *)(a + 96 + 16 * h2)));
      // 256 * (plane 0 + 256 * plane 1) + add, modulo 2^32 (the true value fits an int32)
      __m512i ke = _mm512_add_epi32(_mm512_slli_epi32(_mm512_add_epi32(e0, _mm512_slli_epi32(e1, 8)), 8), vadd);
      __m512i ko = _mm512_add_epi32(_mm512_slli_epi32(_mm512_add_epi32(o0, _mm512_slli_epi32(o1, 8)), 8), vadd);
      if (pvq) {
        const int32_t *pq = pvq + (size_t)g * 64 + 32 * h2;  // vectors 32 * h2 .. + 31 of the group
        const __m512i p_lo = _mm512_loadu_si512((const void *)pq);
        const __m512i p_hi = _mm512_loadu_si512((const void *)(pq + 16));
        ke = _mm512_add_epi32(ke, _mm512_permutex2var_epi32(p_lo, idx_even, p_hi));
        ko = _mm512_add_epi32(ko, _mm512_permutex2var_epi32(p_lo, idx_odd, p_hi));
      }
      // word w of this half is vector 32 * h2 + 2 * w (even) or + 1 (odd)
      const int rem = left - 32 * h2;  // vectors of the group from this half on
      const __mmask16 ve = rem >= 32 ? (__mmask16)0xffff : rem <= 0 ? (__mmask16)0 : (__mmask16)((1u << ((rem + 1) / 2)) - 1u);
      const __mmask16 vo = rem >= 32 ? (__mmask16)0xffff : rem <= 0 ? (__mmask16)0 : (__mmask16)((1u << (rem / 2)) - 1u);
      const uint64_t me = _mm512_mask_cmple_epi32_mask(ve, ke, vbound);
      const uint64_t mo = _mm512_mask_cmple_epi32_mask(vo, ko, vbound);
      any |= (_pdep_u64(me, 0x55555555ull) | _pdep_u64(mo, 0xaaaaaaaaull)) << (32 * h2);
    }
    if (any) {
      gsel[kept] = g;
      gmask[kept++] = any;
    }
  }
  return kept;
}

// int32 sums in vector order from the partial sums of plane_accumulate
static void plane_combine(const uint16_t *acc, int ng, int32_t *sums) {
  for (int g = 0; g < ng; ++g) {
    const uint16_t *a = acc + (size_t)g * 256;
    int32_t *out = sums + (size_t)g * 64;
    for (int w = 0; w < 32; ++w) {
      uint32_t ev = 0, od = 0;
      for (int p = 0; p < 4; ++p) {
        ev += (uint32_t)a[(2 * p) * 32 + w] << (8 * p);
        od += (uint32_t)a[(2 * p + 1) * 32 + w] << (8 * p);
      }
      out[2 * w] = (int32_t)ev;
      out[2 * w + 1] = (int32_t)od;
    }
  }
}

namespace {
// bounded max-heap on (key, id): the worst kept candidate sits on top
struct TopK {
  std::vector<HostCand> heap;
  int k;
  int32_t cap;  // keys above it are not wanted at all
  TopK(int k_, int32_t cap_) : k(k_), cap(cap_) { heap.reserve((size_t)k_); }
  // every candidate with key above this is certainly rejected
  int32_t bound() const { return (int)heap.size() < k ? cap : std::min(cap, heap.front().key); }
  void offer(const HostCand &cand) {
    if (cand.key > cap) return;
    if ((int)heap.size() < k) {
      heap.push_back(cand);
      std::push_heap(heap.begin(), heap.end(), cand_less);
    } else if (cand_less(cand, heap.front())) {
      std::pop_heap(heap.begin(), heap.end(), cand_less);
      heap.back() = cand;
      std::push_heap(heap.begin(), heap.end(), cand_less);
    }
  }
  void finish(HostCand *out) {
    std::sort_heap(heap.begin(), heap.end(), cand_less);
    for (int r = 0; r < k; ++r)
      out[r] = r < (int)heap.size() ? heap[r] : HostCand{kKeyInvalid, -1};
  }
};
}  // namespace

static const int g_plane_variant = __builtin_cpu_is("intel") ? 1 : 0;

// The filter pass runs unless the environment says IVF_HOST_FILTER=0 (read per
// query, so a test can compare the two in one process).
static bool host_filter_on() {
  const char *e = getenv("IVF_HOST_FILTER");
  return !(e && !strcmp(e, "0"));
}

struct PlaneTables {
  const int32_t *lut;     // the query's table
  const uint8_t *planes;  // build_planes (filter pass off), else NULL
  const uint8_t *filt;    // build_filter (filter pass on), else NULL
  int32_t filt_base;
};

static void plane_scan_list(const HostIndexView &ix, const PlaneTables &tb, int e, int cl,
                            int32_t bias_key, TopK &top, PrefetchCursor *pf) {
  const int64_t v0 = ix.list_offsets[cl], len = ix.list_offsets[cl + 1] - v0;
  const int64_t lpad = (len + 63) / 64 * 64;
  const uint8_t *base = ix.codes_t + ix.list_toff[cl];
  alignas(64) uint16_t acc[kPlaneSegGroups * 256];
  alignas(64) int32_t sums[kPlaneSegGroups * 64];
  alignas(64) int32_t pvq[kPlaneSegGroups * 64];
  int gidx[kPlaneSegGroups];
  uint64_t gmask[kPlaneSegGroups];
  const float scale = ldexpf(1.0f, e);
  // exact key of vector i of the segment at s0, by plain lookups in the row-major codes
  auto exact_offer = [&](int64_t s0, int64_t i, int32_t &bound) {
    const int64_t v = v0 + s0 + i;
    uint32_t sum = (uint32_t)code_sum(tb.lut, ix.codes + (size_t)v * ix.M, ix.M) + (uint32_t)bias_key;
    if (ix.pv) sum += (uint32_t)pvq[i];
    const int32_t key = (int32_t)sum;
    if (key > bound) return;
    top.offer(HostCand{key, ix.ids[v]});
    bound = top.bound();
  };
  for (int64_t s0 = 0; s0 < len; s0 += kPlaneSegGroups * 64) {
    const int64_t nv = std::min<int64_t>(kPlaneSegGroups * 64, len - s0);
    const int ng = (int)((nv + 63) / 64);
    if (ix.pv) {
      // lut_quantize(pv, e), the scaling written as an exact product
      const float *pv = ix.pv + v0 + s0;
      for (int64_t i = 0; i < nv; ++i) {
        const float r = __builtin_rintf(pv[i] * scale);
        pvq[i] = __builtin_fabsf(r) < 2147483520.0f ? (int)r : 0;
      }
    }
    int32_t bound = top.bound();
    if (tb.filt) {
      // With nothing to compare against yet (no bound from the device and the result
      // list not full) whole groups are summed exactly until there is; then the two-
      // plane lower bounds of the remaining groups, and exact sums for the few
      // vectors whose bound does not rule them out.
      int g0 = 0;
      for (; g0 < ng && bound == kKeyInvalid; ++g0) {
        const int64_t i1 = std::min<int64_t>(nv, (int64_t)(g0 + 1) * 64);
        for (int64_t i = (int64_t)g0 * 64; i < i1; ++i) exact_offer(s0, i, bound);
      }
      if (g0 == ng) continue;
      // The columns are taken in four stretches (an eighth, a quarter, a half, all of
      // them); after each, the groups in which every vector's bound already exceeds
      // the worst kept key are dropped, and the rows of the remaining columns are
      // never read for them.
      const int64_t off = (int64_t)g0 * 64;
      int n_alive = ng - g0;
      for (int g = 0; g < n_alive; ++g) gidx[g] = g;
      const int M = ix.M;
      const int stops[4] = {std::max(4, M / 8), M / 4, M / 2, M};
      int m0 = 0;
      for (int p = 0; p < 4 && n_alive > 0; ++p) {
        const int m1 = stops[p];
        if (m1 <= m0) continue;
        if (g_plane_variant == 0)
          filter_accumulate<0>(base + s0 + off, (size_t)lpad, m0, m1, gidx, n_alive, tb.filt, acc, pf);
        else
          filter_accumulate<1>(base + s0 + off, (size_t)lpad, m0, m1, gidx, n_alive, tb.filt, acc, pf);
        n_alive = filter_survivors(acc, gidx, n_alive, nv - off,
                                   (uint32_t)tb.filt_base + (uint32_t)bias_key,
                                   ix.pv ? pvq + off : nullptr, bound, gmask);
        m0 = m1;
      }
      for (int j = 0; j < n_alive; ++j) {
        const int64_t i0 = off + (int64_t)gidx[j] * 64;
        for (uint64_t mk = gmask[j]; mk; mk &= mk - 1)
          exact_offer(s0, i0 + __builtin_ctzll(mk), bound);
      }
      continue;
    }
    if (g_plane_variant == 0)
      plane_accumulate<0>(base + s0, (size_t)lpad, ix.M, ng, tb.planes, acc);
    else
      plane_accumulate<1>(base + s0, (size_t)lpad, ix.M, ng, tb.planes, acc);
    plane_combine(acc, ng, sums);
    for (int64_t i = 0; i < nv; ++i) {
      uint32_t sum = (uint32_t)sums[i] + (uint32_t)bias_key;
      if (ix.pv) sum += (uint32_t)pvq[i];
      const int32_t key = (int32_t)sum;
      if (key > bound) continue;
      top.offer(HostCand{key, ix.ids[v0 + s0 + i]});
      bound = top.bound();
    }
  }
}

void cpu_scan_lists(const HostIndexView &ix, const int32_t *lut, int e, const float *q,
                    const int32_t *clusters, int n_clusters, int k, HostCand *out,
                    int32_t *scanned, int32_t key_cap) {
  TopK top(k, key_cap);
  const int M = ix.M;
  const bool planes_on = ix.codes_t != nullptr;
  thread_local std::vector<uint8_t> planes;
  PlaneTables tb{lut, nullptr, nullptr, 0};
  if (planes_on && n_clusters > 0) {
    if (host_filter_on()) {
      planes.resize((size_t)M * 512);
      tb.filt = planes.data();
      tb.filt_base = build_filter(lut, M, planes.data());
    } else {
      planes.resize((size_t)M * 1024);
      build_planes(lut, M, planes.data());
      tb.planes = planes.data();
    }
  }
  for (int c = 0; c < n_clusters; ++c) {
    const int cl = clusters[c];
    if (scanned) __atomic_store_n(scanned, c, __ATOMIC_RELAXED);
    if (cl < 0) continue;
    int32_t bias_key = 0;
    if (ix.by_residual)
      bias_key = lut_quantize(
          residual_bias_host(ix.metric_ip, q, ix.centroids + (size_t)cl * ix.d, ix.d), e);
    if (planes_on) {
      // The lists lie at unrelated places in memory.  The head of a list (its first
      // stretch of columns: the rest is rarely read) is requested two lists ahead, one
      // line per line of codes read meanwhile; the first two are requested at once.
      constexpr int kAhead = 2;
      auto head_of = [&](int list, const uint8_t **at, const uint8_t **end) {
        const int64_t row_bytes = (ix.list_toff[list + 1] - ix.list_toff[list]) / ix.M;
        *at = ix.codes_t + ix.list_toff[list];
        *end = *at + row_bytes * std::max(4, ix.M / 8);
      };
      if (c == 0) {
        for (int a = 0; a < kAhead && a < n_clusters; ++a) {
          if (clusters[a] < 0) continue;
          const uint8_t *at, *end;
          head_of(clusters[a], &at, &end);
          for (; at < end; at += 64) __builtin_prefetch(at, 0, 2);
        }
      }
      PrefetchCursor pf;
      if (c + kAhead < n_clusters && clusters[c + kAhead] >= 0)
        head_of(clusters[c + kAhead], &pf.at, &pf.end);
      plane_scan_list(ix, tb, e, cl, bias_key, top, &pf);
      continue;
    }
    for (int64_t v = ix.list_offsets[cl]; v < ix.list_offsets[cl + 1]; ++v) {
      const uint8_t *code = ix.codes + (size_t)v * M;
      int32_t sum = bias_key;
      if (ix.pv) sum += lut_quantize(ix.pv[v], e);
      sum += code_sum(lut, code, M);
      top.offer(HostCand{sum, ix.ids[v]});
    }
  }
  top.finish(out);
  if (scanned) __atomic_store_n(scanned, n_clusters, __ATOMIC_RELEASE);
}

void merge_topk(const HostCand *a, const HostCand *b, int k, HostCand *out) {
  int i = 0, j = 0;
  for (int r = 0; r < k; ++r) {
    const bool a_ok = i < k && a[i].key != kKeyInvalid;
    const bool b_ok = j < k && b[j].key != kKeyInvalid;
    if (a_ok && (!b_ok || cand_less(a[i], b[j]))) out[r] = a[i++];
    else if (b_ok) out[r] = b[j++];
    else out[r] = HostCand{kKeyInvalid, -1};
  }
}

}  // namespace ivf
