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

void parallel_for(int64_t n, const std::function<void(int64_t)> &fn) {
  if (n <= 0) return;
  int nt = (int)std::min<int64_t>(cpu_threads(), n);
  if (nt <= 1) {
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
    work();
    pool.wait();
    return;
  }
  std::vector<std::thread> th;  // the pool is taken: threads of our own
  th.reserve(nt - 1);
  for (int t = 1; t < nt; ++t) th.emplace_back(work);
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

int cpu_build_lut(const HostIndexView &ix, const float *q, float max_bias, int32_t *lut) {
  const int M = ix.M, dsub = ix.dsub;
  const int kind = ix.metric_ip ? kLutIP : (ix.by_residual ? kLutL2Res : kLutL2);
  const size_t n = (size_t)M * 256;
  thread_local std::vector<float> f, t;
  f.resize(n);
  if (ix.nbits == 8) {
    for (int m = 0; m < M; ++m)
      lut_column(kind, q + (size_t)m * dsub, ix.codebooks_t + (size_t)m * dsub * 256, dsub, 256,
                 &f[(size_t)m * 256]);
  } else {
    // 16 entries per sub-quantizer, then one 256-entry column per code byte
    t.resize((size_t)ix.msub * 16);
    for (int s = 0; s < ix.msub; ++s)
      lut_column(kind, q + (size_t)s * dsub, ix.codebooks_t + (size_t)s * dsub * 16, dsub, 16,
                 &t[(size_t)s * 16]);
    for (int m = 0; m < M; ++m) {
      const float *lo = &t[(size_t)(2 * m) * 16], *hi = &t[(size_t)(2 * m + 1) * 16];
      float *col = &f[(size_t)m * 256];
      for (int jh = 0; jh < 16; ++jh)
        for (int jl = 0; jl < 16; ++jl) col[jh * 16 + jl] = lut_pair_entry(lo[jl], hi[jh]);
    }
  }
  // largest |entry|: sixteen running maxima so that the loop vectorizes (a
  // NaN entry is skipped, as fmaxf skips it on the device)
  float lane_mx[16];
  for (int l = 0; l < 16; ++l) lane_mx[l] = 0.0f;
  for (size_t i = 0; i < n; i += 16)
    for (int l = 0; l < 16; ++l) {
      const float a = fabsf(f[i + l]);
      lane_mx[l] = a > lane_mx[l] ? a : lane_mx[l];
    }
  float mx = 0.0f;
  for (int l = 0; l < 16; ++l) mx = std::max(mx, lane_mx[l]);
  const int e = lut_exponent(mx, M, max_bias, ix.pv ? ix.pv_max : 0.0f);
  // lut_quantize with the scaling written as a product: |e| <= 60, so 2^e is a
  // normal float and v * 2^e rounds exactly as ldexpf(v, e) does
  const float scale = ldexpf(1.0f, e);
  for (size_t i = 0; i < n; ++i) {
    const float r = __builtin_rintf(f[i] * scale);
    lut[i] = __builtin_fabsf(r) < 2147483520.0f ? (int)r : 0;
  }
  return e;
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
  explicit TopK(int k_) : k(k_) { heap.reserve((size_t)k_); }
  // every candidate with key above this is certainly rejected
  int32_t bound() const { return (int)heap.size() < k ? 0x7fffffff : heap.front().key; }
  void offer(const HostCand &cand) {
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

static void plane_scan_list(const HostIndexView &ix, const uint8_t *planes, int e, int cl,
                            int32_t bias_key, TopK &top) {
  const int64_t v0 = ix.list_offsets[cl], len = ix.list_offsets[cl + 1] - v0;
  const int64_t lpad = (len + 63) / 64 * 64;
  const uint8_t *base = ix.codes_t + ix.list_toff[cl];
  alignas(64) uint16_t acc[kPlaneSegGroups * 256];
  alignas(64) int32_t sums[kPlaneSegGroups * 64];
  const float scale = ldexpf(1.0f, e);
  for (int64_t s0 = 0; s0 < len; s0 += kPlaneSegGroups * 64) {
    const int64_t nv = std::min<int64_t>(kPlaneSegGroups * 64, len - s0);
    const int ng = (int)((nv + 63) / 64);
    if (g_plane_variant == 0) plane_accumulate<0>(base + s0, (size_t)lpad, ix.M, ng, planes, acc);
    else plane_accumulate<1>(base + s0, (size_t)lpad, ix.M, ng, planes, acc);
    plane_combine(acc, ng, sums);
    if (ix.pv) {
      // + lut_quantize(pv, e), the scaling written as an exact product
      const float *pv = ix.pv + v0 + s0;
      for (int64_t i = 0; i < nv; ++i) {
        const float r = __builtin_rintf(pv[i] * scale);
        sums[i] += __builtin_fabsf(r) < 2147483520.0f ? (int)r : 0;
      }
    }
    int32_t bound = top.bound();
    for (int64_t i = 0; i < nv; ++i) {
      const int32_t key = (int32_t)((uint32_t)sums[i] + (uint32_t)bias_key);
      if (key > bound) continue;
      top.offer(HostCand{key, ix.ids[v0 + s0 + i]});
      bound = top.bound();
    }
  }
}

void cpu_scan_lists(const HostIndexView &ix, const int32_t *lut, int e, const float *q,
                    const int32_t *clusters, int n_clusters, int k, HostCand *out,
                    int32_t *scanned) {
  TopK top(k);
  const int M = ix.M;
  const bool planes_on = ix.codes_t != nullptr;
  thread_local std::vector<uint8_t> planes;
  if (planes_on && n_clusters > 0) {
    planes.resize((size_t)M * 1024);
    build_planes(lut, M, planes.data());
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
      plane_scan_list(ix, planes.data(), e, cl, bias_key, top);
      continue;
    }
    for (int64_t v = ix.list_offsets[cl]; v < ix.list_offsets[cl + 1]; ++v) {
      const uint8_t *code = ix.codes + (size_t)v * M;
      int32_t sum = bias_key;
      if (ix.pv) sum += lut_quantize(ix.pv[v], e);
      // eight code bytes per 64-bit load, two independent accumulators (integer sums:
      // the order does not matter); M is a multiple of 16
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
      sum += s0 + s1;
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
