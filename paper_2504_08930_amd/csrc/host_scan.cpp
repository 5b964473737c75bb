#include "host_scan.h"

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

int cpu_build_lut(const HostIndexView &ix, const float *q, float max_bias, int32_t *lut) {
  const int M = ix.M, dsub = ix.dsub;
  const int kind = ix.metric_ip ? kLutIP : (ix.by_residual ? kLutL2Res : kLutL2);
  std::vector<float> f((size_t)M * 256);
  float mx = 0.0f;
  if (ix.nbits == 8) {
    for (int m = 0; m < M; ++m) {
      for (int j = 0; j < 256; ++j) {
        float v = lut_entry(kind, q + (size_t)m * dsub,
                            ix.codebooks + ((size_t)m * 256 + j) * dsub, dsub);
        f[(size_t)m * 256 + j] = v;
        mx = std::max(mx, fabsf(v));
      }
    }
  } else {
    // 16 entries per sub-quantizer, then one 256-entry column per code byte
    std::vector<float> t((size_t)ix.msub * 16);
    for (int s = 0; s < ix.msub; ++s)
      for (int j = 0; j < 16; ++j)
        t[(size_t)s * 16 + j] = lut_entry(kind, q + (size_t)s * dsub,
                                          ix.codebooks + ((size_t)s * 16 + j) * dsub, dsub);
    for (int m = 0; m < M; ++m) {
      for (int j = 0; j < 256; ++j) {
        float v = lut_pair_entry(t[(size_t)(2 * m) * 16 + (j & 15)],
                                 t[(size_t)(2 * m + 1) * 16 + (j >> 4)]);
        f[(size_t)m * 256 + j] = v;
        mx = std::max(mx, fabsf(v));
      }
    }
  }
  const int e = lut_exponent(mx, M, max_bias, ix.pv ? ix.pv_max : 0.0f);
  for (size_t i = 0; i < f.size(); ++i) lut[i] = lut_quantize(f[i], e);
  return e;
}

static inline bool cand_less(const HostCand &a, const HostCand &b) {
  return a.key < b.key || (a.key == b.key && a.id < b.id);
}

void cpu_scan_lists(const HostIndexView &ix, const int32_t *lut, int e, const float *q,
                    const int32_t *clusters, int n_clusters, int k, HostCand *out,
                    int32_t *scanned) {
  // bounded max-heap on (key, id): the worst kept candidate sits on top
  std::vector<HostCand> heap;
  heap.reserve((size_t)k);
  const int M = ix.M;
  for (int c = 0; c < n_clusters; ++c) {
    const int cl = clusters[c];
    if (scanned) __atomic_store_n(scanned, c, __ATOMIC_RELAXED);
    if (cl < 0) continue;
    int32_t bias_key = 0;
    if (ix.by_residual)
      bias_key = lut_quantize(
          residual_bias_host(ix.metric_ip, q, ix.centroids + (size_t)cl * ix.d, ix.d), e);
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
      HostCand cand{sum, ix.ids[v]};
      if ((int)heap.size() < k) {
        heap.push_back(cand);
        std::push_heap(heap.begin(), heap.end(), cand_less);
      } else if (cand_less(cand, heap.front())) {
        std::pop_heap(heap.begin(), heap.end(), cand_less);
        heap.back() = cand;
        std::push_heap(heap.begin(), heap.end(), cand_less);
      }
    }
  }
  std::sort_heap(heap.begin(), heap.end(), cand_less);
  for (int r = 0; r < k; ++r)
    out[r] = r < (int)heap.size() ? heap[r] : HostCand{kKeyInvalid, -1};
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
