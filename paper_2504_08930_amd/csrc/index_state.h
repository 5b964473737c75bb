// State of an index and the helpers shared by the files that implement the C
// ABI (index.cpp: lifetime, layout, counters; residency.cpp: mapping tables,
// cluster copies, migration; search.cpp: the search driver; dispatcher.cpp:
// per-query completion).  Nothing here is exported from the library.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <sys/mman.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <map>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "host_scan.h"
#include "internal.h"
#include "lut_quant.h"

using namespace ivf;  // the C ABI files are the only users of this header

#define IVF_INTERNAL __attribute__((visibility("hidden")))

// A large host array that asks for 2 MB pages: the CPU scan reads lists of tens of
// kilobytes at random places of a gigabyte, and with 4 KB pages nearly every list
// starts with a run of TLB misses (which also make the hardware drop prefetches).
struct HugeBytes {
  uint8_t *p = nullptr;
  size_t n = 0;
  HugeBytes() = default;
  HugeBytes(const HugeBytes &) = delete;
  HugeBytes &operator=(const HugeBytes &) = delete;
  ~HugeBytes() { ::free(p); }
  bool alloc(size_t bytes) {
    ::free(p);
    p = nullptr;
    n = 0;
    if (bytes == 0) return true;
    constexpr size_t kAlign = (size_t)2 << 20;
    void *q = nullptr;
    if (posix_memalign(&q, kAlign, (bytes + kAlign - 1) & ~(kAlign - 1)) != 0) return false;
    (void)madvise(q, (bytes + kAlign - 1) & ~(kAlign - 1), MADV_HUGEPAGE);  // advice only
    p = static_cast<uint8_t *>(q);
    n = bytes;
    return true;
  }
  bool empty() const { return n == 0; }
  uint8_t *data() const { return p; }
};

// Sets the calling thread's error message (ivf_last_error) and returns code.
IVF_INTERNAL int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

#define HIP_TRY(expr)                                                                     \
  do {                                                                                    \
    hipError_t _e = (expr);                                                               \
    if (_e != hipSuccess)                                                                 \
      return fail(IVF_EDEVICE, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e),     \
                  __FILE__, __LINE__);                                                    \
  } while (0)

// ---------------------------------------------------------------------------
// cluster-region allocator: first fit over free tile ranges, coalescing
// ---------------------------------------------------------------------------
struct Extent {
  int64_t start, len;
};

class TileAllocator {
 public:
  void reset(int64_t cap) {
    free_.clear();
    if (cap > 0) free_[0] = cap;
  }
  // returns start or -1
  int64_t alloc(int64_t n) {
    if (n == 0) return 0;
    for (auto it = free_.begin(); it != free_.end(); ++it) {
      if (it->second >= n) {
        int64_t s = it->first, l = it->second;
        free_.erase(it);
        if (l > n) free_[s + n] = l - n;
        return s;
      }
    }
    return -1;
  }
  void release(int64_t s, int64_t n) {
    if (n == 0) return;
    auto it = free_.emplace(s, n).first;
    auto nx = std::next(it);
    if (nx != free_.end() && it->first + it->second == nx->first) {
      it->second += nx->second;
      free_.erase(nx);
    }
    if (it != free_.begin()) {
      auto pv = std::prev(it);
      if (pv->first + pv->second == it->first) {
        pv->second += it->second;
        free_.erase(it);
      }
    }
  }
  int64_t free_tiles() const {
    int64_t t = 0;
    for (auto &kv : free_) t += kv.second;
    return t;
  }

 private:
  std::map<int64_t, int64_t> free_;
};

// ---------------------------------------------------------------------------
// index object
// ---------------------------------------------------------------------------
struct Version {
  uint64_t id = 0;
  int buf = 0;                      // which mapping-table copy it reads
  int refs = 0;                     // searches running on the host side
  std::vector<hipEvent_t> events;   // searches still running on the device
  std::vector<Extent> retire;       // space to free once this and older versions drain
};

struct Migration {
  bool active = false;
  hipStream_t stream = nullptr;
  hipEvent_t begin = nullptr;   // timing pair around the copies on the side stream
  hipEvent_t done = nullptr;
  std::vector<int32_t> new_map;
  std::vector<Extent> evicted;
  int32_t *pinned_map = nullptr;
  TileDesc *pinned_descs = nullptr;
  uint64_t bytes = 0;
  int32_t d_clusters = 0;
  int64_t d_vectors = 0;
  int target_buf = 0;
};

struct TimingRec {
  hipEvent_t ev[IVF_N_STAGES + 1];
  bool valid[IVF_N_STAGES + 1];
};

struct ivf_index {
  ivf_index_desc_t desc;
  Shape sh;
  int64_t n_total = 0;
  bool has_dev = false;
  int device = 0;               // HIP device the arena lives on
  void *static_scratch = nullptr;  // that device's copy of the library's file-scope scratch array
  bool dispatch_active = false; // an asynchronous batch owns the pinned host buffers
  DevLayout L;
  hipStream_t own_stream = nullptr;
  hipEvent_t ev_routed = nullptr;  // bulk hybrid search: the cold probe lists are on the host
  std::mutex mu;

  std::vector<int32_t> h_map;      // published mapping table (host mirror)
  std::vector<int32_t> h_len;      // list lengths
  std::deque<Version> versions;    // back() is current
  TileAllocator alloc;
  int32_t resident_clusters = 0;
  int64_t resident_vectors = 0;
  Migration mig;
  uint64_t bytes_migrated = 0;
  double migrate_ms = 0.0;      // device time of completed migrations' copies
  uint64_t n_migrations = 0;
  std::vector<hipEvent_t> event_pool;
  std::vector<hipEvent_t> timing_pool;  // events with timing enabled, reused by timed batches

  std::vector<float> cb_t;  // codebooks, element-major (host table construction)
  HugeBytes codes_t;               // codes, column-major per list (byte-plane CPU scan), or empty
  std::vector<int64_t> list_toff;  // start of each list in codes_t

  // residual encoding: per-vector term of L2 (host copy; also uploaded with the tiles)
  std::vector<float> pv;        // host-only index
  float *pv_pinned = nullptr;   // index with a device: pinned, so the copy kernel can read it
  float pv_max = 0.0f;
  const float *pv_host() const { return pv_pinned ? pv_pinned : (pv.empty() ? nullptr : pv.data()); }

  // Device-visible addresses of the caller's codes and ids (and of pv) when they lie
  // in pinned host memory: cluster copies then read them from a kernel.  NULL: the
  // copies go through hipMemcpyAsync and the staging area.
  const uint8_t *zc_codes = nullptr;
  const int64_t *zc_ids = nullptr;
  const float *zc_pv = nullptr;

  // host-only counters (device-less index)
  std::vector<uint64_t> hc_hits;
  uint64_t hc_probes = 0, hc_queries = 0;

  // pinned host buffers
  int32_t *h_ncold = nullptr, *h_cold = nullptr, *h_reskey = nullptr, *h_lutmax = nullptr;
  int64_t *h_resid = nullptr, *h_outids = nullptr;
  float *h_outd = nullptr, *h_queries = nullptr, *h_qbmax = nullptr;
  int32_t *h_probe = nullptr;
  unsigned long long *h_stats = nullptr;

  // workspace slots: a slot belongs to the stream that used it last; a call on
  // a new stream takes the least recently used slot after that slot's stream
  // has drained
  hipStream_t slot_stream[kWsSlots] = {nullptr, nullptr};
  bool slot_used[kWsSlots] = {false, false};
  uint64_t slot_tick[kWsSlots] = {0, 0};
  uint64_t tick = 0;

  int32_t tune_slices = 0;
  int32_t timing = 0;
  std::vector<TimingRec> trecs;
  double t_ms[IVF_N_STAGES] = {0};
  uint64_t t_n[IVF_N_STAGES] = {0};
};


// Pinned host memory is always allocated, never registered.
template <typename T>
static inline hipError_t pinned_alloc(T **p, size_t count) {
  return hipHostMalloc(reinterpret_cast<void **>(p), std::max<size_t>(count, 1) * sizeof(T),
                       hipHostMallocDefault);
}

// ---- search driver pieces shared with the dispatcher (search.cpp) ----
struct SearchArgs {
  const float *q_dev = nullptr;    // device queries (may be NULL if q_host given)
  const float *q_host = nullptr;   // host queries (may be NULL if q_dev given)
  const int32_t *probe_host = nullptr;  // forced probe list (host) or NULL
  int64_t nq = 0;
  int nprobe = 0;
  int k = 0;
  int64_t *out_ids = nullptr;
  float *out_dists = nullptr;
  bool out_device = false;
  hipStream_t st = nullptr;
};

// One batch's hold on a workspace slot and on a mapping-table version.
struct BatchCtx {
  int slot = 0;
  int buf = 0;
  bool all_resident = false, any_resident = false;
  int timing = 0;  // 0: no events; 1: around every stage; 2: around the scan only
  int list_tiles = 1;  // average tiles (64 vectors) of a resident list, at least 1
  uint64_t ver_id = 0;
};

// index.cpp
IVF_INTERNAL HostIndexView host_view(const ivf_index *ix);
// the router's counters, as ivf_hit_stats returns them (caller holds ix->mu)
IVF_INTERNAL int read_counters_locked(ivf_index *ix, uint64_t *per_cluster_hits,
                                      double *mean_hit_rate, double *min_hit_rate,
                                      uint64_t *n_queries, int reset);
IVF_INTERNAL int reset_counters_locked(ivf_index *ix);
// cluster ids from the most to the least accessed, equal counts by id
IVF_INTERNAL void rank_clusters(const std::vector<uint64_t> &hits, std::vector<int32_t> &order);
// residency.cpp (callers hold ix->mu)
IVF_INTERNAL hipEvent_t get_event(ivf_index *ix);
IVF_INTERNAL void reclaim(ivf_index *ix);
IVF_INTERNAL int publish_if_done_locked(ivf_index *ix, bool wait);
// search.cpp
IVF_INTERNAL int begin_batch(ivf_index *ix, hipStream_t st, BatchCtx *c);
IVF_INTERNAL void end_batch(ivf_index *ix, const BatchCtx &c, hipStream_t st, bool async_tail);
IVF_INTERNAL int enqueue_gpu(ivf_index *ix, const SearchArgs &a, const BatchCtx &c,
                             bool final_on_gpu, hipEvent_t ev_route);
IVF_INTERNAL bool finish_query(const ivf_index *ix, const HostIndexView &view,
                               bool any_resident, int64_t q, int k, const HostCand *cpu,
                               int cpu_e, int64_t *ids, float *dists);
IVF_INTERNAL int32_t device_key_cap(const ivf_index *ix, const HostIndexView &view, int64_t q,
                                    int k, int e);
IVF_INTERNAL int check_search_args(const ivf_index *ix, const void *queries, int64_t nq,
                                   int32_t nprobe, int32_t k, const void *out_ids,
                                   const void *out_dists);
IVF_INTERNAL int check_probe_list(const ivf_index *ix, const int32_t *probe, int64_t nq,
                                  int nprobe);
