// C ABI of the library: index lifetime, residency (mapping table, cluster
// region allocator, load / migrate), the search driver that strings the
// kernels together and runs the CPU scan of cold probes, router counters.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

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

using namespace ivf;

// ---------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------
static thread_local std::string g_err;

static int fail(int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define HIP_TRY(expr)                                                                     \
  do {                                                                                    \
    hipError_t _e = (expr);                                                               \
    if (_e != hipSuccess)                                                                 \
      return fail(IVF_EDEVICE, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e),     \
                  __FILE__, __LINE__);                                                    \
  } while (0)

extern "C" const char *ivf_last_error(void) { return g_err.c_str(); }

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
  bool dispatch_active = false; // an asynchronous batch owns the pinned host buffers
  DevLayout L;
  hipStream_t own_stream = nullptr;
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

  // residual encoding: per-vector term of L2 (host copy; also uploaded with the tiles)
  std::vector<float> pv;
  float pv_max = 0.0f;

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

static HostIndexView host_view(const ivf_index *ix) {
  HostIndexView v;
  v.d = ix->sh.d;
  v.nlist = ix->sh.nlist;
  v.M = ix->sh.M;
  v.nbits = ix->sh.nbits;
  v.msub = ix->sh.msub;
  v.dsub = ix->sh.dsub;
  v.metric_ip = ix->sh.metric_ip;
  v.by_residual = ix->desc.by_residual;
  v.centroids = ix->desc.centroids;
  v.pv = ix->pv.empty() ? nullptr : ix->pv.data();
  v.pv_max = ix->pv_max;
  v.codebooks = ix->desc.codebooks;
  v.list_offsets = ix->desc.list_offsets;
  v.codes = ix->desc.codes;
  v.ids = ix->desc.ids;
  return v;
}

// Bytes of one stored code = columns of the scan's lookup table.
static int code_bytes(const ivf_index_desc_t &d) { return d.M * d.nbits / 8; }

static int validate_desc(const ivf_index_desc_t *d) {
  if (!d) return fail(IVF_EINVAL, "desc is NULL");
  if (d->nbits != 8 && d->nbits != 4)
    return fail(IVF_EINVAL, "nbits must be 8 or 4 (got %d)", d->nbits);
  if (d->metric != IVF_METRIC_L2 && d->metric != IVF_METRIC_IP)
    return fail(IVF_EINVAL, "unknown metric %d", d->metric);
  if (d->nlist < 1 || d->d < 1) return fail(IVF_EINVAL, "nlist and d must be positive");
  if (d->M < 1 || d->M > 1024) return fail(IVF_EINVAL, "M out of range (got %d)", d->M);
  const int cb = code_bytes(*d);
  if (cb < 16 || cb > 128 || cb % 16 != 0 || cb * 8 != d->M * d->nbits)
    return fail(IVF_EINVAL, "M * nbits / 8 must be a multiple of 16 in [16, 128] (M = %d, nbits = %d)",
                d->M, d->nbits);
  if (d->d % d->M != 0) return fail(IVF_EINVAL, "d (%d) must be a multiple of M (%d)", d->d, d->M);
  if (d->by_residual != 0 && d->by_residual != 1)
    return fail(IVF_EINVAL, "by_residual must be 0 or 1");
  if (d->max_nq < 1) return fail(IVF_EINVAL, "max_nq must be >= 1");
  if (d->max_nprobe < 1 || d->max_nprobe > kMaxNprobe)
    return fail(IVF_EINVAL, "max_nprobe must be in [1, %d]", kMaxNprobe);
  if (d->max_k < 1 || d->max_k > kMaxK) return fail(IVF_EINVAL, "max_k must be in [1, %d]", kMaxK);
  return IVF_OK;
}

// Carve the arena.  base may be NULL (size query only).  Returns total bytes.
static size_t plan_layout(const ivf_index_desc_t &d, int64_t resident_vectors, size_t staging,
                          unsigned char *base, DevLayout *L) {
  size_t off = 0;
  auto take = [&](size_t bytes) -> unsigned char * {
    off = (off + 255) & ~(size_t)255;
    unsigned char *p = base ? base + off : nullptr;
    off += bytes;
    return p;
  };
  const size_t nl = (size_t)d.nlist, D = (size_t)d.d, M = (size_t)code_bytes(d);
  const size_t nq = (size_t)d.max_nq, np = (size_t)d.max_nprobe, k = (size_t)d.max_k;
  if (staging == 0) staging = (size_t)64 << 20;
  DevLayout t;
  t.centroids = (float *)take(nl * D * 4);
  t.cent_norm = (float *)take(nl * 4);
  t.cent_parts = take(nl * D * 4 + kSplitPadBytes);
  t.cent_exp = (int32_t *)take(nl * 4);
  t.cbT = (float *)take(256 * D * 4);
  t.clus_len = (int32_t *)take(nl * 4);
  for (int i = 0; i < 3; ++i) t.clus_tile[i] = (int32_t *)take(nl * 4);
  t.hits = (unsigned long long *)take(nl * 8);
  t.qstats = (unsigned long long *)take(QS_COUNT * 8);
  for (int sl = 0; sl < kWsSlots; ++sl) {
    BatchWs &w = t.ws[sl];
    w.q_parts = take(nq * D * 4 + kSplitPadBytes);
    w.q_exp = (int32_t *)take(nq * 4);
    w.queries = (float *)take(nq * D * 4);
    w.scores = (float *)take(nq * nl * 4);
    w.probe = (int32_t *)take(nq * np * 4);
    w.g_base = (int32_t *)take(nq * np * 4);
    w.g_len = (int32_t *)take(nq * np * 4);
    w.g_prefix = (int32_t *)take(nq * (np + 1) * 4);
    w.g_n = (int32_t *)take(nq * 4);
    w.cold = (int32_t *)take(nq * np * 4);
    w.n_cold = (int32_t *)take(nq * 4);
    w.lut = (float *)take(nq * 256 * M * 4);
    w.lutpart = (uint32_t *)take(nq * kLutMaxParts * 4);
    w.lutmax = (uint32_t *)take(nq * 4);
    w.q_vecs = (int32_t *)take(nq * 4);
    w.order = (int32_t *)take(nq * 4);
    w.bias = (float *)take(nq * np * 4);
    w.g_bias = (float *)take(nq * np * 4);
    w.qbmax = (float *)take(nq * 4);
    w.part_key = (int32_t *)take(nq * kMaxSlices * k * 4);
    w.part_id = (int64_t *)take(nq * kMaxSlices * k * 8);
    w.res_key = (int32_t *)take(nq * k * 4);
    w.res_id = (int64_t *)take(nq * k * 8);
    w.out_ids = (int64_t *)take(nq * k * 8);
    w.out_dists = (float *)take(nq * k * 4);
  }
  t.staging = (unsigned char *)take(staging);
  t.staging_bytes = staging;
  int64_t cap_tiles = (resident_vectors + kTileVecs - 1) / kTileVecs;
  if (cap_tiles < 0) cap_tiles = 0;
  t.cap_tiles = cap_tiles;
  t.tile_codes = (uint8_t *)take((size_t)cap_tiles * kTileVecs * M);
  t.tile_ids = (int64_t *)take((size_t)cap_tiles * kTileVecs * 8);
  t.tile_pv = nullptr;
  if (d.by_residual && d.metric == IVF_METRIC_L2)
    t.tile_pv = (float *)take((size_t)cap_tiles * kTileVecs * 4);
  off = (off + 255) & ~(size_t)255;
  if (L) *L = t;
  return off;
}

extern "C" size_t ivf_index_arena_bytes(const ivf_index_desc_t *desc, int64_t resident_vectors,
                                        size_t staging_bytes) {
  if (validate_desc(desc) != IVF_OK || resident_vectors < 0) return 0;
  return plan_layout(*desc, resident_vectors, staging_bytes, nullptr, nullptr);
}

template <typename T>
static hipError_t pinned_alloc(T **p, size_t count) {
  return hipHostMalloc(reinterpret_cast<void **>(p), std::max<size_t>(count, 1) * sizeof(T),
                       hipHostMallocDefault);
}

static void free_host_buffers(ivf_index *ix) {
  void *ptrs[] = {ix->h_ncold, ix->h_cold,   ix->h_reskey,  ix->h_lutmax, ix->h_resid,
                  ix->h_outids, ix->h_outd,  ix->h_queries, ix->h_probe,  ix->h_stats,
                  ix->h_qbmax};
  for (void *p : ptrs)
    if (p) (void)hipHostFree(p);
}

extern "C" void ivf_index_destroy(ivf_index_t *ix) {
  if (!ix) return;
  if (ix->has_dev) {
    (void)hipDeviceSynchronize();
    if (ix->mig.active) {
      if (ix->mig.begin) (void)hipEventDestroy(ix->mig.begin);
      if (ix->mig.done) (void)hipEventDestroy(ix->mig.done);
      if (ix->mig.pinned_map) (void)hipHostFree(ix->mig.pinned_map);
      if (ix->mig.pinned_descs) (void)hipHostFree(ix->mig.pinned_descs);
    }
    for (auto &v : ix->versions)
      for (auto e : v.events) (void)hipEventDestroy(e);
    for (auto e : ix->event_pool) (void)hipEventDestroy(e);
    for (auto &r : ix->trecs)
      for (int i = 0; i <= IVF_N_STAGES; ++i)
        if (r.valid[i]) (void)hipEventDestroy(r.ev[i]);
    free_host_buffers(ix);
    if (ix->own_stream) (void)hipStreamDestroy(ix->own_stream);
  }
  delete ix;
}

extern "C" int ivf_index_create(const ivf_index_desc_t *desc, void *dev_arena, size_t arena_bytes,
                                size_t staging_bytes, ivf_index_t **out) {
  if (!out) return fail(IVF_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = validate_desc(desc);
  if (rc != IVF_OK) return rc;
  if (!desc->centroids || !desc->codebooks || !desc->list_offsets)
    return fail(IVF_EINVAL, "centroids, codebooks and list_offsets are required");
  const int64_t n_total = desc->list_offsets[desc->nlist];
  if (desc->list_offsets[0] != 0) return fail(IVF_EINVAL, "list_offsets[0] must be 0");
  for (int c = 0; c < desc->nlist; ++c) {
    int64_t len = desc->list_offsets[c + 1] - desc->list_offsets[c];
    if (len < 0 || len > 0x7fffffff - 64)
      return fail(IVF_EINVAL, "list %d has invalid length %lld", c, (long long)len);
  }
  if (n_total > 0 && (!desc->codes || !desc->ids))
    return fail(IVF_EINVAL, "codes and ids are required");

  ivf_index *ix = new ivf_index();
  ix->desc = *desc;
  ix->sh = Shape{desc->d, desc->nlist, code_bytes(*desc), desc->d / desc->M,
                 desc->metric == IVF_METRIC_IP, desc->by_residual, 0.0f, desc->nbits, desc->M};
  ix->n_total = n_total;
  ix->h_map.assign(desc->nlist, -1);
  ix->h_len.resize(desc->nlist);
  for (int c = 0; c < desc->nlist; ++c)
    ix->h_len[c] = (int32_t)(desc->list_offsets[c + 1] - desc->list_offsets[c]);
  ix->hc_hits.assign(desc->nlist, 0);
  ix->versions.emplace_back();
  if (desc->by_residual && desc->metric == IVF_METRIC_L2 && n_total > 0) {
    ix->pv.resize((size_t)n_total);
    HostIndexView v = host_view(ix);
    v.pv = nullptr;
    ix->pv_max = cpu_residual_pv(v, n_total, ix->pv.data());
    ix->sh.pv_max = ix->pv_max;
  }

  if (!dev_arena) {
    *out = ix;
    return IVF_OK;
  }
  if (((uintptr_t)dev_arena & 255) != 0) {
    delete ix;
    return fail(IVF_EINVAL, "dev_arena must be 256-byte aligned");
  }
  if (!scan_supports(code_bytes(*desc), desc->max_k)) {
    delete ix;
    return fail(IVF_EINVAL, "no scan kernel for %d code bytes (supported: 16, 32, 48, 64, 96, 128)",
                code_bytes(*desc));
  }
  // how many resident vectors does the arena leave room for?
  const size_t fixed = plan_layout(*desc, 0, staging_bytes, nullptr, nullptr);
  if (arena_bytes < fixed) {
    delete ix;
    return fail(IVF_ENOMEM, "arena of %zu bytes is smaller than the %zu bytes of fixed state",
                arena_bytes, fixed);
  }
  const size_t per_tile =
      (size_t)kTileVecs *
      (code_bytes(*desc) + 8 + ((desc->by_residual && desc->metric == IVF_METRIC_L2) ? 4 : 0));
  int64_t tiles = (int64_t)((arena_bytes - fixed) / per_tile);
  while (tiles > 0 &&
         plan_layout(*desc, tiles * kTileVecs, staging_bytes, nullptr, nullptr) > arena_bytes)
    --tiles;
  plan_layout(*desc, tiles * kTileVecs, staging_bytes, (unsigned char *)dev_arena, &ix->L);
  ix->alloc.reset(ix->L.cap_tiles);
  ix->has_dev = true;
  (void)hipGetDevice(&ix->device);

  auto bail = [&](hipError_t e, const char *what) {
    std::string msg = std::string(what) + ": " + hipGetErrorString(e);
    ivf_index_destroy(ix);
    return fail(IVF_EDEVICE, "%s", msg.c_str());
  };
  hipError_t e;
  if ((e = hipStreamCreateWithFlags(&ix->own_stream, hipStreamNonBlocking)) != hipSuccess)
    return bail(e, "hipStreamCreateWithFlags");
  const size_t nq = desc->max_nq, np = desc->max_nprobe, k = desc->max_k;
  if ((e = pinned_alloc(&ix->h_ncold, nq)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_cold, nq * np)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_reskey, nq * k)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_resid, nq * k)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_lutmax, nq)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_qbmax, nq)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_outids, nq * k)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_outd, nq * k)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_queries, nq * (size_t)desc->d)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_probe, nq * np)) != hipSuccess ||
      (e = pinned_alloc(&ix->h_stats, (size_t)QS_COUNT)) != hipSuccess)
    return bail(e, "hipHostMalloc");

  hipStream_t st = ix->own_stream;
  const DevLayout &L = ix->L;
  const size_t D = desc->d, M = desc->M, dsub = D / M, ksub = (size_t)1 << desc->nbits;
  // transposed codebooks [ksub][M][dsub]
  std::vector<float> cbT(ksub * D);
  for (size_t m = 0; m < M; ++m)
    for (size_t j = 0; j < ksub; ++j)
      memcpy(&cbT[(j * M + m) * dsub], desc->codebooks + (m * ksub + j) * dsub, dsub * 4);
  if ((e = hipMemcpyAsync(L.centroids, desc->centroids, (size_t)desc->nlist * D * 4,
                          hipMemcpyHostToDevice, st)) != hipSuccess ||
      (e = hipMemcpyAsync(L.cbT, cbT.data(), cbT.size() * 4, hipMemcpyHostToDevice, st)) !=
          hipSuccess ||
      (e = hipMemcpyAsync(L.clus_len, ix->h_len.data(), (size_t)desc->nlist * 4,
                          hipMemcpyHostToDevice, st)) != hipSuccess)
    return bail(e, "hipMemcpyAsync");
  for (int i = 0; i < 3; ++i)
    if ((e = launch_fill_u32((uint32_t *)L.clus_tile[i], desc->nlist, 0xffffffffu, st)) !=
        hipSuccess)
      return bail(e, "fill");
  if ((e = launch_fill_u32((uint32_t *)L.hits, (size_t)desc->nlist * 2, 0u, st)) != hipSuccess ||
      (e = launch_fill_u32((uint32_t *)L.qstats, QS_COUNT * 2, 0u, st)) != hipSuccess ||
      (e = launch_fill_u32((uint32_t *)&L.qstats[QS_MIN_RATE_BITS], 1, 0x3f800000u, st)) !=
          hipSuccess ||
      (e = launch_cent_norms(L.centroids, desc->nlist, desc->d, L.cent_norm, st)) != hipSuccess ||
      (e = launch_split_f16(L.centroids, (size_t)desc->nlist, desc->d, L.cent_parts, L.cent_exp,
                            st)) !=
          hipSuccess)
    return bail(e, "init kernels");
  if ((e = hipStreamSynchronize(st)) != hipSuccess) return bail(e, "hipStreamSynchronize");
  *out = ix;
  return IVF_OK;
}

// ---------------------------------------------------------------------------
// version bookkeeping (caller holds ix->mu)
// ---------------------------------------------------------------------------
static hipEvent_t get_event(ivf_index *ix) {
  if (!ix->event_pool.empty()) {
    hipEvent_t e = ix->event_pool.back();
    ix->event_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
  return e;
}

static bool version_drained(ivf_index *ix, Version &v) {
  if (v.refs > 0) return false;
  while (!v.events.empty()) {
    hipError_t q = hipEventQuery(v.events.back());
    if (q == hipErrorNotReady) return false;
    ix->event_pool.push_back(v.events.back());
    v.events.pop_back();
  }
  return true;
}

// Free the space of clusters evicted by old versions once nothing can read it.
static void reclaim(ivf_index *ix) {
  while (ix->versions.size() > 1 && version_drained(ix, ix->versions.front())) {
    for (auto &x : ix->versions.front().retire) ix->alloc.release(x.start, x.len);
    ix->versions.pop_front();
  }
}

// ---------------------------------------------------------------------------
// host -> device cluster copies through the staging area
// ---------------------------------------------------------------------------
static int64_t tiles_of(int32_t len) { return ((int64_t)len + kTileVecs - 1) / kTileVecs; }

// Enqueue on `st` the copies that fill tiles [bases[i], ...) with cluster
// clusters[i].  descs: pinned host array with room for the sum of tile counts.
static int enqueue_cluster_copies(ivf_index *ix, const std::vector<int32_t> &clusters,
                                  const std::vector<int64_t> &bases, TileDesc *descs,
                                  hipStream_t st) {
  const DevLayout &L = ix->L;
  const size_t M = ix->sh.M;
  const bool with_pv = L.tile_pv != nullptr;
  const size_t per_tile = kTileVecs * (M + 8 + (with_pv ? 4 : 0)) + sizeof(TileDesc);
  if (L.staging_bytes < per_tile + 2048) return fail(IVF_ENOMEM, "staging area too small");
  const int64_t tile_cap = (int64_t)((L.staging_bytes - 1024) / per_tile);
  unsigned char *st_codes = L.staging;
  unsigned char *st_ids = L.staging + (((size_t)tile_cap * kTileVecs * M + 255) & ~(size_t)255);
  unsigned char *st_pv = st_ids + (((size_t)tile_cap * kTileVecs * 8 + 255) & ~(size_t)255);
  unsigned char *st_desc =
      st_pv + (with_pv ? (((size_t)tile_cap * kTileVecs * 4 + 255) & ~(size_t)255) : 0);

  size_t ci = 0;          // current cluster
  int64_t tile_in = 0;    // tiles of it already copied
  size_t desc_used = 0;
  while (ci < clusters.size()) {
    // ---- build one chunk ----
    int64_t chunk_tiles = 0;
    int64_t chunk_vecs = 0;
    TileDesc *cd = descs + desc_used;
    int64_t run_src = -1, run_len = 0, run_dst = 0;  // pending contiguous host range (vectors)
    auto flush_run = [&]() -> int {
      if (run_len == 0) return IVF_OK;
      HIP_TRY(hipMemcpyAsync(st_codes + (size_t)run_dst * M, ix->desc.codes + (size_t)run_src * M,
                             (size_t)run_len * M, hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(st_ids + (size_t)run_dst * 8, ix->desc.ids + run_src,
                             (size_t)run_len * 8, hipMemcpyHostToDevice, st));
      if (with_pv)
        HIP_TRY(hipMemcpyAsync(st_pv + (size_t)run_dst * 4, ix->pv.data() + run_src,
                               (size_t)run_len * 4, hipMemcpyHostToDevice, st));
      run_len = 0;
      return IVF_OK;
    };
    while (ci < clusters.size() && chunk_tiles < tile_cap) {
      const int32_t c = clusters[ci];
      const int32_t len = ix->h_len[c];
      const int64_t nt = tiles_of(len);
      if (tile_in >= nt) {  // done (or empty cluster)
        ++ci;
        tile_in = 0;
        continue;
      }
      const int64_t take = std::min(nt - tile_in, tile_cap - chunk_tiles);
      const int64_t v0 = tile_in * kTileVecs;
      const int64_t v1 = std::min<int64_t>(len, (tile_in + take) * kTileVecs);
      const int64_t src = ix->desc.list_offsets[c] + v0;
      if (run_len > 0 && run_src + run_len != src) {
        int rc = flush_run();
        if (rc != IVF_OK) return rc;
      }
      if (run_len == 0) {
        run_src = src;
        run_dst = chunk_vecs;
      }
      run_len += v1 - v0;
      for (int64_t t = 0; t < take; ++t) {
        TileDesc &d = cd[chunk_tiles + t];
        d.dst_tile = (int32_t)(bases[ci] + tile_in + t);
        d.src_vec = (int32_t)(chunk_vecs + t * kTileVecs);
        d.n_valid = (int32_t)std::min<int64_t>(kTileVecs, (v1 - v0) - t * kTileVecs);
        d.pad = 0;
      }
      chunk_tiles += take;
      chunk_vecs += v1 - v0;
      tile_in += take;
    }
    int rc = flush_run();
    if (rc != IVF_OK) return rc;
    if (chunk_tiles > 0) {
      HIP_TRY(hipMemcpyAsync(st_desc, cd, (size_t)chunk_tiles * sizeof(TileDesc),
                             hipMemcpyHostToDevice, st));
      HIP_TRY(launch_interleave(st_codes, (const int64_t *)st_ids,
                                with_pv ? (const float *)st_pv : nullptr,
                                (const TileDesc *)st_desc, (int)chunk_tiles, (int)M, L.tile_codes,
                                L.tile_ids, L.tile_pv, st));
      desc_used += (size_t)chunk_tiles;
    }
  }
  return IVF_OK;
}

static int check_cluster_list(const ivf_index *ix, const int32_t *ids, int32_t n, const char *what,
                              std::vector<char> &seen) {
  if (n < 0 || (n > 0 && !ids)) return fail(IVF_EINVAL, "%s: bad list", what);
  for (int32_t i = 0; i < n; ++i) {
    if (ids[i] < 0 || ids[i] >= ix->sh.nlist)
      return fail(IVF_EINVAL, "%s: cluster id %d out of range", what, ids[i]);
    if (seen[ids[i]]) return fail(IVF_EINVAL, "%s: cluster id %d listed twice", what, ids[i]);
    seen[ids[i]] = 1;
  }
  return IVF_OK;
}

extern "C" int ivf_index_load_partition(ivf_index_t *ix, const int32_t *cluster_ids, int32_t n,
                                        void *stream) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (!ix->has_dev) return fail(IVF_EDEVICE, "host-only index: no device partition");
  std::lock_guard<std::mutex> lk(ix->mu);
  if (ix->mig.active) return fail(IVF_EBUSY, "a migration is in flight");
  std::vector<char> seen(ix->sh.nlist, 0);
  int rc = check_cluster_list(ix, cluster_ids, n, "load_partition", seen);
  if (rc != IVF_OK) return rc;
  hipStream_t st = (hipStream_t)stream;

  std::vector<int32_t> clusters(cluster_ids, cluster_ids + n);
  std::sort(clusters.begin(), clusters.end());
  int64_t need = 0;
  for (int32_t c : clusters) need += tiles_of(ix->h_len[c]);
  if (need > ix->L.cap_tiles)
    return fail(IVF_ENOMEM, "partition needs %lld tiles, cluster region holds %lld",
                (long long)need, (long long)ix->L.cap_tiles);
  // full refresh: nothing may still be reading the old placement
  HIP_TRY(hipDeviceSynchronize());
  reclaim(ix);
  if (ix->versions.size() > 1 || ix->versions.back().refs > 0)
    return fail(IVF_ESTATE, "load_partition while searches are running");

  std::vector<int32_t> new_map(ix->sh.nlist, -1);
  std::vector<int64_t> bases(clusters.size());
  int64_t next = 0, vecs = 0;
  for (size_t i = 0; i < clusters.size(); ++i) {
    bases[i] = next;
    new_map[clusters[i]] = (int32_t)next;
    next += tiles_of(ix->h_len[clusters[i]]);
    vecs += ix->h_len[clusters[i]];
  }
  TileDesc *descs = nullptr;
  HIP_TRY(pinned_alloc(&descs, (size_t)need));
  rc = enqueue_cluster_copies(ix, clusters, bases, descs, st);
  if (rc == IVF_OK) {
    Version &cur = ix->versions.back();
    hipError_t e = hipMemcpyAsync(ix->L.clus_tile[cur.buf], new_map.data(),
                                  (size_t)ix->sh.nlist * 4, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) rc = fail(IVF_EDEVICE, "load_partition copy: %s", hipGetErrorString(e));
  } else {
    (void)hipStreamSynchronize(st);
  }
  (void)hipHostFree(descs);
  if (rc != IVF_OK) {
    // the old mapping table is still published but the region was overwritten:
    // drop residency entirely so no stale tile can be read
    std::vector<int32_t> none(ix->sh.nlist, -1);
    (void)hipMemcpy(ix->L.clus_tile[ix->versions.back().buf], none.data(),
                    (size_t)ix->sh.nlist * 4, hipMemcpyHostToDevice);
    ix->h_map = none;
    ix->alloc.reset(ix->L.cap_tiles);
    ix->resident_clusters = 0;
    ix->resident_vectors = 0;
    return rc;
  }
  ix->h_map.swap(new_map);
  ix->alloc.reset(ix->L.cap_tiles);
  if (next > 0) {
    int64_t got = ix->alloc.alloc(next);
    (void)got;  // first fit on an empty region returns 0
  }
  ix->resident_clusters = (int32_t)clusters.size();
  ix->resident_vectors = vecs;
  return IVF_OK;
}

extern "C" int ivf_resident_info(ivf_index_t *ix, int32_t *n_clusters, int64_t *n_vectors) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  std::lock_guard<std::mutex> lk(ix->mu);
  if (n_clusters) *n_clusters = ix->resident_clusters;
  if (n_vectors) *n_vectors = ix->resident_vectors;
  return IVF_OK;
}

// ---------------------------------------------------------------------------
// migration (caller holds ix->mu for the *_locked helpers)
// ---------------------------------------------------------------------------
static int publish_if_done_locked(ivf_index *ix, bool wait) {
  Migration &m = ix->mig;
  if (!m.active) return 0;
  if (wait) {
    HIP_TRY(hipEventSynchronize(m.done));
  } else {
    hipError_t q = hipEventQuery(m.done);
    if (q == hipErrorNotReady) return 1;
    if (q != hipSuccess) return fail(IVF_EDEVICE, "migration event: %s", hipGetErrorString(q));
  }
  // copies are complete: flip the mapping table
  Version &old = ix->versions.back();
  old.retire = m.evicted;
  Version nv;
  nv.id = old.id + 1;
  nv.buf = m.target_buf;
  ix->versions.push_back(std::move(nv));
  ix->h_map.swap(m.new_map);
  ix->resident_clusters += m.d_clusters;
  ix->resident_vectors += m.d_vectors;
  ix->bytes_migrated += m.bytes;
  {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, m.begin, m.done) == hipSuccess) ix->migrate_ms += ms;
    ix->n_migrations += 1;
  }
  (void)hipEventDestroy(m.begin);
  (void)hipEventDestroy(m.done);
  (void)hipHostFree(m.pinned_map);
  if (m.pinned_descs) (void)hipHostFree(m.pinned_descs);
  m = Migration();
  reclaim(ix);
  return 0;
}

extern "C" int ivf_migrate_clusters(ivf_index_t *ix, const int32_t *evict, int32_t n_evict,
                                    const int32_t *admit, int32_t n_admit, void *side_stream) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (!ix->has_dev) return fail(IVF_EDEVICE, "host-only index: nothing to migrate");
  std::lock_guard<std::mutex> lk(ix->mu);
  int rc = publish_if_done_locked(ix, false);
  if (rc < 0) return rc;
  if (ix->mig.active) return fail(IVF_EBUSY, "a migration is already in flight");
  std::vector<char> seen(ix->sh.nlist, 0);
  if ((rc = check_cluster_list(ix, evict, n_evict, "evict", seen)) != IVF_OK) return rc;
  if ((rc = check_cluster_list(ix, admit, n_admit, "admit", seen)) != IVF_OK) return rc;
  for (int32_t i = 0; i < n_evict; ++i)
    if (ix->h_map[evict[i]] < 0)
      return fail(IVF_EINVAL, "evict: cluster %d is not resident", evict[i]);
  for (int32_t i = 0; i < n_admit; ++i)
    if (ix->h_map[admit[i]] >= 0)
      return fail(IVF_EINVAL, "admit: cluster %d is already resident", admit[i]);
  hipStream_t st = (hipStream_t)side_stream;

  reclaim(ix);
  const int target = (ix->versions.back().buf + 1) % 3;
  for (auto &v : ix->versions)
    if (v.buf == target)
      return fail(IVF_EBUSY, "searches on an old mapping table have not drained yet");

  // place admitted clusters in free space only
  std::vector<int32_t> clusters(admit, admit + n_admit);
  std::sort(clusters.begin(), clusters.end());
  std::vector<int64_t> bases(clusters.size());
  size_t placed = 0;
  int64_t need_tiles = 0;
  bool ok = true;
  for (; placed < clusters.size(); ++placed) {
    const int64_t nt = tiles_of(ix->h_len[clusters[placed]]);
    const int64_t s = ix->alloc.alloc(nt);
    if (s < 0) {
      ok = false;
      break;
    }
    bases[placed] = s;
    need_tiles += nt;
  }
  auto undo = [&]() {
    for (size_t i = 0; i < placed; ++i)
      ix->alloc.release(bases[i], tiles_of(ix->h_len[clusters[i]]));
  };
  if (!ok) {
    undo();
    return fail(IVF_ENOMEM, "cluster region cannot hold the admitted clusters (%lld tiles free)",
                (long long)ix->alloc.free_tiles());
  }

  Migration m;
  m.stream = st;
  m.target_buf = target;
  m.new_map = ix->h_map;
  for (int32_t i = 0; i < n_evict; ++i) {
    const int32_t c = evict[i];
    m.evicted.push_back(Extent{ix->h_map[c], tiles_of(ix->h_len[c])});
    m.new_map[c] = -1;
    m.d_clusters -= 1;
    m.d_vectors -= ix->h_len[c];
  }
  for (size_t i = 0; i < clusters.size(); ++i) {
    m.new_map[clusters[i]] = (int32_t)bases[i];
    m.d_clusters += 1;
    m.d_vectors += ix->h_len[clusters[i]];
    m.bytes += (uint64_t)ix->h_len[clusters[i]] *
               (uint64_t)(ix->sh.M + 8 + (ix->L.tile_pv ? 4 : 0));
  }
  hipError_t e = pinned_alloc(&m.pinned_map, (size_t)ix->sh.nlist);
  if (e == hipSuccess && need_tiles > 0) e = pinned_alloc(&m.pinned_descs, (size_t)need_tiles);
  if (e == hipSuccess) e = hipEventCreate(&m.begin);
  if (e == hipSuccess) e = hipEventCreate(&m.done);
  if (e != hipSuccess) {
    undo();
    if (m.begin) (void)hipEventDestroy(m.begin);
    if (m.done) (void)hipEventDestroy(m.done);
    if (m.pinned_map) (void)hipHostFree(m.pinned_map);
    if (m.pinned_descs) (void)hipHostFree(m.pinned_descs);
    return fail(IVF_EDEVICE, "migration setup: %s", hipGetErrorString(e));
  }
  memcpy(m.pinned_map, m.new_map.data(), (size_t)ix->sh.nlist * 4);
  e = hipEventRecord(m.begin, st);
  rc = e == hipSuccess ? enqueue_cluster_copies(ix, clusters, bases, m.pinned_descs, st)
                       : fail(IVF_EDEVICE, "migration enqueue: %s", hipGetErrorString(e));
  if (rc == IVF_OK) {
    e = hipMemcpyAsync(ix->L.clus_tile[target], m.pinned_map, (size_t)ix->sh.nlist * 4,
                       hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipEventRecord(m.done, st);
    if (e != hipSuccess) rc = fail(IVF_EDEVICE, "migration enqueue: %s", hipGetErrorString(e));
  }
  if (rc != IVF_OK) {
    // admitted clusters stay cold; whatever was enqueued only touches free tiles
    (void)hipStreamSynchronize(st);
    undo();
    (void)hipEventDestroy(m.begin);
    (void)hipEventDestroy(m.done);
    (void)hipHostFree(m.pinned_map);
    if (m.pinned_descs) (void)hipHostFree(m.pinned_descs);
    return rc;
  }
  m.active = true;
  ix->mig = std::move(m);
  return IVF_OK;
}

extern "C" int ivf_migrate_stats(ivf_index_t *ix, uint64_t *bytes_copied, double *copy_ms,
                                 uint64_t *n_migrations) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  std::lock_guard<std::mutex> lk(ix->mu);
  if (bytes_copied) *bytes_copied = ix->bytes_migrated;
  if (copy_ms) *copy_ms = ix->migrate_ms;
  if (n_migrations) *n_migrations = ix->n_migrations;
  return IVF_OK;
}

extern "C" int ivf_migrate_poll(ivf_index_t *ix, int wait, uint64_t *bytes_copied) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  std::lock_guard<std::mutex> lk(ix->mu);
  int rc = ix->has_dev ? publish_if_done_locked(ix, wait != 0) : 0;
  if (rc < 0) return rc;
  if (ix->has_dev) reclaim(ix);
  if (bytes_copied) *bytes_copied = ix->bytes_migrated;
  return rc;
}

// ---------------------------------------------------------------------------
// tuning / instrumentation
// ---------------------------------------------------------------------------
extern "C" int ivf_set_tuning(ivf_index_t *ix, int32_t scan_slices, int32_t timing) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (scan_slices < 0 || scan_slices > kMaxSlices)
    return fail(IVF_EINVAL, "scan_slices must be in [0, %d]", kMaxSlices);
  if (timing < 0 || timing > 2) return fail(IVF_EINVAL, "timing must be 0, 1 or 2");
  std::lock_guard<std::mutex> lk(ix->mu);
  ix->tune_slices = scan_slices;
  ix->timing = timing;
  return IVF_OK;
}

static int drain_timing(ivf_index *ix) {
  for (auto &r : ix->trecs) {
    hipEvent_t last = nullptr;
    for (int i = 0; i <= IVF_N_STAGES; ++i)
      if (r.valid[i]) last = r.ev[i];
    if (last) HIP_TRY(hipEventSynchronize(last));
    for (int s = 0; s < IVF_N_STAGES; ++s) {
      if (r.valid[s] && r.valid[s + 1]) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, r.ev[s], r.ev[s + 1]));
        ix->t_ms[s] += ms;
        ix->t_n[s] += 1;
      }
    }
    for (int i = 0; i <= IVF_N_STAGES; ++i)
      if (r.valid[i]) (void)hipEventDestroy(r.ev[i]);
  }
  ix->trecs.clear();
  return IVF_OK;
}

extern "C" int ivf_stage_times(ivf_index_t *ix, double *ms, uint64_t *launches,
                               uint64_t *scan_bytes, int reset) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (!ix->has_dev) return fail(IVF_EDEVICE, "host-only index: no device stages");
  std::lock_guard<std::mutex> lk(ix->mu);
  int rc = drain_timing(ix);
  if (rc != IVF_OK) return rc;
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemcpy(ix->h_stats, ix->L.qstats, QS_COUNT * 8, hipMemcpyDeviceToHost));
  for (int s = 0; s < IVF_N_STAGES; ++s) {
    if (ms) ms[s] = ix->t_ms[s];
    if (launches) launches[s] = ix->t_n[s];
  }
  if (scan_bytes) *scan_bytes = ix->h_stats[QS_SCAN_BYTES];
  if (reset) {
    for (int s = 0; s < IVF_N_STAGES; ++s) {
      ix->t_ms[s] = 0;
      ix->t_n[s] = 0;
    }
    HIP_TRY(hipMemset(&ix->L.qstats[QS_SCAN_BYTES], 0, 8));
  }
  return IVF_OK;
}

// ---------------------------------------------------------------------------
// router counters
// ---------------------------------------------------------------------------
extern "C" int ivf_hit_stats(ivf_index_t *ix, uint64_t *per_cluster_hits, double *mean_hit_rate,
                             double *min_hit_rate, uint64_t *n_queries, int reset) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  std::lock_guard<std::mutex> lk(ix->mu);
  if (!ix->has_dev) {
    if (per_cluster_hits)
      memcpy(per_cluster_hits, ix->hc_hits.data(), (size_t)ix->sh.nlist * 8);
    if (mean_hit_rate) *mean_hit_rate = 0.0;
    if (min_hit_rate) *min_hit_rate = ix->hc_queries ? 0.0 : 1.0;
    if (n_queries) *n_queries = ix->hc_queries;
    if (reset) {
      std::fill(ix->hc_hits.begin(), ix->hc_hits.end(), 0);
      ix->hc_probes = ix->hc_queries = 0;
    }
    return IVF_OK;
  }
  HIP_TRY(hipDeviceSynchronize());
  if (per_cluster_hits)
    HIP_TRY(hipMemcpy(per_cluster_hits, ix->L.hits, (size_t)ix->sh.nlist * 8,
                      hipMemcpyDeviceToHost));
  HIP_TRY(hipMemcpy(ix->h_stats, ix->L.qstats, QS_COUNT * 8, hipMemcpyDeviceToHost));
  const unsigned long long res = ix->h_stats[QS_RESIDENT_PROBES], all = ix->h_stats[QS_PROBES];
  if (mean_hit_rate) *mean_hit_rate = all ? (double)res / (double)all : 0.0;
  if (min_hit_rate) {
    uint32_t bits = (uint32_t)(ix->h_stats[QS_MIN_RATE_BITS] & 0xffffffffull);
    float f;
    memcpy(&f, &bits, 4);
    *min_hit_rate = (double)f;
  }
  if (n_queries) *n_queries = ix->h_stats[QS_QUERIES];
  if (reset) {
    hipStream_t st = ix->own_stream;
    HIP_TRY(launch_fill_u32((uint32_t *)ix->L.hits, (size_t)ix->sh.nlist * 2, 0u, st));
    HIP_TRY(launch_fill_u32((uint32_t *)ix->L.qstats, 4 * 2, 0u, st));
    HIP_TRY(launch_fill_u32((uint32_t *)&ix->L.qstats[QS_MIN_RATE_BITS], 1, 0x3f800000u, st));
    HIP_TRY(hipStreamSynchronize(st));
  }
  return IVF_OK;
}

// ---------------------------------------------------------------------------
// search
// ---------------------------------------------------------------------------
static void emit_results(const ivf_index *ix, const HostCand *c, int k, int e, int64_t *ids,
                         float *dists) {
  for (int r = 0; r < k; ++r) {
    if (c[r].key == kKeyInvalid) {
      ids[r] = -1;
      dists[r] = ix->sh.metric_ip ? -INFINITY : INFINITY;
    } else {
      ids[r] = c[r].id;
      dists[r] = key_to_dist(c[r].key, e, ix->sh.metric_ip);
    }
  }
}

static int pick_slices(const ivf_index *ix, int64_t nq) {
  if (ix->tune_slices > 0) return ix->tune_slices;
  // one block per query fills the chip from 256 queries up; below that, split
  int s = (int)((256 + nq - 1) / nq);
  if (s < 1) s = 1;
  if (s > kMaxSlices) s = kMaxSlices;
  return s;
}

// Search on a device-less index: every probe is scanned on the CPU.
static int search_host_only(ivf_index *ix, const float *queries, int64_t nq, const int32_t *probe,
                            int nprobe, int k, int64_t *out_ids, float *out_dists) {
  const HostIndexView view = host_view(ix);
  std::vector<int64_t> ids((size_t)nq * k);
  std::vector<float> dists((size_t)nq * k);
  parallel_for(nq, [&](int64_t q) {
    std::vector<int32_t> lut((size_t)view.M * 256);
    std::vector<HostCand> cand(k);
    const float *qv = queries + (size_t)q * view.d;
    const int32_t *pr = probe + (size_t)q * nprobe;
    const int e = cpu_build_lut(view, qv, cpu_max_bias(view, qv, pr, nprobe), lut.data());
    cpu_scan_lists(view, lut.data(), e, qv, pr, nprobe, k, cand.data());
    emit_results(ix, cand.data(), k, e, &ids[(size_t)q * k], &dists[(size_t)q * k]);
  });
  {
    std::lock_guard<std::mutex> lk(ix->mu);
    for (int64_t i = 0; i < nq * nprobe; ++i)
      if (probe[i] >= 0) {
        ix->hc_hits[probe[i]] += 1;
        ix->hc_probes += 1;
      }
    ix->hc_queries += (uint64_t)nq;
  }
  memcpy(out_ids, ids.data(), ids.size() * 8);
  memcpy(out_dists, dists.data(), dists.size() * 4);
  return IVF_OK;
}

// Workspace slot for a batch on stream st (caller holds ix->mu).
static int acquire_slot_locked(ivf_index *ix, hipStream_t st, int *slot) {
  int pick = -1;
  for (int i = 0; i < kWsSlots; ++i)
    if (ix->slot_used[i] && ix->slot_stream[i] == st) pick = i;
  if (pick < 0)
    for (int i = 0; i < kWsSlots; ++i)
      if (!ix->slot_used[i]) {
        pick = i;
        break;
      }
  if (pick < 0) {
    pick = 0;
    for (int i = 1; i < kWsSlots; ++i)
      if (ix->slot_tick[i] < ix->slot_tick[pick]) pick = i;
    HIP_TRY(hipStreamSynchronize(ix->slot_stream[pick]));
  }
  ix->slot_used[pick] = true;
  ix->slot_stream[pick] = st;
  ix->slot_tick[pick] = ++ix->tick;
  *slot = pick;
  return IVF_OK;
}

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
  uint64_t ver_id = 0;
};

static int begin_batch(ivf_index *ix, hipStream_t st, BatchCtx *c) {
  std::lock_guard<std::mutex> lk(ix->mu);
  int rc = acquire_slot_locked(ix, st, &c->slot);
  if (rc < 0) return rc;
  rc = publish_if_done_locked(ix, false);
  if (rc < 0) return rc;
  reclaim(ix);
  Version &ver = ix->versions.back();
  ver.refs += 1;
  c->ver_id = ver.id;
  c->buf = ver.buf;
  c->all_resident = ix->resident_clusters == ix->sh.nlist;
  c->any_resident = ix->resident_clusters > 0;
  c->timing = ix->timing;
  return IVF_OK;
}

// Drop the hold on the mapping-table version.  async_tail: device work that
// reads the table may still be queued on st, so leave an event behind.
static void end_batch(ivf_index *ix, const BatchCtx &c, hipStream_t st, bool async_tail) {
  std::lock_guard<std::mutex> lk(ix->mu);
  for (auto &v : ix->versions) {
    if (v.id != c.ver_id) continue;
    if (async_tail) {
      hipEvent_t e = get_event(ix);
      if (e && hipEventRecord(e, st) == hipSuccess) v.events.push_back(e);
      else (void)hipStreamSynchronize(st);
    }
    v.refs -= 1;
    break;
  }
}

// Enqueue the device side of one batch on a.st: coarse quantizer (or the
// caller's probes), routing, lookup tables, scan of the resident probes and
// merge of the slices.  final_on_gpu: every probe is resident and the merge
// writes ids and distances; otherwise the per-query partial results, the cold
// probe lists and the scale inputs are copied to the index's pinned buffers.
// ev_route (optional) is recorded once the cold lists are on their way, so a
// host thread can start on them while the device scans.
static int enqueue_gpu(ivf_index *ix, const SearchArgs &a, const BatchCtx &c, bool final_on_gpu,
                       hipEvent_t ev_route) {
  const DevLayout &L = ix->L;
  const Shape &sh = ix->sh;
  const int nq = (int)a.nq, k = a.k, np = a.nprobe;
  hipStream_t st = a.st;
  const BatchWs &W = L.ws[c.slot];

  TimingRec trec;
  memset(&trec, 0, sizeof(trec));
  auto mark = [&](int i) -> hipError_t {
    if (!c.timing) return hipSuccess;
    if (c.timing == 2 && i != IVF_STAGE_SCAN && i != IVF_STAGE_MERGE) return hipSuccess;
    hipError_t e = hipEventCreate(&trec.ev[i]);
    if (e != hipSuccess) return e;
    trec.valid[i] = true;
    return hipEventRecord(trec.ev[i], st);
  };
  auto keep_timing = [&]() {
    if (!c.timing) return;
    std::lock_guard<std::mutex> lk(ix->mu);
    ix->trecs.push_back(trec);
  };
#define G_TRY(expr)                                                                        \
  do {                                                                                     \
    hipError_t _e = (expr);                                                                \
    if (_e != hipSuccess) {                                                                \
      keep_timing();                                                                       \
      return fail(IVF_EDEVICE, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e),      \
                  __FILE__, __LINE__);                                                     \
    }                                                                                      \
  } while (0)

  const float *dq = a.q_dev;
  if (!dq) {
    G_TRY(hipMemcpyAsync(W.queries, a.q_host, (size_t)nq * sh.d * 4, hipMemcpyHostToDevice, st));
    dq = W.queries;
  }
  // ---- stage 2 first: the lookup tables depend on the queries only ----
  G_TRY(mark(IVF_STAGE_LUT));
  int lut_parts = 0;
  if (c.any_resident)
    G_TRY(launch_lut(sh, dq, nq, L.cbT, W.lut, W.lutpart, &lut_parts, st));
  // ---- stage 1: coarse quantizer (or the caller's probe list) ----
  G_TRY(mark(IVF_STAGE_COARSE_GEMM));
  if (a.probe_host) {
    memcpy(ix->h_probe, a.probe_host, (size_t)nq * np * 4);
    G_TRY(hipMemcpyAsync(W.probe, ix->h_probe, (size_t)nq * np * 4, hipMemcpyHostToDevice, st));
    G_TRY(mark(IVF_STAGE_COARSE_SELECT));
  } else {
    G_TRY(launch_split_f16(dq, (size_t)nq, sh.d, W.q_parts, W.q_exp, st));
    G_TRY(launch_coarse_gemm(sh, W.q_parts, W.q_exp, nq, L.cent_parts, L.cent_exp, L.cent_norm,
                             W.scores, st));
    G_TRY(mark(IVF_STAGE_COARSE_SELECT));
    G_TRY(launch_coarse_select(sh, W.scores, nq, np, np, W.probe, st));
  }
  // ---- routing ----
  G_TRY(mark(IVF_STAGE_ROUTE));
  if (sh.by_residual)
    G_TRY(launch_bias(sh, dq, nq, W.probe, np, np, L.centroids, W.bias, st));
  G_TRY(launch_route(W.probe, nq, np, np, sh.nlist, L.clus_tile[c.buf], L.clus_len, sh.M, W.g_base, W.g_len,
                     W.g_prefix, W.g_n, W.cold, W.n_cold, W.q_vecs,
                     sh.by_residual ? W.bias : nullptr, W.g_bias, W.qbmax, L.hits, 1, W.lutpart,
                     lut_parts, W.lutmax, st));
  G_TRY(launch_order(W, nq, np, sh.M, L.qstats, 1, st));
  if (!final_on_gpu) {
    // cold probes go to the CPU (Section 4.3.1)
    G_TRY(hipMemcpyAsync(ix->h_ncold, W.n_cold, (size_t)nq * 4, hipMemcpyDeviceToHost, st));
    G_TRY(hipMemcpyAsync(ix->h_cold, W.cold, (size_t)nq * np * 4, hipMemcpyDeviceToHost, st));
    G_TRY(hipMemcpyAsync(ix->h_qbmax, W.qbmax, (size_t)nq * 4, hipMemcpyDeviceToHost, st));
    if (!a.q_host)
      G_TRY(hipMemcpyAsync(ix->h_queries, dq, (size_t)nq * sh.d * 4, hipMemcpyDeviceToHost, st));
    if (ev_route) G_TRY(hipEventRecord(ev_route, st));
  }
  if (c.any_resident) {
    // ---- stage 3: scan + top-k ----
    const int slices = pick_slices(ix, nq);
    int64_t *oid = nullptr;
    float *od = nullptr;
    if (final_on_gpu) {
      oid = a.out_device ? a.out_ids : W.out_ids;
      od = a.out_device ? a.out_dists : W.out_dists;
    }
    G_TRY(mark(IVF_STAGE_SCAN));
    G_TRY(launch_scan(sh, L, W, nq, np, slices, k, oid, od, st));
    G_TRY(mark(IVF_STAGE_MERGE));
    if (slices > 1) G_TRY(launch_merge(sh, W, nq, slices, k, oid, od, st));
    G_TRY(mark(IVF_N_STAGES));
    if (!final_on_gpu) {
      G_TRY(hipMemcpyAsync(ix->h_reskey, W.res_key, (size_t)nq * k * 4, hipMemcpyDeviceToHost, st));
      G_TRY(hipMemcpyAsync(ix->h_resid, W.res_id, (size_t)nq * k * 8, hipMemcpyDeviceToHost, st));
      G_TRY(hipMemcpyAsync(ix->h_lutmax, W.lutmax, (size_t)nq * 4, hipMemcpyDeviceToHost, st));
    }
  }
  keep_timing();
  return IVF_OK;
#undef G_TRY
}

// Final result of query q of a hybrid batch: the device's partial top-k (if any
// cluster is resident) merged with the CPU scan of its cold probes.  cpu_e is the
// table exponent the CPU scan used (only read when cpu is non-NULL).  Returns
// false if the CPU and the device disagree on the exponent.
static bool finish_query(const ivf_index *ix, const HostIndexView &view, bool any_resident,
                         int64_t q, int k, const HostCand *cpu, int cpu_e, int64_t *ids,
                         float *dists) {
  std::vector<HostCand> gpu((size_t)k), fin((size_t)k);
  for (int r = 0; r < k; ++r) {
    if (any_resident) gpu[r] = HostCand{ix->h_reskey[q * k + r], ix->h_resid[q * k + r]};
    else gpu[r] = HostCand{kKeyInvalid, -1};
  }
  int e = 0;
  if (any_resident) {
    float mx;
    memcpy(&mx, &ix->h_lutmax[q], 4);
    e = lut_exponent(mx, view.M, ix->h_qbmax[q], view.pv ? view.pv_max : 0.0f);
  }
  const HostCand *res = gpu.data();
  bool ok = true;
  if (cpu) {
    if (any_resident && cpu_e != e) ok = false;
    e = cpu_e;
    merge_topk(gpu.data(), cpu, k, fin.data());
    res = fin.data();
  }
  emit_results(ix, res, k, e, ids, dists);
  return ok;
}

static int search_device(ivf_index *ix, const SearchArgs &a) {
  const int nq = (int)a.nq, k = a.k;
  const int np = a.nprobe;
  hipStream_t st = a.st;

  {
    std::lock_guard<std::mutex> lk(ix->mu);
    if (ix->dispatch_active)
      return fail(IVF_EBUSY, "an asynchronous batch is still in flight on this index");
  }
  BatchCtx ctx;
  int rc = begin_batch(ix, st, &ctx);
  if (rc < 0) return rc;
  const BatchWs &W = ix->L.ws[ctx.slot];
  const bool final_on_gpu = ctx.all_resident;
  const bool any_resident = ctx.any_resident;
  rc = enqueue_gpu(ix, a, ctx, final_on_gpu, nullptr);
  if (rc < 0) {
    (void)hipStreamSynchronize(st);
    end_batch(ix, ctx, st, false);
    return rc;
  }
#define S_TRY(expr)                                                                        \
  do {                                                                                     \
    hipError_t _e = (expr);                                                                \
    if (_e != hipSuccess) {                                                                \
      (void)hipStreamSynchronize(st);                                                      \
      end_batch(ix, ctx, st, false);                                                       \
      return fail(IVF_EDEVICE, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e),      \
                  __FILE__, __LINE__);                                                     \
    }                                                                                      \
  } while (0)

  if (final_on_gpu) {
    if (a.out_device) {
      end_batch(ix, ctx, st, true);  // asynchronous: outputs valid when the stream gets here
      return IVF_OK;
    }
    S_TRY(hipMemcpyAsync(ix->h_outids, W.out_ids, (size_t)nq * k * 8, hipMemcpyDeviceToHost, st));
    S_TRY(hipMemcpyAsync(ix->h_outd, W.out_dists, (size_t)nq * k * 4, hipMemcpyDeviceToHost, st));
    S_TRY(hipStreamSynchronize(st));
    end_batch(ix, ctx, st, false);
    memcpy(a.out_ids, ix->h_outids, (size_t)nq * k * 8);
    memcpy(a.out_dists, ix->h_outd, (size_t)nq * k * 4);
    return IVF_OK;
  }

  // ---- hybrid: cold probes on the CPU, then merge (Sections 4.3.1, 4.3.2) ----
  S_TRY(hipStreamSynchronize(st));
  end_batch(ix, ctx, st, false);
  const float *hq = a.q_host ? a.q_host : ix->h_queries;

  const HostIndexView view = host_view(ix);
  std::vector<int> bad(1, 0);
  parallel_for(nq, [&](int64_t q) {
    const int nc = ix->h_ncold[q];
    std::vector<HostCand> cpu;
    int e_cpu = 0;
    if (nc > 0 || !any_resident) {
      std::vector<int32_t> lut((size_t)view.M * 256);
      cpu.resize((size_t)k);
      const float *qv = hq + (size_t)q * view.d;
      e_cpu = cpu_build_lut(view, qv, ix->h_qbmax[q], lut.data());
      cpu_scan_lists(view, lut.data(), e_cpu, qv, ix->h_cold + (size_t)q * np, nc, k, cpu.data());
    }
    if (!finish_query(ix, view, any_resident, q, k, cpu.empty() ? nullptr : cpu.data(), e_cpu,
                      &ix->h_outids[(size_t)q * k], &ix->h_outd[(size_t)q * k]))
      __atomic_store_n(&bad[0], 1, __ATOMIC_RELAXED);
  });
  if (bad[0])
    return fail(IVF_EDEVICE, "internal: CPU and GPU lookup-table scales disagree");
  if (a.out_device) {
    HIP_TRY(hipMemcpyAsync(a.out_ids, ix->h_outids, (size_t)nq * k * 8, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(a.out_dists, ix->h_outd, (size_t)nq * k * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
  } else {
    memcpy(a.out_ids, ix->h_outids, (size_t)nq * k * 8);
    memcpy(a.out_dists, ix->h_outd, (size_t)nq * k * 4);
  }
  return IVF_OK;
#undef S_TRY
}

static int check_search_args(const ivf_index *ix, const void *queries, int64_t nq, int32_t nprobe,
                             int32_t k, const void *out_ids, const void *out_dists) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (nq < 0) return fail(IVF_EINVAL, "nq is negative");
  if (nprobe < 1) return fail(IVF_EINVAL, "nprobe must be >= 1");
  if (k < 1) return fail(IVF_EINVAL, "k must be >= 1");
  if (nq == 0) return IVF_OK;
  if (!queries || !out_ids || !out_dists) return fail(IVF_EINVAL, "NULL buffer");
  if (ix->has_dev) {
    if (nq > ix->desc.max_nq) return fail(IVF_EINVAL, "nq %lld exceeds max_nq %d", (long long)nq, ix->desc.max_nq);
    if (k > ix->desc.max_k) return fail(IVF_EINVAL, "k %d exceeds max_k %d", k, ix->desc.max_k);
  } else if (k > kMaxK) {
    return fail(IVF_EINVAL, "k %d exceeds %d", k, kMaxK);
  }
  return IVF_OK;
}

// A caller's probe list: ids below nlist (negative = no probe), distinct within a query.
static int check_probe_list(const ivf_index *ix, const int32_t *probe, int64_t nq, int nprobe) {
  std::vector<int32_t> row((size_t)nprobe);
  for (int64_t q = 0; q < nq; ++q) {
    int n = 0;
    for (int p = 0; p < nprobe; ++p) {
      const int32_t c = probe[q * nprobe + p];
      if (c >= ix->sh.nlist) return fail(IVF_EINVAL, "probe id %d out of range", c);
      if (c >= 0) row[n++] = c;
    }
    std::sort(row.begin(), row.begin() + n);
    if (std::adjacent_find(row.begin(), row.begin() + n) != row.begin() + n)
      return fail(IVF_EINVAL, "query %lld lists a cluster twice", (long long)q);
  }
  return IVF_OK;
}

extern "C" int ivf_search_batch(ivf_index_t *ix, const float *queries, int64_t nq, int32_t nprobe,
                                int32_t k, int64_t *out_ids, float *out_dists) {
  int rc = check_search_args(ix, queries, nq, nprobe, k, out_ids, out_dists);
  if (rc != IVF_OK || nq == 0) return rc;
  if (!ix->has_dev)
    return fail(IVF_EDEVICE, "host-only index: the coarse quantizer needs the device "
                             "(use ivf_search_batch_probes)");
  SearchArgs a;
  a.q_host = queries;
  a.nq = nq;
  a.nprobe = std::min<int32_t>(nprobe, ix->sh.nlist);
  if (a.nprobe > ix->desc.max_nprobe)
    return fail(IVF_EINVAL, "nprobe %d exceeds max_nprobe %d", a.nprobe, ix->desc.max_nprobe);
  a.k = k;
  a.out_ids = out_ids;
  a.out_dists = out_dists;
  a.st = ix->own_stream;
  return search_device(ix, a);
}

extern "C" int ivf_search_batch_dev(ivf_index_t *ix, const float *queries, int64_t nq,
                                    int32_t nprobe, int32_t k, int64_t *out_ids, float *out_dists,
                                    void *stream) {
  int rc = check_search_args(ix, queries, nq, nprobe, k, out_ids, out_dists);
  if (rc != IVF_OK || nq == 0) return rc;
  if (!ix->has_dev) return fail(IVF_EDEVICE, "host-only index: no device search");
  SearchArgs a;
  a.q_dev = queries;
  a.nq = nq;
  a.nprobe = std::min<int32_t>(nprobe, ix->sh.nlist);
  if (a.nprobe > ix->desc.max_nprobe)
    return fail(IVF_EINVAL, "nprobe %d exceeds max_nprobe %d", a.nprobe, ix->desc.max_nprobe);
  a.k = k;
  a.out_ids = out_ids;
  a.out_dists = out_dists;
  a.out_device = true;
  a.st = (hipStream_t)stream;
  return search_device(ix, a);
}

extern "C" int ivf_coarse_probe_dev(ivf_index_t *ix, const float *queries, int64_t nq,
                                    int32_t nprobe, int32_t *out_probe, void *stream) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (!ix->has_dev) return fail(IVF_EDEVICE, "host-only index: no device coarse quantizer");
  if (nq < 0 || nprobe < 1) return fail(IVF_EINVAL, "bad nq / nprobe");
  if (nq == 0) return IVF_OK;
  if (!queries || !out_probe) return fail(IVF_EINVAL, "NULL buffer");
  if (nq > ix->desc.max_nq) return fail(IVF_EINVAL, "nq exceeds max_nq");
  if (nprobe > kMaxNprobe) return fail(IVF_EINVAL, "nprobe exceeds %d", kMaxNprobe);
  hipStream_t st = (hipStream_t)stream;
  int slot = 0;
  {
    std::lock_guard<std::mutex> lk(ix->mu);
    int rc = acquire_slot_locked(ix, st, &slot);
    if (rc < 0) return rc;
  }
  const BatchWs &W = ix->L.ws[slot];
  HIP_TRY(launch_split_f16(queries, (size_t)nq, ix->sh.d, W.q_parts, W.q_exp, st));
  HIP_TRY(launch_coarse_gemm(ix->sh, W.q_parts, W.q_exp, (int)nq, ix->L.cent_parts, ix->L.cent_exp,
                             ix->L.cent_norm,
                             W.scores, st));
  HIP_TRY(launch_coarse_select(ix->sh, W.scores, (int)nq, nprobe, nprobe, out_probe, st));
  return IVF_OK;
}

extern "C" int ivf_search_batch_probes(ivf_index_t *ix, const float *queries, int64_t nq,
                                       const int32_t *probe, int32_t nprobe, int32_t k,
                                       int64_t *out_ids, float *out_dists) {
  int rc = check_search_args(ix, queries, nq, nprobe, k, out_ids, out_dists);
  if (rc != IVF_OK || nq == 0) return rc;
  if (!probe) return fail(IVF_EINVAL, "probe is NULL");
  if (ix->has_dev && nprobe > ix->desc.max_nprobe)
    return fail(IVF_EINVAL, "nprobe %d exceeds max_nprobe %d", nprobe, ix->desc.max_nprobe);
  rc = check_probe_list(ix, probe, nq, nprobe);
  if (rc != IVF_OK) return rc;
  if (!ix->has_dev) return search_host_only(ix, queries, nq, probe, nprobe, k, out_ids, out_dists);
  SearchArgs a;
  a.q_host = queries;
  a.probe_host = probe;
  a.nq = nq;
  a.nprobe = nprobe;
  a.k = k;
  a.out_ids = out_ids;
  a.out_dists = out_dists;
  a.st = ix->own_stream;
  return search_device(ix, a);
}

// ---------------------------------------------------------------------------
// dynamic dispatcher (Section 4.3.2): per-query completion of a hybrid batch
// ---------------------------------------------------------------------------
struct ivf_ticket {
  ivf_index *ix = nullptr;
  int nq = 0, np = 0, k = 0;
  bool device = false;        // the batch has a device side
  bool any_resident = false;
  BatchCtx ctx;
  hipStream_t st = nullptr;
  hipEvent_t ev_route = nullptr, ev_gpu = nullptr;
  const float *hq = nullptr;        // caller's queries (borrowed until wait)
  std::vector<int32_t> own_probe;   // device-less index: the caller's probe list
  int64_t *out_ids = nullptr;
  float *out_dists = nullptr;
  ivf_query_done_fn on_done = nullptr;
  void *user = nullptr;

  std::thread dispatcher;
  std::mutex mu;
  std::condition_variable cv;
  std::deque<int32_t> ready;        // queries whose CPU scan count reached its expected value
  std::vector<int32_t> forwarded;   // queries handed downstream, in completion order
  size_t polled = 0;
  bool finished = false;
  int rc = IVF_OK;
  std::string err;

  std::vector<HostCand> cpu_res;    // [nq][k] CPU partial results
  std::vector<int> cpu_e;           // table exponent of each query's CPU scan
  std::vector<int32_t> scanned;     // clusters scanned so far, per query
  std::vector<double> done_ms;      // time from the call to the hand-off, per query
  std::chrono::steady_clock::time_point t0;
};

static void ticket_fail(ivf_ticket *t, int code, const std::string &msg) {
  std::lock_guard<std::mutex> lk(t->mu);
  if (t->rc == IVF_OK) {
    t->rc = code;
    t->err = msg;
  }
}

static void dispatcher_main(ivf_ticket *t) {
  ivf_index *ix = t->ix;
  const int nq = t->nq, np = t->np, k = t->k;
  const HostIndexView view = host_view(ix);
  bool gpu_ok = true;
  if (t->device) {
    hipError_t e = hipSetDevice(ix->device);
    // the cold probe lists and scale inputs are on the host once routing is done
    if (e == hipSuccess) e = hipEventSynchronize(t->ev_route);
    if (e != hipSuccess) {
      ticket_fail(t, IVF_EDEVICE, std::string("routing failed: ") + hipGetErrorString(e));
      gpu_ok = false;
    }
  }
  const int32_t *cold = t->device ? ix->h_cold : t->own_probe.data();
  auto expected = [&](int q) { return t->device ? ix->h_ncold[q] : np; };

  std::vector<std::thread> workers;
  std::atomic<int64_t> next(0);
  std::vector<int32_t> order((size_t)nq);
  if (gpu_ok) {
    // CPU search loop.  Queries are taken fewest cold probes first, so that the
    // ones the GPU served almost entirely are handed on earliest.
    for (int q = 0; q < nq; ++q) order[q] = q;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return expected(a) < expected(b); });
    auto work = [&]() {
      std::vector<int32_t> lut((size_t)view.M * 256);
      for (;;) {
        const int64_t i = next.fetch_add(1, std::memory_order_relaxed);
        if (i >= nq) break;
        const int q = order[(size_t)i];
        const int nc = expected(q);
        if (nc > 0) {
          const float *qv = t->hq + (size_t)q * view.d;
          const int32_t *pr = cold + (size_t)q * np;
          const float mb = t->device ? ix->h_qbmax[q] : cpu_max_bias(view, qv, pr, nc);
          const int e = cpu_build_lut(view, qv, mb, lut.data());
          t->cpu_e[q] = e;
          cpu_scan_lists(view, lut.data(), e, qv, pr, nc, k, &t->cpu_res[(size_t)q * k],
                         &t->scanned[q]);
        }
        // scan count == expected count: the query goes to the completed queue
        if (__atomic_load_n(&t->scanned[q], __ATOMIC_ACQUIRE) == nc) {
          {
            std::lock_guard<std::mutex> lk(t->mu);
            t->ready.push_back(q);
          }
          t->cv.notify_one();
        }
      }
    };
    const int nt = (int)std::min<int64_t>(cpu_threads(), nq);
    for (int i = 0; i < nt; ++i) workers.emplace_back(work);
  }

  // the GPU's completion flag: its partial results are on the host
  if (t->device && gpu_ok) {
    hipError_t e = hipEventSynchronize(t->ev_gpu);
    if (e != hipSuccess) {
      ticket_fail(t, IVF_EDEVICE, std::string("device scan failed: ") + hipGetErrorString(e));
      gpu_ok = false;
    }
  }
  if (t->device) end_batch(ix, t->ctx, t->st, false);

  // poll the completed queue: merge, re-rank, hand on
  int n_done = 0;
  std::vector<int32_t> batch;
  while (gpu_ok && n_done < nq) {
    {
      std::unique_lock<std::mutex> lk(t->mu);
      t->cv.wait_for(lk, std::chrono::microseconds(200), [&] { return !t->ready.empty(); });
      batch.assign(t->ready.begin(), t->ready.end());
      t->ready.clear();
    }
    for (int32_t q : batch) {
      int64_t *ids = t->out_ids + (size_t)q * k;
      float *dists = t->out_dists + (size_t)q * k;
      const bool has_cpu = expected(q) > 0;
      if (!finish_query(ix, view, t->any_resident, q, k,
                        has_cpu ? &t->cpu_res[(size_t)q * k] : nullptr, t->cpu_e[q], ids, dists))
        ticket_fail(t, IVF_EDEVICE, "internal: CPU and GPU lookup-table scales disagree");
      t->done_ms[q] =
          std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t->t0)
              .count();
      {
        std::lock_guard<std::mutex> lk(t->mu);
        t->forwarded.push_back(q);
      }
      if (t->on_done) t->on_done(t->user, q, ids, dists, k);
      ++n_done;
    }
  }
  for (auto &w : workers) w.join();
  {
    std::lock_guard<std::mutex> lk(t->mu);
    t->finished = true;
  }
}

extern "C" int ivf_search_batch_async(ivf_index_t *ix, const float *queries, int64_t nq,
                                      const int32_t *probe, int32_t nprobe, int32_t k,
                                      int64_t *out_ids, float *out_dists,
                                      ivf_query_done_fn on_done, void *user,
                                      ivf_ticket_t **ticket) {
  if (!ticket) return fail(IVF_EINVAL, "ticket is NULL");
  *ticket = nullptr;
  int rc = check_search_args(ix, queries, nq, nprobe, k, out_ids, out_dists);
  if (rc != IVF_OK) return rc;
  if (nq > 0x7fffffff) return fail(IVF_EINVAL, "nq too large");
  if (!ix->has_dev && !probe)
    return fail(IVF_EDEVICE, "host-only index: the coarse quantizer needs the device "
                             "(pass a probe list)");
  int np = nprobe;
  if (!probe) np = std::min<int32_t>(nprobe, ix->sh.nlist);
  if (ix->has_dev && np > ix->desc.max_nprobe)
    return fail(IVF_EINVAL, "nprobe %d exceeds max_nprobe %d", np, ix->desc.max_nprobe);
  if (!ix->has_dev && np > kMaxNprobe) return fail(IVF_EINVAL, "nprobe %d exceeds %d", np, kMaxNprobe);
  if (probe && nq > 0) {
    rc = check_probe_list(ix, probe, nq, np);
    if (rc != IVF_OK) return rc;
  }
  {
    std::lock_guard<std::mutex> lk(ix->mu);
    if (ix->dispatch_active)
      return fail(IVF_EBUSY, "an asynchronous batch is still in flight on this index");
    ix->dispatch_active = true;
  }
  ivf_ticket *t = new ivf_ticket();
  auto abandon = [&](int code) {
    if (t->ev_route) (void)hipEventDestroy(t->ev_route);
    if (t->ev_gpu) (void)hipEventDestroy(t->ev_gpu);
    delete t;
    std::lock_guard<std::mutex> lk(ix->mu);
    ix->dispatch_active = false;
    return code;
  };
  t->ix = ix;
  t->nq = (int)nq;
  t->np = np;
  t->k = k;
  t->hq = queries;
  t->out_ids = out_ids;
  t->out_dists = out_dists;
  t->on_done = on_done;
  t->user = user;
  t->device = ix->has_dev;
  t->cpu_res.resize((size_t)nq * k);
  t->cpu_e.assign((size_t)nq, 0);
  t->scanned.assign((size_t)nq, 0);
  t->done_ms.assign((size_t)nq, 0.0);
  t->t0 = std::chrono::steady_clock::now();
  if (nq == 0) {
    t->finished = true;
    *ticket = t;
    return IVF_OK;
  }
  if (t->device) {
    hipError_t e;
    if ((e = hipEventCreateWithFlags(&t->ev_route, hipEventDisableTiming)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&t->ev_gpu, hipEventDisableTiming)) != hipSuccess)
      return abandon(fail(IVF_EDEVICE, "hipEventCreate failed: %s", hipGetErrorString(e)));
    t->st = ix->own_stream;
    rc = begin_batch(ix, t->st, &t->ctx);
    if (rc < 0) return abandon(rc);
    t->any_resident = t->ctx.any_resident;
    SearchArgs a;
    a.q_host = queries;
    a.probe_host = probe;
    a.nq = nq;
    a.nprobe = np;
    a.k = k;
    a.st = t->st;
    rc = enqueue_gpu(ix, a, t->ctx, /*final_on_gpu=*/false, t->ev_route);
    if (rc == IVF_OK && hipEventRecord(t->ev_gpu, t->st) != hipSuccess)
      rc = fail(IVF_EDEVICE, "hipEventRecord failed");
    if (rc < 0) {
      (void)hipStreamSynchronize(t->st);
      end_batch(ix, t->ctx, t->st, false);
      return abandon(rc);
    }
  } else {
    t->own_probe.assign(probe, probe + (size_t)nq * np);
    std::lock_guard<std::mutex> lk(ix->mu);
    for (int64_t i = 0; i < nq * np; ++i)
      if (probe[i] >= 0) {
        ix->hc_hits[probe[i]] += 1;
        ix->hc_probes += 1;
      }
    ix->hc_queries += (uint64_t)nq;
  }
  t->dispatcher = std::thread(dispatcher_main, t);
  *ticket = t;
  return IVF_OK;
}

extern "C" int ivf_search_poll(ivf_ticket_t *t, int64_t *queries_done, int64_t cap,
                               int64_t *n_done, int32_t *finished) {
  if (!t || !n_done || !finished || cap < 0 || (cap > 0 && !queries_done))
    return fail(IVF_EINVAL, "bad argument");
  std::lock_guard<std::mutex> lk(t->mu);
  int64_t n = 0;
  while (n < cap && t->polled < t->forwarded.size()) queries_done[n++] = t->forwarded[t->polled++];
  *n_done = n;
  *finished = (t->finished && t->polled == t->forwarded.size()) ? 1 : 0;
  if (t->rc != IVF_OK) return fail(t->rc, "%s", t->err.c_str());
  return IVF_OK;
}

extern "C" int ivf_search_wait(ivf_ticket_t *t, double *done_ms) {
  if (!t) return fail(IVF_EINVAL, "ticket is NULL");
  if (t->dispatcher.joinable()) t->dispatcher.join();
  if (done_ms && t->rc == IVF_OK)
    for (int q = 0; q < t->nq; ++q) done_ms[q] = t->done_ms[q];
  const int rc = t->rc;
  const std::string err = t->err;
  if (t->ev_route) (void)hipEventDestroy(t->ev_route);
  if (t->ev_gpu) (void)hipEventDestroy(t->ev_gpu);
  {
    std::lock_guard<std::mutex> lk(t->ix->mu);
    t->ix->dispatch_active = false;
  }
  delete t;
  if (rc != IVF_OK) return fail(rc, "%s", err.c_str());
  return IVF_OK;
}

extern "C" int ivf_calib_copy(const void *src, void *dst, size_t bytes, void *stream) {
  if (!src || !dst || bytes % 16 != 0) return fail(IVF_EINVAL, "calib copy: bad arguments");
  HIP_TRY(launch_calib_copy(src, dst, bytes, (hipStream_t)stream));
  return IVF_OK;
}

extern "C" int ivf_calib_read(const void *src, void *sink, size_t bytes, void *stream) {
  if (!src || !sink || bytes % 16 != 0) return fail(IVF_EINVAL, "calib read: bad arguments");
  HIP_TRY(launch_calib_read(src, sink, bytes, (hipStream_t)stream));
  return IVF_OK;
}
