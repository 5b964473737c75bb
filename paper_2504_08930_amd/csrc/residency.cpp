// C ABI, part 2: residency.  Mapping-table versions, the cluster-region
// allocator's clients (full refresh and per-cluster migration), host-to-device
// cluster copies through the staging area.
#include "index_state.h"

// ---------------------------------------------------------------------------
// version bookkeeping (caller holds ix->mu)
// ---------------------------------------------------------------------------
hipEvent_t get_event(ivf_index *ix) {
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
void reclaim(ivf_index *ix) {
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
  if (ix->zc_codes && (!with_pv || ix->zc_pv)) {
    // the caller's arrays are pinned: the kernel reads them itself, only the tile
    // descriptors pass through the staging area
    const size_t desc_cap = std::min<size_t>(L.staging_bytes / sizeof(TileDesc), (size_t)1 << 20);
    if (desc_cap == 0) return fail(IVF_ENOMEM, "staging area too small");
    size_t n = 0;       // descriptors written
    size_t sent = 0;    // descriptors already handed to a launch
    auto flush = [&]() -> int {
      if (n == sent) return IVF_OK;
      HIP_TRY(hipMemcpyAsync(L.staging, descs + sent, (n - sent) * sizeof(TileDesc),
                             hipMemcpyHostToDevice, st));
      HIP_TRY(launch_interleave_direct(ix->zc_codes, ix->zc_ids, ix->zc_pv,
                                       (const TileDesc *)L.staging, (int)(n - sent), (int)M,
                                       L.tile_codes, L.tile_ids, L.tile_pv, st));
      sent = n;
      return IVF_OK;
    };
    for (size_t ci = 0; ci < clusters.size(); ++ci) {
      const int32_t c = clusters[ci];
      const int32_t len = ix->h_len[c];
      const int64_t nt = tiles_of(len);
      for (int64_t t = 0; t < nt; ++t) {
        TileDesc &d = descs[n++];
        d.dst_tile = (int32_t)(bases[ci] + t);
        d.src_vec = (int32_t)(ix->desc.list_offsets[c] + t * kTileVecs);
        d.n_valid = (int32_t)std::min<int64_t>(kTileVecs, len - t * kTileVecs);
        d.pad = 0;
        if (n - sent == desc_cap) {
          int rc = flush();
          if (rc != IVF_OK) return rc;
        }
      }
    }
    return flush();
  }
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
        HIP_TRY(hipMemcpyAsync(st_pv + (size_t)run_dst * 4, ix->pv_host() + run_src,
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

extern "C" int ivf_resident_list(ivf_index_t *ix, int32_t *cluster_ids, int32_t cap, int32_t *n) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (!n || cap < 0 || (cap > 0 && !cluster_ids)) return fail(IVF_EINVAL, "resident_list: bad arguments");
  std::lock_guard<std::mutex> lk(ix->mu);
  *n = ix->resident_clusters;
  if (cap < ix->resident_clusters)
    return fail(IVF_EINVAL, "resident_list: %d clusters are resident, the array holds %d",
                ix->resident_clusters, cap);
  int32_t w = 0;
  for (int32_t c = 0; c < ix->sh.nlist && ix->has_dev; ++c)
    if (ix->h_map[c] >= 0) cluster_ids[w++] = c;
  return IVF_OK;
}

// ---------------------------------------------------------------------------
// migration (caller holds ix->mu for the *_locked helpers)
// ---------------------------------------------------------------------------
int publish_if_done_locked(ivf_index *ix, bool wait) {
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

// Starts the migration evict -> admit on side stream st (caller holds ix->mu, no
// migration is in flight).  partial: admitted clusters are placed in the order
// given and one that finds no free space is left out instead of failing the call;
// *n_placed (may be NULL) receives how many were placed.
static int migrate_locked(ivf_index *ix, const int32_t *evict, int32_t n_evict,
                          const int32_t *admit, int32_t n_admit, hipStream_t st, bool partial,
                          int32_t *n_placed) {
  int rc;
  std::vector<char> seen(ix->sh.nlist, 0);
  if ((rc = check_cluster_list(ix, evict, n_evict, "evict", seen)) != IVF_OK) return rc;
  if ((rc = check_cluster_list(ix, admit, n_admit, "admit", seen)) != IVF_OK) return rc;
  for (int32_t i = 0; i < n_evict; ++i)
    if (ix->h_map[evict[i]] < 0)
      return fail(IVF_EINVAL, "evict: cluster %d is not resident", evict[i]);
  for (int32_t i = 0; i < n_admit; ++i)
    if (ix->h_map[admit[i]] >= 0)
      return fail(IVF_EINVAL, "admit: cluster %d is already resident", admit[i]);

  reclaim(ix);
  const int target = (ix->versions.back().buf + 1) % 3;
  for (auto &v : ix->versions)
    if (v.buf == target)
      return fail(IVF_EBUSY, "searches on an old mapping table have not drained yet");

  // place admitted clusters in free space only
  std::vector<int32_t> clusters(admit, admit + n_admit);
  if (!partial) std::sort(clusters.begin(), clusters.end());
  std::vector<int64_t> bases(clusters.size());
  size_t placed = 0;
  int64_t need_tiles = 0;
  bool ok = true;
  for (size_t i = 0; i < clusters.size(); ++i) {
    const int64_t nt = tiles_of(ix->h_len[clusters[i]]);
    const int64_t s = ix->alloc.alloc(nt);
    if (s < 0) {
      if (partial) continue;  // stays cold; a later refresh finds the evicted space free
      ok = false;
      break;
    }
    clusters[placed] = clusters[i];
    bases[placed] = s;
    need_tiles += nt;
    ++placed;
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
  clusters.resize(placed);
  bases.resize(placed);
  if (partial) {  // the copies take the clusters in id order, like the caller's list above
    std::vector<size_t> by_id(placed);
    for (size_t i = 0; i < placed; ++i) by_id[i] = i;
    std::sort(by_id.begin(), by_id.end(),
              [&](size_t a, size_t b) { return clusters[a] < clusters[b]; });
    std::vector<int32_t> c2(placed);
    std::vector<int64_t> b2(placed);
    for (size_t i = 0; i < placed; ++i) {
      c2[i] = clusters[by_id[i]];
      b2[i] = bases[by_id[i]];
    }
    clusters.swap(c2);
    bases.swap(b2);
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
  if (n_placed) *n_placed = (int32_t)placed;
  return IVF_OK;
}

extern "C" int ivf_migrate_clusters(ivf_index_t *ix, const int32_t *evict, int32_t n_evict,
                                    const int32_t *admit, int32_t n_admit, void *side_stream) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (!ix->has_dev) return fail(IVF_EDEVICE, "host-only index: nothing to migrate");
  std::lock_guard<std::mutex> lk(ix->mu);
  int rc = publish_if_done_locked(ix, false);
  if (rc < 0) return rc;
  if (ix->mig.active) return fail(IVF_EBUSY, "a migration is already in flight");
  return migrate_locked(ix, evict, n_evict, admit, n_admit, (hipStream_t)side_stream,
                        /*partial=*/false, nullptr);
}

extern "C" int ivf_refresh_hot_set(ivf_index_t *ix, int32_t n_hot, int reset, void *side_stream,
                                   int32_t *n_evicted, int32_t *n_admitted, int32_t *n_deferred,
                                   double *mean_hit_rate) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (!ix->has_dev) return fail(IVF_EDEVICE, "host-only index: nothing to migrate");
  const int32_t nlist = ix->sh.nlist;
  if (n_hot < 0 || n_hot > nlist)
    return fail(IVF_EINVAL, "refresh: n_hot = %d, the index has %d clusters", n_hot, nlist);
  std::lock_guard<std::mutex> lk(ix->mu);
  int rc = publish_if_done_locked(ix, false);
  if (rc < 0) return rc;
  if (ix->mig.active) return fail(IVF_EBUSY, "a migration is already in flight");
  reclaim(ix);
  {
    const int target = (ix->versions.back().buf + 1) % 3;
    for (auto &v : ix->versions)
      if (v.buf == target)
        return fail(IVF_EBUSY, "searches on an old mapping table have not drained yet");
  }
  std::vector<uint64_t> hits((size_t)nlist);
  uint64_t counted = 0;
  {
    // without any search since the last reset the ranking below would be by id alone
    // and would throw the hot set away: look before the counters are cleared
    rc = read_counters_locked(ix, hits.data(), mean_hit_rate, nullptr, &counted, 0);
    if (rc != IVF_OK) return rc;
    if (counted == 0) return fail(IVF_ESTATE, "refresh: no search has been counted since the reset");
  }
  // the n_hot most accessed clusters, ties to the smaller id
  std::vector<int32_t> order;
  rank_clusters(hits, order);
  std::vector<char> want((size_t)nlist, 0);
  for (int32_t i = 0; i < n_hot; ++i) want[order[i]] = 1;
  std::vector<int32_t> evict, admit;
  for (int32_t c = 0; c < nlist; ++c)
    if (ix->h_map[c] >= 0 && !want[c]) evict.push_back(c);
  for (int32_t i = 0; i < n_hot; ++i)  // hottest first: they are placed first
    if (ix->h_map[order[i]] < 0) admit.push_back(order[i]);
  int32_t placed = 0;
  if (!evict.empty() || !admit.empty()) {
    rc = migrate_locked(ix, evict.data(), (int32_t)evict.size(), admit.data(),
                        (int32_t)admit.size(), (hipStream_t)side_stream, /*partial=*/true, &placed);
    if (rc != IVF_OK) return rc;
  }
  // (clears on the index's own stream: a device-wide wait would wait for the copies just started)
  if (reset && (rc = reset_counters_locked(ix)) != IVF_OK) return rc;
  if (n_evicted) *n_evicted = (int32_t)evict.size();
  if (n_admitted) *n_admitted = placed;
  if (n_deferred) *n_deferred = (int32_t)admit.size() - placed;
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

