// C ABI, part 1: errors, index lifetime and arena layout, tuning, stage
// timers, router counters, counter-calibration kernels.
#include "index_state.h"

// ---------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------
static thread_local std::string g_err;

int fail(int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

extern "C" const char *ivf_last_error(void) { return g_err.c_str(); }

HostIndexView host_view(const ivf_index *ix) {
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
  v.pv = ix->pv_host();
  v.pv_max = ix->pv_max;
  v.codebooks = ix->desc.codebooks;
  v.codebooks_t = ix->cb_t.data();
  v.list_offsets = ix->desc.list_offsets;
  v.codes = ix->desc.codes;
  v.ids = ix->desc.ids;
  v.codes_t = ix->codes_t.empty() ? nullptr : ix->codes_t.data();
  v.list_toff = ix->list_toff.empty() ? nullptr : ix->list_toff.data();
  return v;
}

extern "C" int ivf_host_scan_form(const ivf_index_t *ix) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  return ix->codes_t.empty() ? 0 : 1;
}

extern "C" int ivf_copy_form(const ivf_index_t *ix) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  return ix->zc_codes ? 1 : 0;
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
    w.sel_split = take(coarse_select_split_bytes());
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
    w.heavy = (int32_t *)take(nq * 4);
    w.hslot = (int32_t *)take(nq * 4);
    w.bias = (float *)take(nq * np * 4);
    w.g_bias = (float *)take(nq * np * 4);
    w.qbmax = (float *)take(nq * 4);
    w.part_key = (int32_t *)take((size_t)part_rows((int64_t)nq) * k * 4);
    w.part_id = (int64_t *)take((size_t)part_rows((int64_t)nq) * k * 8);
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
    for (auto e : ix->timing_pool) (void)hipEventDestroy(e);
    for (auto &r : ix->trecs)
      for (int i = 0; i <= IVF_N_STAGES; ++i)
        if (r.valid[i]) (void)hipEventDestroy(r.ev[i]);
    free_host_buffers(ix);
    if (ix->pv_pinned) (void)hipHostFree(ix->pv_pinned);
    if (ix->ev_routed) (void)hipEventDestroy(ix->ev_routed);
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
  ix->cb_t.resize((size_t)desc->d << desc->nbits);
  {
    HostIndexView v = host_view(ix);
    cpu_transpose_codebooks(v, ix->cb_t.data());
    if (cpu_has_plane_scan() && n_total > 0) {
      // column-major copy of the codes for the CPU's byte-plane scan of cold clusters
      ix->list_toff.resize((size_t)desc->nlist + 1);
      const int64_t bytes = cpu_transposed_bytes(v, ix->list_toff.data());
      if (!ix->codes_t.alloc((size_t)bytes)) {
        delete ix;
        return fail(IVF_ENOMEM, "no host memory for the column-major code copy (%lld bytes)",
                    (long long)bytes);
      }
      cpu_transpose_codes(v, ix->list_toff.data(), ix->codes_t.data());
    }
  }
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
  if (desc->nbits == 4 && desc->d > 2048) {
    delete ix;
    return fail(IVF_EINVAL, "4-bit codes on the device need d <= 2048 (got %d)", desc->d);
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
  if ((e = static_scratch_for_device(ix->device, &ix->static_scratch)) != hipSuccess)
    return bail(e, "hipGetSymbolAddress(scratch)");
  if ((e = hipStreamCreateWithFlags(&ix->own_stream, hipStreamNonBlocking)) != hipSuccess)
    return bail(e, "hipStreamCreateWithFlags");
  if ((e = hipEventCreateWithFlags(&ix->ev_routed, hipEventDisableTiming)) != hipSuccess)
    return bail(e, "hipEventCreateWithFlags");
  if (!ix->pv.empty()) {  // the per-vector term moves to pinned memory
    if ((e = pinned_alloc(&ix->pv_pinned, ix->pv.size())) != hipSuccess)
      return bail(e, "hipHostMalloc");
    memcpy(ix->pv_pinned, ix->pv.data(), ix->pv.size() * sizeof(float));
    std::vector<float>().swap(ix->pv);
  }
  // Pinned host arrays can be read by the copy kernel itself.  A pointer the
  // runtime does not know (pageable memory) is no error: such an index copies
  // through the staging area.  IVF_COPY_PATH=staged forces that path.
  const char *copy_path = getenv("IVF_COPY_PATH");
  if (n_total > 0 && n_total < 0x7fffffff && !(copy_path && !strcmp(copy_path, "staged"))) {
    void *dc = nullptr, *di = nullptr, *dp = nullptr;
    bool ok = hipHostGetDevicePointer(&dc, const_cast<uint8_t *>(desc->codes), 0) == hipSuccess &&
              hipHostGetDevicePointer(&di, const_cast<int64_t *>(desc->ids), 0) == hipSuccess &&
              dc && di && ((uintptr_t)dc & 15) == 0 && ((uintptr_t)di & 7) == 0;
    if (ok && ix->pv_pinned)
      ok = hipHostGetDevicePointer(&dp, ix->pv_pinned, 0) == hipSuccess && dp;
    if (ok) {
      ix->zc_codes = static_cast<const uint8_t *>(dc);
      ix->zc_ids = static_cast<const int64_t *>(di);
      ix->zc_pv = static_cast<const float *>(dp);
    } else {
      (void)hipGetLastError();
    }
  }
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
  // timed batches take their events from a pool; stock it here, outside any timed region
  while (timing && ix->has_dev && ix->timing_pool.size() < 1024) {
    hipEvent_t e = nullptr;
    HIP_TRY(hipEventCreate(&e));
    ix->timing_pool.push_back(e);
  }
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
      if (r.valid[i]) {
        if (ix->timing_pool.size() < 4096) ix->timing_pool.push_back(r.ev[i]);
        else (void)hipEventDestroy(r.ev[i]);
      }
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
// Clears the device's counters on the index's own stream and waits for that
// stream only (not for copies running on a migration's side stream).
int reset_counters_locked(ivf_index *ix) {
  hipStream_t st = ix->own_stream;
  HIP_TRY(launch_fill_u32((uint32_t *)ix->L.hits, (size_t)ix->sh.nlist * 2, 0u, st));
  HIP_TRY(launch_fill_u32((uint32_t *)ix->L.qstats, 4 * 2, 0u, st));
  HIP_TRY(launch_fill_u32((uint32_t *)&ix->L.qstats[QS_MIN_RATE_BITS], 1, 0x3f800000u, st));
  HIP_TRY(launch_fill_u32((uint32_t *)&ix->L.qstats[QS_RATE_SUM], 2 * 2, 0u, st));
  HIP_TRY(hipStreamSynchronize(st));
  return IVF_OK;
}

int read_counters_locked(ivf_index *ix, uint64_t *per_cluster_hits, double *mean_hit_rate,
                         double *min_hit_rate, uint64_t *n_queries, int reset) {
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
  if (reset) return reset_counters_locked(ix);
  return IVF_OK;
}

extern "C" int ivf_hit_stats(ivf_index_t *ix, uint64_t *per_cluster_hits, double *mean_hit_rate,
                             double *min_hit_rate, uint64_t *n_queries, int reset) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  std::lock_guard<std::mutex> lk(ix->mu);
  return read_counters_locked(ix, per_cluster_hits, mean_hit_rate, min_hit_rate, n_queries, reset);
}

extern "C" int ivf_hit_rate_moments(ivf_index_t *ix, double *mean, double *variance,
                                    double *sigma_max2, uint64_t *n_queries) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  std::lock_guard<std::mutex> lk(ix->mu);
  double m = 0.0, var = 0.0;
  uint64_t n = 0;
  if (ix->has_dev) {
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(ix->h_stats, ix->L.qstats, QS_COUNT * 8, hipMemcpyDeviceToHost));
    n = ix->h_stats[QS_QUERIES];
    if (n) {
      // the two sums are integers in units of 2^-32
      m = ldexp((double)ix->h_stats[QS_RATE_SUM], -32) / (double)n;
      var = std::max(0.0, ldexp((double)ix->h_stats[QS_RATE_SQ], -32) / (double)n - m * m);
    }
  } else {
    n = ix->hc_queries;  // nothing is resident: every hit rate is 0
  }
  if (mean) *mean = m;
  if (variance) *variance = var;
  if (sigma_max2) *sigma_max2 = (m > 0.0 && m < 1.0) ? var / (4.0 * m * (1.0 - m)) : NAN;
  if (n_queries) *n_queries = n;
  return IVF_OK;
}

extern "C" int ivf_weighted_hit_rate(ivf_index_t *ix, double *rate, double *probed_bytes) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  std::lock_guard<std::mutex> lk(ix->mu);
  const int32_t nlist = ix->sh.nlist;
  std::vector<uint64_t> hits((size_t)nlist);
  int rc = read_counters_locked(ix, hits.data(), nullptr, nullptr, nullptr, 0);
  if (rc != IVF_OK) return rc;
  // every probe of list c scans M * L_c bytes of codes, on the device if c is resident
  double all = 0.0, res = 0.0;
  for (int32_t c = 0; c < nlist; ++c) {
    const double b = (double)hits[c] * (double)ix->h_len[c] * (double)ix->sh.M;
    all += b;
    if (ix->h_map[c] >= 0) res += b;
  }
  if (rate) *rate = all > 0.0 ? res / all : 0.0;
  if (probed_bytes) *probed_bytes = all;
  return IVF_OK;
}

// Clusters from the most to the least accessed, equal counts by id.
void rank_clusters(const std::vector<uint64_t> &hits, std::vector<int32_t> &order) {
  order.resize(hits.size());
  for (size_t c = 0; c < hits.size(); ++c) order[c] = (int32_t)c;
  std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
    return hits[a] != hits[b] ? hits[a] > hits[b] : a < b;
  });
}

extern "C" int ivf_profile_curves(ivf_index_t *ix, int32_t *ranked, double *hit_cdf,
                                  double *mem_index) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  const int32_t nlist = ix->sh.nlist;
  std::vector<uint64_t> hits((size_t)nlist);
  {
    std::lock_guard<std::mutex> lk(ix->mu);
    int rc = read_counters_locked(ix, hits.data(), nullptr, nullptr, nullptr, 0);
    if (rc != IVF_OK) return rc;
  }
  uint64_t total = 0;
  for (uint64_t h : hits) total += h;
  if (total == 0) return fail(IVF_ESTATE, "profile: no probe has been counted since the reset");
  std::vector<int32_t> order;
  rank_clusters(hits, order);
  // what a resident vector costs on the device: its code, its id, and for residual
  // codes under L2 its per-vector term
  const double per_vec = (double)ix->sh.M + 8.0 + (ix->sh.by_residual && !ix->sh.metric_ip ? 4.0 : 0.0);
  uint64_t acc = 0;
  double bytes = 0.0;
  if (hit_cdf) hit_cdf[0] = 0.0;
  if (mem_index) mem_index[0] = 0.0;
  for (int32_t i = 0; i < nlist; ++i) {
    const int32_t c = order[i];
    acc += hits[c];
    bytes += per_vec * (double)ix->h_len[c];
    if (ranked) ranked[i] = c;
    if (hit_cdf) hit_cdf[i + 1] = i + 1 == nlist ? 1.0 : (double)acc / (double)total;
    if (mem_index) mem_index[i + 1] = bytes;
  }
  return IVF_OK;
}

extern "C" int ivf_calib_copy(const void *src, void *dst, size_t bytes, void *stream) {
  if (!src || !dst || bytes % 16 != 0) return fail(IVF_EINVAL, "calib copy: bad arguments");
  HIP_TRY(launch_calib_copy(src, dst, bytes, (hipStream_t)stream));
  return IVF_OK;
}

extern "C" int ivf_calib_read(const void *src, void *sink, size_t sink_bytes, size_t bytes,
                              void *stream) {
  if (!src || !sink || bytes % 16 != 0) return fail(IVF_EINVAL, "calib read: bad arguments");
  if (sink_bytes < IVF_CALIB_SINK_BYTES)
    return fail(IVF_EINVAL, "calib read: the sink holds %zu bytes, %zu are written", sink_bytes,
                IVF_CALIB_SINK_BYTES);
  HIP_TRY(launch_calib_read(src, sink, bytes, (hipStream_t)stream));
  return IVF_OK;
}

