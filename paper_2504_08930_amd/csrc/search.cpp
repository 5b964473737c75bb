// C ABI, part 3: the search driver.  Strings the kernels together on the
// caller's stream, runs the CPU scan of cold probes and merges (bulk path).
#include "index_state.h"

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

// How a batch's scan is cut into blocks: every query into `slices` blocks, the `extra`
// queries with the most resident vectors into one more.
struct ScanCut {
  int slices;
  int extra;
};

static ScanCut pick_slices(const ivf_index *ix, const BatchCtx &c, int64_t nq, int nprobe, int k) {
  // the workspace holds part_rows(max_nq) partial results of a launch
  const int room = (int)std::min<int64_t>(std::min<int64_t>(kMaxSlices, kMaxMergeCand / k),
                                          part_rows(ix->desc.max_nq) / nq);
  if (ix->tune_slices > 0) return ScanCut{std::min(ix->tune_slices, std::max(room, 1)), 0};
  // One block per query fills the chip's 256 compute units (each holding one or two
  // scan blocks) from that many queries up.  Smaller batches are split; the number of
  // blocks per query is the one a small cost model likes best (in units of one tile's
  // streaming time): a launch of N blocks takes about r rounds of the chip, r between
  // N / fill and its ceiling (blocks are handed out as units come free, and a part-full
  // last round runs faster than a full one), each round streams a block's tiles, and
  // every block costs a fixed overhead on top (it stages the query's table again and
  // ends with its own selection: about 8 us, forty tiles' worth; twice that for long
  // result lists).  Never so many that a block's wavefronts get fewer than two tiles each.
  // A cut that leaves the last round part-full can be topped up: the queries with the
  // most vectors get one block more, as many of them as it takes to fill the round,
  // which also evens out the blocks' lengths (the model then takes a block's tiles as
  // the batch's tiles over its blocks).
  const int per_cu = scan_blocks_per_cu(ix->sh.M, k);
  const int fill_i = 256 * per_cu;
  const double fill = (double)fill_i;
  if ((double)nq > 1.25 * fill) return ScanCut{1, 0};
  const int waves = per_cu == 2 ? 8 : 16;
  const double tiles = (double)nprobe * c.list_tiles;  // estimate per query
  const double overhead = k <= 48 ? 40.0 : 80.0;
  const int s_max = (int)std::min<double>(room, std::max(1.0, tiles / (2 * waves)));
  ScanCut best{1, 0};
  double best_cost = 0.0;
  for (int s = 1; s <= s_max; ++s) {
    const double r = (double)nq * s / fill;
    const double rounds = r <= 1.0 ? 1.0 : 0.5 * (r + ceil(r));
    const double cost = rounds * (tiles / s) + ceil(r) * overhead;
    if (s == 1 || cost < best_cost) {
      best = ScanCut{s, 0};
      best_cost = cost;
    }
    const int64_t units = nq * s;
    const int extra = (int)((fill_i - units % fill_i) % fill_i);
    if (extra > 0 && extra <= nq && (int64_t)(s + 1) * k <= kMaxMergeCand &&
        s + 1 <= kMaxSlices && units + extra <= part_rows(ix->desc.max_nq)) {
      const double full_rounds = (double)(units + extra) / fill;  // whole rounds, even blocks
      const double cost_x = full_rounds * (tiles * (double)nq / (double)(units + extra)) +
                            full_rounds * overhead;
      if (cost_x < best_cost) {
        best = ScanCut{s, extra};
        best_cost = cost_x;
      }
    }
  }
  return best;
}

// Search on a device-less index: every probe is scanned on the CPU.
static int search_host_only(ivf_index *ix, const float *queries, int64_t nq, const int32_t *probe,
                            int nprobe, int k, int64_t *out_ids, float *out_dists) {
  const HostIndexView view = host_view(ix);
  std::vector<int64_t> ids((size_t)nq * k);
  std::vector<float> dists((size_t)nq * k);
  parallel_for(nq, [&](int64_t q) {
    thread_local std::vector<int32_t> lut;  // every entry is written before it is read
    thread_local std::vector<HostCand> cand;
    lut.resize((size_t)view.M * 256);
    cand.resize((size_t)k);
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

// True if p lies in pinned host memory that the runtime knows: a copy from or to it
// is a DMA transfer that runs asynchronously at the bus rate.  Anything else
// (pageable memory) the runtime would stage by itself, synchronously and slowly.
static bool host_ptr_pinned(const void *p) {
  hipPointerAttribute_t at;
  memset(&at, 0, sizeof(at));
  if (hipPointerGetAttributes(&at, p) != hipSuccess) {
    (void)hipGetLastError();  // an unknown pointer is no error here
    return false;
  }
  return at.type == hipMemoryTypeHost;
}

// Copy n bytes of pageable host memory into one of the index's pinned buffers on
// the library's worker threads (one thread moves about 10 GB/s; a batch of 1024
// queries is 3 MB).
static void staged_copy(void *dst, const void *src, size_t n) {
  constexpr size_t kChunk = (size_t)256 << 10;
  if (n <= 2 * kChunk) {
    memcpy(dst, src, n);
    return;
  }
  const int64_t chunks = (int64_t)((n + kChunk - 1) / kChunk);
  parallel_for(chunks, [&](int64_t i) {
    const size_t off = (size_t)i * kChunk;
    memcpy((char *)dst + off, (const char *)src + off, std::min(kChunk, n - off));
  });
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


int begin_batch(ivf_index *ix, hipStream_t st, BatchCtx *c) {
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
  c->list_tiles = ix->resident_clusters > 0
                      ? (int)std::max<int64_t>(1, (ix->resident_vectors / ix->resident_clusters + kTileVecs - 1) / kTileVecs)
                      : 1;
  // events of timed batches are kept until ivf_stage_times() reads them; a caller
  // that never does stops collecting after this many batches instead of growing
  c->timing = ix->trecs.size() < 8192 ? ix->timing : 0;
  return IVF_OK;
}

// Drop the hold on the mapping-table version.  async_tail: device work that
// reads the table may still be queued on st, so leave an event behind.
void end_batch(ivf_index *ix, const BatchCtx &c, hipStream_t st, bool async_tail) {
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
int enqueue_gpu(ivf_index *ix, const SearchArgs &a, const BatchCtx &c, bool final_on_gpu,
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
    // events come from a pool that ivf_stage_times() refills: in steady state a timed
    // batch creates none
    {
      std::lock_guard<std::mutex> lk(ix->mu);
      if (!ix->timing_pool.empty()) {
        trec.ev[i] = ix->timing_pool.back();
        ix->timing_pool.pop_back();
        trec.valid[i] = true;
      }
    }
    if (!trec.valid[i]) {
      hipError_t e = hipEventCreate(&trec.ev[i]);
      if (e != hipSuccess) return e;
      trec.valid[i] = true;
    }
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
    // pinned caller memory goes over the bus as it is; pageable memory is first
    // gathered in the index's pinned buffer (the host-pointer calls are synchronous
    // and the asynchronous one holds the index, so that buffer is free)
    const float *src = a.q_host;
    if (!host_ptr_pinned(src)) {
      staged_copy(ix->h_queries, src, (size_t)nq * sh.d * 4);
      src = ix->h_queries;
    }
    G_TRY(hipMemcpyAsync(W.queries, src, (size_t)nq * sh.d * 4, hipMemcpyHostToDevice, st));
    dq = W.queries;
  }
  // ---- stage 2 first: the lookup tables depend on the queries only ----
  G_TRY(mark(IVF_STAGE_LUT));
  int lut_parts = 0;
  // ... and so does the fp16 split of the queries for the coarse GEMM: one launch
  const bool split_with_lut = c.any_resident && !a.probe_host;
  if (c.any_resident)
    G_TRY(launch_lut(sh, dq, nq, L.cbT, W.lut, W.lutpart, &lut_parts,
                     split_with_lut ? W.q_parts : nullptr, W.q_exp, st));
  // ---- stage 1: coarse quantizer (or the caller's probe list) ----
  G_TRY(mark(IVF_STAGE_COARSE_GEMM));
  if (a.probe_host) {
    memcpy(ix->h_probe, a.probe_host, (size_t)nq * np * 4);
    G_TRY(hipMemcpyAsync(W.probe, ix->h_probe, (size_t)nq * np * 4, hipMemcpyHostToDevice, st));
    G_TRY(mark(IVF_STAGE_COARSE_SELECT));
  } else {
    if (!split_with_lut) G_TRY(launch_split_f16(dq, (size_t)nq, sh.d, W.q_parts, W.q_exp, st));
    G_TRY(launch_coarse_gemm(sh, W.q_parts, W.q_exp, nq, L.cent_parts, L.cent_exp, L.cent_norm,
                             W.scores, st));
    G_TRY(mark(IVF_STAGE_COARSE_SELECT));
    G_TRY(launch_coarse_select(sh, W.scores, nq, np, np, W.probe, W.sel_split, /*ordered=*/0, st));
  }
  // ---- routing ----
  G_TRY(mark(IVF_STAGE_ROUTE));
  if (sh.by_residual)
    G_TRY(launch_bias(sh, dq, nq, W.probe, np, np, L.centroids, W.bias, st));
  G_TRY(launch_route(W.probe, nq, np, np, sh.nlist, L.clus_tile[c.buf], L.clus_len, sh.M, W.g_base, W.g_len,
                     W.g_prefix, W.g_n, W.cold, W.n_cold, W.q_vecs,
                     sh.by_residual ? W.bias : nullptr, W.g_bias, W.qbmax, L.hits, 1, W.lutpart,
                     lut_parts, W.lutmax, st));
  const ScanCut cut = c.any_resident ? pick_slices(ix, c, nq, np, k) : ScanCut{1, 0};
  G_TRY(launch_order(W, nq, np, sh.M, L.qstats, 1, cut.extra, st));
  if (!final_on_gpu) {
    // cold probes go to the CPU (Section 4.2.1)
    G_TRY(hipMemcpyAsync(ix->h_ncold, W.n_cold, (size_t)nq * 4, hipMemcpyDeviceToHost, st));
    G_TRY(hipMemcpyAsync(ix->h_cold, W.cold, (size_t)nq * np * 4, hipMemcpyDeviceToHost, st));
    G_TRY(hipMemcpyAsync(ix->h_qbmax, W.qbmax, (size_t)nq * 4, hipMemcpyDeviceToHost, st));
    if (!a.q_host)
      G_TRY(hipMemcpyAsync(ix->h_queries, dq, (size_t)nq * sh.d * 4, hipMemcpyDeviceToHost, st));
    if (ev_route) G_TRY(hipEventRecord(ev_route, st));
  }
  if (c.any_resident) {
    // ---- stage 3: scan + top-k ----
    int64_t *oid = nullptr;
    float *od = nullptr;
    if (final_on_gpu) {
      oid = a.out_device ? a.out_ids : W.out_ids;
      od = a.out_device ? a.out_dists : W.out_dists;
    }
    G_TRY(mark(IVF_STAGE_SCAN));
    G_TRY(launch_scan(sh, L, W, nq, np, cut.slices, cut.extra, k, oid, od, st));
    G_TRY(mark(IVF_STAGE_MERGE));
    if (cut.slices > 1 || cut.extra > 0)
      G_TRY(launch_merge(sh, W, nq, cut.slices, cut.extra, k, oid, od, st));
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
bool finish_query(const ivf_index *ix, const HostIndexView &view, bool any_resident,
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

// The k-th best key of the device's partial result for query q (on the host once
// the batch's stream has drained), if the device found k candidates and quantized
// with the exponent e the CPU scan uses; kKeyInvalid otherwise.  The resident and the
// cold lists are disjoint, so a vector of a cold list with a larger key cannot be
// among the k best of both.
int32_t device_key_cap(const ivf_index *ix, const HostIndexView &view, int64_t q, int k, int e) {
  const int32_t kth = ix->h_reskey[q * k + (k - 1)];
  if (kth == kKeyInvalid) return kKeyInvalid;
  float mx;
  memcpy(&mx, &ix->h_lutmax[q], 4);
  const int e_dev = lut_exponent(mx, view.M, ix->h_qbmax[q], view.pv ? view.pv_max : 0.0f);
  return e_dev == e ? kth : kKeyInvalid;
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
  // Host results of a fully resident batch: when the caller's buffers are pinned host
  // memory that the device can address, the last kernel writes ids and distances into
  // them itself (120 KB at nq = 1024, k = 10) and no copy follows; the stream
  // synchronization below makes them visible to the host.
  SearchArgs dev_args = a;
  bool zero_copy_out = false;
  if (final_on_gpu && !a.out_device && host_ptr_pinned(a.out_ids) && host_ptr_pinned(a.out_dists)) {
    void *di = nullptr, *dd = nullptr;
    if (hipHostGetDevicePointer(&di, a.out_ids, 0) == hipSuccess &&
        hipHostGetDevicePointer(&dd, a.out_dists, 0) == hipSuccess && di && dd) {
      dev_args.out_ids = static_cast<int64_t *>(di);
      dev_args.out_dists = static_cast<float *>(dd);
      dev_args.out_device = true;
      zero_copy_out = true;
    } else {
      (void)hipGetLastError();
    }
  }
  rc = enqueue_gpu(ix, dev_args, ctx, final_on_gpu, final_on_gpu ? nullptr : ix->ev_routed);
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
    if (zero_copy_out) {
      S_TRY(hipStreamSynchronize(st));
      end_batch(ix, ctx, st, false);
      return IVF_OK;
    }
    // pageable results: one pair of copies into the index's pinned buffers, then out
    S_TRY(hipMemcpyAsync(ix->h_outids, W.out_ids, (size_t)nq * k * 8, hipMemcpyDeviceToHost, st));
    S_TRY(hipMemcpyAsync(ix->h_outd, W.out_dists, (size_t)nq * k * 4, hipMemcpyDeviceToHost, st));
    S_TRY(hipStreamSynchronize(st));
    end_batch(ix, ctx, st, false);
    memcpy(a.out_ids, ix->h_outids, (size_t)nq * k * 8);
    memcpy(a.out_dists, ix->h_outd, (size_t)nq * k * 4);
    return IVF_OK;
  }

  // ---- hybrid: cold probes on the CPU, then merge (Sections 4.2.1, 4.2.2) ----
  // The cold probe lists reach the host right after routing; the CPU scans them
  // while the device scans the resident ones.
  S_TRY(hipEventSynchronize(ix->ev_routed));
  const float *hq = a.q_host ? a.q_host : ix->h_queries;

  const HostIndexView view = host_view(ix);
  std::vector<HostCand> cpu_res((size_t)nq * k);
  std::vector<int> cpu_e((size_t)nq, 0);
  // The calling thread first waits for the device (a fraction of a millisecond; the
  // other threads are already scanning) and then joins them.  From then on a query's
  // CPU scan starts with the k-th best key of the device's partial result as its
  // bound: the resident lists are the query's nearest, so hardly any vector of a
  // cold list gets past the filter pass.
  std::atomic<int> gpu_ready(0);
  hipError_t sync_err = hipSuccess;
  const std::function<void()> wait_gpu = [&]() {
    sync_err = hipStreamSynchronize(st);  // the device's partial results are on the host
    if (sync_err == hipSuccess) gpu_ready.store(1, std::memory_order_release);
  };
  // two queries per work item: their tables are built together (the codebooks are read
  // once for both), then each is scanned
  parallel_for((nq + 1) / 2, [&](int64_t item) {
    thread_local std::vector<int32_t> lut;
    lut.resize((size_t)view.M * 512);
    int64_t qs[2];
    int n_act = 0;
    for (int64_t q = 2 * item; q < std::min<int64_t>(nq, 2 * item + 2); ++q)
      if (ix->h_ncold[q] > 0 || !any_resident) qs[n_act++] = q;
    if (n_act == 0) return;
    int32_t *luts[2] = {lut.data(), lut.data() + (size_t)view.M * 256};
    int es[2] = {0, 0};
    cpu_build_lut_pair(view, hq + (size_t)qs[0] * view.d,
                       n_act == 2 ? hq + (size_t)qs[1] * view.d : nullptr, ix->h_qbmax[qs[0]],
                       n_act == 2 ? ix->h_qbmax[qs[1]] : 0.0f, luts[0], luts[1], &es[0], &es[1]);
    for (int a = 0; a < n_act; ++a) {
      const int64_t q = qs[a];
      const int e = es[a];
      cpu_e[(size_t)q] = e;
      int32_t cap = kKeyInvalid;
      if (any_resident && gpu_ready.load(std::memory_order_acquire))
        cap = device_key_cap(ix, view, q, k, e);
      cpu_scan_lists(view, luts[a], e, hq + (size_t)q * view.d, ix->h_cold + (size_t)q * np,
                     ix->h_ncold[q], k, &cpu_res[(size_t)q * k], nullptr, cap);
    }
  }, &wait_gpu);
  S_TRY(sync_err);
  end_batch(ix, ctx, st, false);
  std::vector<int> bad(1, 0);
  parallel_for(nq, [&](int64_t q) {
    const bool has_cpu = ix->h_ncold[q] > 0 || !any_resident;
    if (!finish_query(ix, view, any_resident, q, k, has_cpu ? &cpu_res[(size_t)q * k] : nullptr,
                      cpu_e[(size_t)q], &ix->h_outids[(size_t)q * k], &ix->h_outd[(size_t)q * k]))
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

int check_search_args(const ivf_index *ix, const void *queries, int64_t nq, int32_t nprobe,
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
int check_probe_list(const ivf_index *ix, const int32_t *probe, int64_t nq, int nprobe) {
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
  HIP_TRY(launch_coarse_select(ix->sh, W.scores, (int)nq, nprobe, nprobe, out_probe, W.sel_split,
                               /*ordered=*/1, st));
  return IVF_OK;
}

extern "C" int ivf_coarse_probe_dev_noalloc(ivf_index_t *ix, const float *queries, int64_t nq,
                                            int32_t nprobe, int32_t *out_probe, void *stream) {
  if (!ix) return fail(IVF_EINVAL, "index is NULL");
  if (!ix->has_dev) return fail(IVF_EDEVICE, "host-only index: no device coarse quantizer");
  if (nq < 0 || nprobe < 1) return fail(IVF_EINVAL, "bad nq / nprobe");
  if (nq == 0) return IVF_OK;
  if (!queries || !out_probe) return fail(IVF_EINVAL, "NULL buffer");
  if (nprobe > kMaxNprobe) return fail(IVF_EINVAL, "nprobe exceeds %d", kMaxNprobe);
  if (nq > 0x7fffffff || coarse_static_bytes(ix->sh, nq) > kStaticScratchBytes)
    return fail(IVF_EINVAL,
                "nq = %lld needs %zu bytes of the library's static scratch array, which holds "
                "%zu (nq * (nlist + d) * 4 bytes, about): use a smaller batch or "
                "ivf_coarse_probe_dev",
                (long long)nq, nq > 0x7fffffff ? (size_t)0 : coarse_static_bytes(ix->sh, nq),
                kStaticScratchBytes);
  // no workspace slot, no lock, no event: the kernels' intermediates go to the
  // file-scope device array whose address ivf_index_create looked up
  HIP_TRY(launch_coarse_probe_static(ix->sh, queries, (int)nq, nprobe, ix->L.cent_parts,
                                     ix->L.cent_exp, ix->L.cent_norm, ix->static_scratch,
                                     out_probe, (hipStream_t)stream));
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
  if (!ix->has_dev) {
    {
      std::lock_guard<std::mutex> lk(ix->mu);
      if (ix->dispatch_active)
        return fail(IVF_EBUSY, "an asynchronous batch is still in flight on this index");
    }
    return search_host_only(ix, queries, nq, probe, nprobe, k, out_ids, out_dists);
  }
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

