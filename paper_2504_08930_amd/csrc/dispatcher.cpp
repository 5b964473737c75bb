// C ABI, part 4: the dynamic dispatcher.
#include "index_state.h"

// ---------------------------------------------------------------------------
// dynamic dispatcher (Section 4.2.2): per-query completion of a hybrid batch
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

  std::vector<std::thread> workers;  // only if the worker pool is taken
  bool pooled = false;
  std::atomic<int64_t> next(0);
  // set once the device's partial results are on the host: queries the CPU loop starts
  // after that scan with the device's k-th best key as their bound
  std::atomic<int> gpu_ready(0);
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
          int32_t cap = kKeyInvalid;
          if (t->device && t->any_resident && gpu_ready.load(std::memory_order_acquire))
            cap = device_key_cap(ix, view, q, k, e);
          cpu_scan_lists(view, lut.data(), e, qv, pr, nc, k, &t->cpu_res[(size_t)q * k],
                         &t->scanned[q], cap);
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
    pooled = WorkerPool::get().start(nt, work);
    if (!pooled)
      for (int i = 0; i < nt; ++i) workers.emplace_back(work);
  }

  // the GPU's completion flag: its partial results are on the host
  if (t->device && gpu_ok) {
    hipError_t e = hipEventSynchronize(t->ev_gpu);
    if (e != hipSuccess) {
      ticket_fail(t, IVF_EDEVICE, std::string("device scan failed: ") + hipGetErrorString(e));
      gpu_ok = false;
    } else {
      gpu_ready.store(1, std::memory_order_release);
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
  if (pooled) WorkerPool::get().wait();
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

