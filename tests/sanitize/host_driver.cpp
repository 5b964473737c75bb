// Exercise of the library's host side through the C ABI, meant to be built with
// -fsanitize=address,undefined and with -fsanitize=thread (tests/test_host_sanitizers.py):
// device-less indexes of random small shapes, the CPU scan of every probed cluster on the
// library's worker threads, the dynamic dispatcher's threads (CPU search loop, completed
// queue, dispatcher, a polling caller), the router counters, the partitioning model and the
// argument errors.  Results are checked for what must hold whatever the sanitizer: the
// asynchronous call returns the bulk call's bytes, repeated calls return the same bytes,
// every query is handed on once.  Prints "host driver ok" and exits 0 on success.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <random>
#include <thread>
#include <vector>

#include "../../include/ivfpq_hot.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "%s:%d: CHECK failed: %s (last error: %s)\n", __FILE__, __LINE__, #cond, \
              ivf_last_error());                                           \
      exit(1);                                                             \
    }                                                                      \
  } while (0)

struct Index {
  int d, nlist, M, nbits, metric, residual;
  std::vector<float> centroids, codebooks;
  std::vector<int64_t> offsets, ids;
  std::vector<uint8_t> codes;
  ivf_index_t *h = nullptr;
};

static void make_index(Index &ix, std::mt19937 &rng) {
  std::normal_distribution<float> nd(0.f, 1.f);
  const int ksub = 1 << ix.nbits;
  ix.centroids.resize((size_t)ix.nlist * ix.d);
  ix.codebooks.resize((size_t)ix.M * ksub * (ix.d / ix.M));
  for (auto &x : ix.centroids) x = nd(rng);
  for (auto &x : ix.codebooks) x = 0.3f * nd(rng);
  ix.offsets.assign(1, 0);
  for (int c = 0; c < ix.nlist; ++c) {
    // empty lists, lists shorter than one 64-vector group, and lists longer than one
    // pass of the byte-plane scan
    const int pick = (int)(rng() % 8);
    const int len = pick == 0 ? 0 : (pick == 1 ? 2500 : (int)(rng() % 200));
    ix.offsets.push_back(ix.offsets.back() + len);
  }
  const int64_t n = ix.offsets.back();
  const int cb = ix.M * ix.nbits / 8;
  ix.codes.resize((size_t)n * cb);
  for (auto &x : ix.codes) x = (uint8_t)rng();
  ix.ids.resize((size_t)n);
  for (int64_t i = 0; i < n; ++i) ix.ids[(size_t)i] = (n - i) * 3 + 1;
  ivf_index_desc_t desc;
  memset(&desc, 0, sizeof(desc));
  desc.d = ix.d;
  desc.nlist = ix.nlist;
  desc.M = ix.M;
  desc.nbits = ix.nbits;
  desc.metric = ix.metric;
  desc.max_nq = 64;
  desc.max_nprobe = 64;
  desc.max_k = 128;
  desc.by_residual = ix.residual;
  desc.centroids = ix.centroids.data();
  desc.codebooks = ix.codebooks.data();
  desc.list_offsets = ix.offsets.data();
  desc.codes = ix.codes.data();
  desc.ids = ix.ids.data();
  CHECK(ivf_index_create(&desc, nullptr, 0, 0, &ix.h) == IVF_OK);
}

struct Seen {
  std::atomic<int> calls{0};
  std::vector<std::atomic<int>> per_query;
  explicit Seen(int nq) : per_query(nq) {
    for (auto &x : per_query) x = 0;
  }
};

static void on_done(void *user, int64_t q, const int64_t *ids, const float *dists, int32_t k) {
  Seen *s = static_cast<Seen *>(user);
  // the row is final when the callback runs: read all of it
  long long acc = 0;
  for (int r = 0; r < k; ++r) acc += ids[r] + (long long)(dists[r] == dists[r]);
  (void)acc;
  s->per_query[(size_t)q].fetch_add(1);
  s->calls.fetch_add(1);
}

static void run_case(int M, int nbits, int dsub, int metric, int residual, unsigned seed) {
  std::mt19937 rng(seed);
  Index ix;
  ix.M = M;
  ix.nbits = nbits;
  ix.d = M * dsub;
  ix.nlist = 37;
  ix.metric = metric;
  ix.residual = residual;
  make_index(ix, rng);
  std::normal_distribution<float> nd(0.f, 1.f);
  for (int round = 0; round < 3; ++round) {
    const int nq = round == 0 ? 1 : (round == 1 ? 33 : 64);
    const int nprobe = round == 0 ? 37 : 9;
    const int k = round == 2 ? 100 : 10;
    std::vector<float> q((size_t)nq * ix.d);
    for (auto &x : q) x = nd(rng);
    std::vector<int32_t> probe((size_t)nq * nprobe);
    for (int i = 0; i < nq; ++i) {
      std::vector<int32_t> perm(ix.nlist);
      for (int c = 0; c < ix.nlist; ++c) perm[c] = c;
      std::shuffle(perm.begin(), perm.end(), rng);
      for (int p = 0; p < nprobe; ++p)
        probe[(size_t)i * nprobe + p] = (rng() % 11 == 0) ? -1 : perm[p];  // -1: no probe
    }
    std::vector<int64_t> ids((size_t)nq * k), ids2(ids.size()), ids3(ids.size());
    std::vector<float> dist((size_t)nq * k), dist2(dist.size()), dist3(dist.size());
    CHECK(ivf_search_batch_probes(ix.h, q.data(), nq, probe.data(), nprobe, k, ids.data(),
                                  dist.data()) == IVF_OK);
    CHECK(ivf_search_batch_probes(ix.h, q.data(), nq, probe.data(), nprobe, k, ids2.data(),
                                  dist2.data()) == IVF_OK);
    CHECK(ids == ids2 && !memcmp(dist.data(), dist2.data(), dist.size() * 4));
    for (int i = 0; i < nq; ++i)  // best first
      for (int r = 1; r < k; ++r) {
        const float a = dist[(size_t)i * k + r - 1], b = dist[(size_t)i * k + r];
        if (ids[(size_t)i * k + r] >= 0) CHECK(metric == IVF_METRIC_IP ? a >= b : a <= b);
      }
    // the dispatcher: a polling caller beside the library's own threads
    for (int rep = 0; rep < 4; ++rep) {
      Seen seen(nq);
      ivf_ticket_t *t = nullptr;
      CHECK(ivf_search_batch_async(ix.h, q.data(), nq, probe.data(), nprobe, k, ids3.data(),
                                   dist3.data(), rep % 2 ? on_done : nullptr, &seen, &t) == IVF_OK);
      // a second search while the first is in flight is refused
      CHECK(ivf_search_batch_probes(ix.h, q.data(), nq, probe.data(), nprobe, k, ids2.data(),
                                    dist2.data()) == IVF_EBUSY);
      std::vector<int64_t> got(16);
      std::vector<int> polled((size_t)nq, 0);
      int32_t fin = 0;
      while (!fin) {
        int64_t n = 0;
        CHECK(ivf_search_poll(t, got.data(), (int64_t)got.size(), &n, &fin) >= 0);
        for (int64_t i = 0; i < n; ++i) polled[(size_t)got[(size_t)i]] += 1;
        if (!n && !fin) std::this_thread::yield();
      }
      std::vector<double> done_ms((size_t)nq);
      CHECK(ivf_search_wait(t, done_ms.data()) == IVF_OK);
      for (int i = 0; i < nq; ++i) CHECK(polled[(size_t)i] == 1 && done_ms[(size_t)i] >= 0.0);
      if (rep % 2) {
        CHECK(seen.calls.load() == nq);
        for (int i = 0; i < nq; ++i) CHECK(seen.per_query[(size_t)i].load() == 1);
      }
      CHECK(ids == ids3 && !memcmp(dist.data(), dist3.data(), dist.size() * 4));
    }
  }
  // router counters of a device-less index
  std::vector<uint64_t> hits((size_t)ix.nlist);
  uint64_t nqs = 0;
  double mean = -1, mn = -1;
  {
    // the access profile from those counters: a permutation of the ids, curves that rise to
    // the whole (read before the counters are cleared below)
    std::vector<int32_t> ranked((size_t)ix.nlist);
    std::vector<double> cdf((size_t)ix.nlist + 1), mem((size_t)ix.nlist + 1);
    CHECK(ivf_profile_curves(ix.h, ranked.data(), cdf.data(), mem.data()) == IVF_OK);
    std::vector<char> seen_id((size_t)ix.nlist, 0);
    for (int32_t c : ranked) {
      CHECK(c >= 0 && c < ix.nlist && !seen_id[(size_t)c]);
      seen_id[(size_t)c] = 1;
    }
    CHECK(cdf[0] == 0.0 && cdf[(size_t)ix.nlist] == 1.0 && mem[0] == 0.0);
    for (int i = 0; i < ix.nlist; ++i) CHECK(cdf[(size_t)i + 1] >= cdf[(size_t)i] && mem[(size_t)i + 1] >= mem[(size_t)i]);
    double rm = -1, rv = -1, rs2 = 0;
    uint64_t rn = 0;
    CHECK(ivf_hit_rate_moments(ix.h, &rm, &rv, &rs2, &rn) == IVF_OK);
    CHECK(rn > 0 && rm == 0.0 && rv == 0.0 && rs2 != rs2);  // nothing resident: no spread, no model
    double wr = -1, wb = -1;
    CHECK(ivf_weighted_hit_rate(ix.h, &wr, &wb) == IVF_OK && wr == 0.0 && wb > 0.0);
    int32_t nres = -1;
    CHECK(ivf_resident_list(ix.h, nullptr, 0, &nres) == IVF_OK && nres == 0);
    CHECK(ivf_refresh_hot_set(ix.h, 1, 0, nullptr, nullptr, nullptr, nullptr, nullptr) == IVF_EDEVICE);
  }
  CHECK(ivf_hit_stats(ix.h, hits.data(), &mean, &mn, &nqs, 1) == IVF_OK);
  CHECK(nqs > 0 && mean == 0.0);
  CHECK(ivf_profile_curves(ix.h, nullptr, nullptr, nullptr) == IVF_ESTATE);
  CHECK(ivf_hit_stats(ix.h, hits.data(), nullptr, nullptr, &nqs, 0) == IVF_OK && nqs == 0);
  // what needs the device says so
  std::vector<int64_t> oi(10);
  std::vector<float> od(10), q1((size_t)ix.d, 0.5f);
  CHECK(ivf_search_batch(ix.h, q1.data(), 1, 4, 10, oi.data(), od.data()) == IVF_EDEVICE);
  CHECK(ivf_index_load_partition(ix.h, nullptr, 0, nullptr) == IVF_EDEVICE);
  int32_t twice[2] = {3, 3};
  CHECK(ivf_search_batch_probes(ix.h, q1.data(), 1, twice, 2, 10, oi.data(), od.data()) ==
        IVF_EINVAL);
  CHECK(ivf_host_scan_form(ix.h) >= 0);
  ivf_index_destroy(ix.h);
}

static void partition_model() {
  const double kb[4] = {1, 4, 16, 64}, cq[4] = {1e-3, 1.5e-3, 3e-3, 9e-3},
               lut[4] = {4e-3, 6e-3, 14e-3, 50e-3};
  ivf_latency_model_t m = {4, kb, cq, lut};
  const int nlist = 32;
  std::vector<double> cdf(nlist + 1), mem(nlist + 1);
  double h = 0;
  for (int i = 1; i <= nlist; ++i) h += 1.0 / i;
  cdf[0] = mem[0] = 0;
  for (int i = 1; i <= nlist; ++i) {
    cdf[(size_t)i] = cdf[(size_t)i - 1] + 1.0 / i / h;
    mem[(size_t)i] = mem[(size_t)i - 1] + 5e4;
  }
  cdf[nlist] = 1.0;
  CHECK(fabs(ivf_model_min_hit_rate(0.5, 1.0 / 12.0, 3) - 0.25) < 1e-6);
  CHECK(ivf_model_hybrid_latency(&m, 4, 1.0) == 1.5e-3);
  const double c = ivf_model_hitrate_to_coverage(cdf.data(), nlist, 0.02, 8, 0.4);
  CHECK(c > 0.0 && c <= 1.0);
  double rho = -1;
  CHECK(ivf_model_partition_point(&m, cdf.data(), mem.data(), nlist, 0.02, 20e-3, 1.0,
                                  4 * mem[nlist], 900.0, 1.0 / 64, &rho) == IVF_OK);
  CHECK(rho >= 0.0 && rho <= 1.0);
  CHECK(ivf_model_partition_point(&m, cdf.data(), mem.data(), nlist, 0.3, 20e-3, 1.0, 1.0, 1.0,
                                  0.1, &rho) == IVF_EINVAL);
}

int main() {
  unsigned seed = 1;
  run_case(16, 8, 4, IVF_METRIC_L2, 0, seed++);
  run_case(48, 8, 2, IVF_METRIC_IP, 1, seed++);
  run_case(128, 8, 1, IVF_METRIC_L2, 1, seed++);
  run_case(64, 4, 3, IVF_METRIC_IP, 0, seed++);
  run_case(192, 4, 1, IVF_METRIC_L2, 1, seed++);
  partition_model();
  CHECK(ivf_index_arena_bytes(nullptr, 0, 0) == 0);
  printf("host driver ok\n");
  return 0;
}
