// CPU side of the hybrid search: the library's own scan of non-resident
// ("cold") clusters (Section 4.3.1: the part of the search not held by the GPU
// is handled by the CPU) and the merge of CPU and GPU partial results
// (Section 4.3.2).  Uses the same fixed-point table arithmetic as the kernels,
// so a cluster yields bit-identical distances wherever it is scanned.
#pragma once
#include <stdint.h>

#include <functional>
#include <vector>

namespace ivf {

struct HostCand {
  int32_t key;
  int64_t id;
};

struct HostIndexView {
  int d, nlist, M, dsub, metric_ip;
  const float *codebooks;       // [M][256][dsub]
  const int64_t *list_offsets;  // [nlist+1]
  const uint8_t *codes;         // [N][M]
  const int64_t *ids;           // [N]
};

int cpu_threads();

// Run fn(i) for i in [0, n) on up to cpu_threads() threads.
void parallel_for(int64_t n, const std::function<void(int64_t)> &fn);

// Fixed-point table of one query: lut[m*256 + j]; returns the scale exponent.
int cpu_build_lut(const HostIndexView &ix, const float *q, int32_t *lut);

// Scan the listed clusters for one query; writes k candidates, best first,
// padded with (kKeyInvalid, -1).
void cpu_scan_lists(const HostIndexView &ix, const int32_t *lut, const int32_t *clusters,
                    int n_clusters, int k, HostCand *out);

// Merge two best-first lists of k candidates into the k best.
void merge_topk(const HostCand *a, const HostCand *b, int k, HostCand *out);

}  // namespace ivf
