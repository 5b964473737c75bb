// CPU side of the hybrid search: the library's own scan of non-resident
// ("cold") clusters (Section 4.2.1: the part of the search not held by the GPU
// is handled by the CPU) and the merge of CPU and GPU partial results
// (Section 4.2.2).  Uses the same fixed-point table arithmetic as the kernels,
// so a cluster yields bit-identical distances wherever it is scanned.
#pragma once
#include <stdint.h>

#include <functional>
#include <vector>

#include "lut_quant.h"

namespace ivf {

struct HostCand {
  int32_t key;
  int64_t id;
};

struct HostIndexView {
  int d, nlist;
  int M;                        // bytes per stored code = columns of the lookup table
  int dsub, metric_ip;
  int nbits = 8;                // bits per code (8, or 4: two codes per byte)
  int msub = 0;                 // sub-quantizers (= M for 8-bit codes, 2 M for 4-bit)
  int by_residual;              // codes encode x - centroid of the list
  const float *centroids;       // [nlist][d] (residual encoding only)
  const float *pv;              // [N] per-vector term (residual-encoded L2 only), else NULL
  float pv_max;                 // largest |pv|
  const float *codebooks;       // [msub][2^nbits][dsub]
  const float *codebooks_t;     // [msub][dsub][2^nbits]: the same, element-major (cpu_transpose_codebooks)
  const int64_t *list_offsets;  // [nlist+1]
  const uint8_t *codes;         // [N][M]
  const int64_t *ids;           // [N]
  // column-major copy of the codes for the byte-plane scan, or NULL: list c starts at
  // codes_t + list_toff[c]; row m (byte m of every vector of the list, zero-padded
  // to a multiple of 64 vectors) follows row m - 1
  const uint8_t *codes_t = nullptr;
  const int64_t *list_toff = nullptr;  // [nlist+1], in bytes
};

int cpu_threads();

// Run fn(i) for i in [0, n) on up to cpu_threads() threads.
// caller_first (optional) runs on the calling thread before it joins the others.
void parallel_for(int64_t n, const std::function<void(int64_t)> &fn,
                  const std::function<void()> *caller_first = nullptr);

// The library's worker threads: created once (cpu_threads() of them) and parked
// between batches, so a small hybrid batch does not pay for thread creation.
// One job at a time; a caller that finds the pool taken runs its job on threads
// of its own.
class WorkerPool {
 public:
  static WorkerPool &get();
  // Start fn() on n pool threads (n is clamped to the pool size) and return at
  // once; false (nothing started) if another job holds the pool.
  bool start(int n, std::function<void()> fn);
  // Block until the job given to start() has finished on every thread; frees the pool.
  void wait();
  int size() const { return n_threads_; }
  ~WorkerPool();

 private:
  WorkerPool();
  void worker();
  struct Impl;
  Impl *impl_;
  int n_threads_;
};

// Per-vector term |r|^2 + 2 c.r of residual-encoded L2 for every stored vector
// (r = decoded residual, c = centroid of its list); returns the largest |pv|.
float cpu_residual_pv(const HostIndexView &ix, int64_t n_total, float *pv);

// Largest |bias(q, list)| over the listed clusters (negative ids skipped);
// 0 without residual encoding.
float cpu_max_bias(const HostIndexView &ix, const float *q, const int32_t *clusters, int n);

// Element-major copy of the codebooks, [msub][dsub][2^nbits] floats, which lets
// cpu_build_lut run its lanes along the codeword index.
void cpu_transpose_codebooks(const HostIndexView &ix, float *out);

// Fixed-point table of one query: lut[m*256 + j], one column per code byte (for
// 4-bit codes entry j of column m is the float sum of the entries of the two
// sub-quantizers packed in that byte, formed before quantization); max_bias: largest |bias| among
// ALL of the query's probes (resident or not).  Returns the scale exponent.
int cpu_build_lut(const HostIndexView &ix, const float *q, float max_bias, int32_t *lut);
// The same for two queries at once (q1 may be NULL: one query): the codebooks, the
// larger operand, are read once for both.  Same tables, bit for bit.
void cpu_build_lut_pair(const HostIndexView &ix, const float *q0, const float *q1, float max_bias0,
                        float max_bias1, int32_t *lut0, int32_t *lut1, int *e0, int *e1);

// True if this CPU runs the byte-plane scan (AVX-512 VBMI) and the environment
// does not ask for the plain loop (IVF_HOST_SCAN=scalar, read at every call).
bool cpu_has_plane_scan();
// Size in bytes of the column-major code copy; fills list_toff[nlist+1] if given.
int64_t cpu_transposed_bytes(const HostIndexView &ix, int64_t *list_toff);
void cpu_transpose_codes(const HostIndexView &ix, const int64_t *list_toff, uint8_t *out);

// Scan the listed clusters for one query with the table and exponent from
// cpu_build_lut; writes k candidates, best first, padded with (kKeyInvalid, -1).
// Clusters are taken one by one; `scanned` (optional) holds the number of list
// entries finished so far and reaches n_clusters once `out` is written, which is
// what the dispatcher compares with the query's expected count (Section 4.2.2).
// key_cap: only candidates with key <= key_cap are wanted (kKeyInvalid: all of them).
// A hybrid batch passes the k-th best key of the device's partial result once that
// is on the host: vectors of the cold lists that cannot displace it are then
// rejected by the filter pass from the first list on, and `out` may hold fewer than
// k candidates.
void cpu_scan_lists(const HostIndexView &ix, const int32_t *lut, int e, const float *q,
                    const int32_t *clusters, int n_clusters, int k, HostCand *out,
                    int32_t *scanned = nullptr, int32_t key_cap = kKeyInvalid);

// Merge two best-first lists of k candidates into the k best.
void merge_topk(const HostCand *a, const HostCand *b, int k, HostCand *out);

}  // namespace ivf
