/*
 * ivfpq_hot — IVF-PQ similarity search over the GPU-resident (hot-cluster)
 * partition of an inverted-file index on AMD MI355X (gfx950), with probes of
 * non-resident clusters scanned on the host CPU and merged.
 *
 * The calls follow the tiered search structure of the paper: frequently hit
 * clusters are placed on the GPU and the rest stay on the CPU (Section 3.2,
 * Takeaway 2); a query is coarse-quantized, each probed cluster is looked up
 * in a mapping table and routed to the GPU or the CPU scan (Section 4.2.1
 * "Router"), partial results are merged and re-ranked (Section 4.2.2); the
 * router's counters and the refresh of the GPU-resident set follow Section
 * 4.2.3 "Adaptive Runtime Index Update".  Search itself is the three-stage
 * IVF-PQ procedure of Section 2.2: coarse quantization, per-query lookup
 * table, table scan with top-k.
 *
 * Conventions
 *  - Plain C ABI.  Every pointer is documented as HOST or DEVICE memory.
 *  - A negative return value is an error; ivf_last_error() then holds a
 *    message (thread-local).  On an argument, state or memory error no output
 *    buffer is written; after a HIP failure (IVF_EDEVICE) outputs are undefined.
 *  - The library never frees or reallocates caller memory.  Arrays named in
 *    ivf_index_desc_t are BORROWED for the lifetime of the index: they are the
 *    source of the CPU scan and of host-to-device cluster copies.
 *  - The library performs no device allocation of its own: all device state
 *    lives in the caller-supplied arena.
 *  - "L2" is squared Euclidean distance (smaller is better); "IP" is the inner
 *    product (larger is better).  PQ codes are 8 bits per sub-quantizer, or 4
 *    (nbits = 4, two per byte), and encode either the raw vector or
 *    (by_residual) its residual to the centroid of its list; a stored code then
 *    stands for centroid + representative values.  Either way one lookup table
 *    per query serves every probed list.
 *  - Results are ordered best first; ties on distance go to the smaller id.
 *    Missing results are id = -1, dist = +INF (L2) / -INF (IP).
 *  - Threading: one searcher thread plus one migrator thread per index.
 *    The CPU scan of non-resident clusters runs on worker threads of the
 *    library's own, created once per process: as many as the environment
 *    variable IVF_CPU_THREADS says, else OMP_NUM_THREADS, else the hardware
 *    concurrency.
 *  - Streams are raw hipStream_t values passed as void*; NULL is HIP's null
 *    stream.  All streams must have default priority.  The host-pointer entry
 *    points run on a stream the index owns.  The index holds two per-batch
 *    workspaces, each tied to the stream that used it last, so batches issued
 *    on two different streams may be in flight together; a call on a third
 *    stream first waits for the least recently used of them to drain.
 */
#ifndef IVFPQ_HOT_H
#define IVFPQ_HOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#if defined(__GNUC__)
#pragma GCC visibility push(default) /* the library is built with hidden visibility */
#endif

typedef struct ivf_index ivf_index_t; /* opaque */

enum { IVF_METRIC_L2 = 0, IVF_METRIC_IP = 1 };

enum {
  IVF_OK = 0,
  IVF_EINVAL = -1,  /* bad argument / unsupported shape */
  IVF_ENOMEM = -2,  /* arena (or its cluster region) too small */
  IVF_EDEVICE = -3, /* HIP error, or a device call on an index without arena */
  IVF_EBUSY = -4,   /* a migration or an asynchronous batch is still in flight */
  IVF_ESTATE = -5   /* call not valid in the current state */
};

/*
 * Index description.  All pointers are HOST memory, borrowed until
 * ivf_index_destroy().  `codes` and `ids` should be pinned: cluster copies are
 * then read from them by a kernel (ivf_copy_form).
 *
 * Supported shapes: nbits == 8 or 4; M * nbits / 8 (bytes per code) a multiple
 * of 16 and <= 128, i.e. M <= 128 for 8-bit and M <= 256 for 4-bit codes; d a multiple
 * of M; nlist >= 1; with a device and 4-bit codes d <= 2048; the device scan
 * has kernels for 16, 32, 48, 64, 96 and 128 bytes per code.  max_nq /
 * max_nprobe / max_k size the per-batch workspace (max_k <= 128,
 * max_nprobe <= 2048).
 */
typedef struct {
  int32_t d;      /* vector dimension */
  int32_t nlist;  /* number of IVF clusters */
  int32_t M;      /* PQ sub-quantizers */
  int32_t nbits;  /* bits per code: 8, or 4 (short codes as used by fast-scan indexes, Section
                     2.2): 16 codewords per sub-quantizer, two codes per byte, sub-quantizer
                     2i in the low half of byte i */
  int32_t metric; /* IVF_METRIC_L2 or IVF_METRIC_IP (also the coarse metric) */
  int32_t max_nq;
  int32_t max_nprobe;
  int32_t max_k;
  int32_t by_residual; /* 0: codes encode the vector; 1: the vector minus its list's centroid */
  const float *centroids;      /* [nlist][d] */
  const float *codebooks;      /* [M][2^nbits][d/M] */
  const int64_t *list_offsets; /* [nlist+1] prefix sums, in vectors */
  const uint8_t *codes;        /* [N][M * nbits / 8], cluster after cluster */
  const int64_t *ids;          /* [N] caller ids, same order as codes */
} ivf_index_desc_t;

/*
 * Bytes of device arena needed for `desc` with room for `resident_vectors`
 * vectors in GPU-resident clusters (each cluster is padded to a multiple of
 * 64 vectors; pass N + 64*nlist for a fully resident index) and
 * `staging_bytes` of copy staging (0 = default 64 MiB).  Returns 0 if desc is
 * invalid.  No device call is made.
 */
size_t ivf_index_arena_bytes(const ivf_index_desc_t *desc, int64_t resident_vectors,
                             size_t staging_bytes);

/*
 * Create an index.  dev_arena: DEVICE memory owned by the caller, 256-byte
 * aligned, of arena_bytes bytes, valid until destroy; the library places
 * centroids, codebooks, mapping tables, counters, batch workspace and the
 * cluster region inside it.  No cluster is resident after creation.
 *
 * The codes, ids, centroids and codebooks of `desc` stay borrowed; the index
 * adds host copies of its own only in derived layouts (codebooks element-major;
 * codes column-major when the byte-plane CPU scan is used, see
 * ivf_host_scan_form).
 *
 * dev_arena == NULL creates a host-only index: every cluster is non-resident
 * and only ivf_search_batch_probes(), ivf_hit_stats() and destroy are valid
 * (anything that needs the device returns IVF_EDEVICE).
 */
int ivf_index_create(const ivf_index_desc_t *desc, void *dev_arena, size_t arena_bytes,
                     size_t staging_bytes, ivf_index_t **out);

/*
 * Destroy the index (NULL is a no-op).  Waits for the device.  Must not run while
 * another thread is inside a call on the index, nor before ivf_search_wait()
 * has returned for an asynchronous batch started on it.
 */
void ivf_index_destroy(ivf_index_t *index);

/*
 * Make exactly the listed clusters GPU-resident (Section 4.1.4: the hot
 * clusters chosen from the access profile are placed on the GPU; the mapping
 * table records cluster id -> resident location).  Re-packs the cluster region
 * from scratch, i.e. a full refresh.  cluster_ids: HOST, n entries, distinct,
 * each in [0, nlist).  Copies run on `stream`; the call
 * returns after the copies have completed and the mapping table is published.
 * IVF_ENOMEM if the cluster region cannot hold them (nothing changes).
 * Must not run concurrently with a search or a migration.
 */
int ivf_index_load_partition(ivf_index_t *index, const int32_t *cluster_ids, int32_t n,
                             void *stream);

/*
 * Search a batch (Section 2.2 stages 1-3, routed per Section 4.2.1, merged per
 * Section 4.2.2).  queries: HOST fp32 [nq][d].  out_ids: HOST int64 [nq][k];
 * out_dists: HOST fp32 [nq][k].  nprobe > nlist is clamped.  nq == 0 is a
 * no-op.  Requires 1 <= nq <= max_nq, 1 <= nprobe <= max_nprobe,
 * 1 <= k <= max_k.  Returns after the results are written.  Buffers in pinned
 * host memory (hipHostMalloc) are copied from and to by DMA as they are;
 * pageable queries are first gathered in a pinned buffer of the index by the
 * library's worker threads, pageable results pass through one.
 */
int ivf_search_batch(ivf_index_t *index, const float *queries, int64_t nq, int32_t nprobe,
                     int32_t k, int64_t *out_ids, float *out_dists);

/*
 * Same search with DEVICE buffers: queries, out_ids, out_dists are device
 * pointers, work is enqueued on `stream`.  When every probed cluster can be
 * served from the GPU (the index is fully resident) the call is asynchronous:
 * it returns after enqueueing and the outputs are valid once `stream` reaches
 * that point.  Otherwise the call synchronizes with `stream`, scans cold
 * probes on the CPU, and returns with the outputs complete.
 */
int ivf_search_batch_dev(ivf_index_t *index, const float *queries, int64_t nq, int32_t nprobe,
                         int32_t k, int64_t *out_ids, float *out_dists, void *stream);

/*
 * Stage 1 only (coarse quantizer): the nprobe best clusters per query, best
 * first, ties to the smaller cluster id.  queries: DEVICE fp32 [nq][d];
 * out_probe: DEVICE int32 [nq][nprobe] (entries beyond nlist are -1).
 * Asynchronous on `stream`.  Does not touch the hit counters.
 */
int ivf_coarse_probe_dev(ivf_index_t *index, const float *queries, int64_t nq, int32_t nprobe,
                         int32_t *out_probe, void *stream);

/*
 * ivf_coarse_probe_dev for callers that cannot allocate device memory or hand
 * over a workspace, and must not be made to wait for one: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same result (the selection is exact on either path; this one always
 * uses the one-block-per-query selection kernel).  What differs is where the
 * kernels' intermediates live (the queries' fp16 split, their scales, the
 * nq x nlist score matrix): not in one of the index's two per-batch workspaces
 * but in a file-scope device array of IVF_STATIC_SCRATCH_BYTES that is part of
 * the library's code object; every GPU the library runs on holds its own copy
 * until the process ends.  Its device address is looked up once per device by
 * ivf_index_create.  The call takes no workspace slot, no lock and no event,
 * never waits for another stream, and calls no hipMalloc / hipFree or any other
 * allocating routine; the caller still passes queries and out_probe (DEVICE).
 *
 * Limit: 256-byte-rounded nq * d * 4 + 16384, nq * 4 and nq * nlist * 4 bytes
 * together must fit the array (e.g. nq <= 126 at nlist = 65536, d = 768;
 * nq <= 488 at nlist = 16384); a larger batch returns IVF_EINVAL and launches
 * nothing.  Nothing in the array needs clearing between calls.  All calls on
 * one GPU, from any index, share that GPU's array: calls that overlap on one GPU
 * (different streams or threads) race on it and return garbage; calls on one
 * stream are ordered by the stream.
 */
#define IVF_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int ivf_coarse_probe_dev_noalloc(ivf_index_t *index, const float *queries, int64_t nq,
                                 int32_t nprobe, int32_t *out_probe, void *stream);

/*
 * Stages 2-3 with a caller-given probe list instead of the coarse quantizer
 * (routing, GPU scan of resident probes, CPU scan of the rest, merge).  All
 * pointers HOST.  probe: int32 [nq][nprobe]; negative entries are skipped;
 * other entries must be in [0, nlist) and distinct within a query.  Valid on a
 * host-only index (everything is scanned on the CPU).
 */
int ivf_search_batch_probes(ivf_index_t *index, const float *queries, int64_t nq,
                            const int32_t *probe, int32_t nprobe, int32_t k, int64_t *out_ids,
                            float *out_dists);

/*
 * Dynamic dispatcher (Section 4.2.2 "Dynamic Dispatcher"): the same search as
 * ivf_search_batch() (probe == NULL) or ivf_search_batch_probes() (probe given),
 * but every query is merged, re-ranked and handed on as soon as its own probes
 * are done instead of when the whole batch is.  The call enqueues the device
 * side, starts a dispatcher thread and returns.  The CPU search loop takes the
 * queries' cold clusters one by one and keeps a scan count per query; when it
 * equals the number of cold probes routed to the CPU, the query enters a
 * thread-safe completed queue.  Once the device has signalled completion of
 * the resident probes, the dispatcher takes queries off that queue, merges the
 * CPU and GPU partial results, writes row q of out_ids / out_dists and calls
 * on_done(user, q, row of ids, row of dists, k) on the dispatcher thread
 * (on_done may be NULL).  Results are bit-identical to the synchronous calls.
 *
 * queries, probe (optional), out_ids, out_dists: HOST; queries and the outputs
 * must stay valid until ivf_search_wait() returns.  A device-less index needs
 * a probe list.  One asynchronous batch per index at a time: until
 * ivf_search_wait() has returned, other searches on the index return
 * IVF_EBUSY.  on_done must not call into this index.
 */
typedef struct ivf_ticket ivf_ticket_t; /* opaque */
typedef void (*ivf_query_done_fn)(void *user, int64_t query, const int64_t *ids,
                                  const float *dists, int32_t k);
int ivf_search_batch_async(ivf_index_t *index, const float *queries, int64_t nq,
                           const int32_t *probe, int32_t nprobe, int32_t k, int64_t *out_ids,
                           float *out_dists, ivf_query_done_fn on_done, void *user,
                           ivf_ticket_t **ticket);

/*
 * Take up to cap finished queries off the ticket, in the order they were
 * handed on (each is reported once).  queries_done: HOST [cap].  *finished is
 * set to 1 once every query of the batch has been reported through this call.
 * Returns the batch's error, if it has failed.
 */
int ivf_search_poll(ivf_ticket_t *ticket, int64_t *queries_done, int64_t cap, int64_t *n_done,
                    int32_t *finished);

/*
 * Wait for the batch, release the ticket (it is invalid afterwards, also on
 * error) and return the batch's status.  done_ms: HOST double [nq] or NULL, the
 * time in milliseconds from the ivf_search_batch_async() call to each query's
 * hand-off.
 */
int ivf_search_wait(ivf_ticket_t *ticket, double *done_ms);

/*
 * Router counters (Section 4.2.3; per-query hit rate as defined in Section
 * 3.3: resident probes / probes).  per_cluster_hits: HOST uint64 [nlist] or
 * NULL, number of times each cluster was probed since the last reset.
 * mean_hit_rate = resident probes / all probes; min_hit_rate = smallest
 * per-query hit rate; n_queries = queries counted.  Any output may be NULL.
 * reset != 0 clears the counters after reading.  Synchronizes with searches
 * already enqueued.
 */
int ivf_hit_stats(ivf_index_t *index, uint64_t *per_cluster_hits, double *mean_hit_rate,
                  double *min_hit_rate, uint64_t *n_queries, int reset);

/*
 * Change the resident set while searches continue (Section 4.2.3).  evict /
 * admit: HOST cluster ids.  Evicted clusters stop being routed to the GPU at
 * the next publish; admitted clusters are copied host->device on side_stream
 * (pinned asynchronous copies when `codes` is pinned) and become resident when
 * the copy has completed, observed at the start of the next search or by
 * ivf_migrate_poll().  Until then their probes are served by the CPU scan, so
 * results never change.  Space of evicted clusters is reused only after every
 * search that could read it has drained.  IVF_EBUSY if a migration is in
 * flight; IVF_ENOMEM if the admitted clusters do not fit without the space
 * still held by evicted ones (nothing changes); IVF_EINVAL for an id out of
 * range, evicting a non-resident or admitting a resident cluster.
 */
int ivf_migrate_clusters(ivf_index_t *index, const int32_t *evict, int32_t n_evict,
                         const int32_t *admit, int32_t n_admit, void *side_stream);

/*
 * Progress of the migration in flight.  wait != 0 blocks until the copies have
 * completed.  Publishes the new mapping table when complete.  Returns 1 if a
 * migration is still in flight after the call, 0 if none is, negative on
 * error.  bytes_copied (HOST, may be NULL): code + id bytes of clusters
 * admitted by migrations completed since creation.
 */
int ivf_migrate_poll(ivf_index_t *index, int wait, uint64_t *bytes_copied);

/*
 * One step of the runtime index update (Section 4.2.3 "Adaptive Runtime Index
 * Update": the access counters name a new hot set and the device's copy is
 * refreshed while the CPU serves what is not there yet).  Reads the router's
 * per-cluster counters, takes the n_hot most accessed clusters as the hot set
 * (Section 4.1.4 "Index Splitter": clusters ranked by access frequency; equal
 * counts go to the smaller cluster id), and starts the migration from the
 * current resident set to it on side_stream exactly as ivf_migrate_clusters
 * would: resident clusters outside the hot set are evicted, hot clusters that
 * are not resident are admitted, hottest first.  A cluster that finds no free
 * space (space of evicted clusters is reusable only once the searches that
 * might read it have drained) is left cold and counted in *n_deferred; the next
 * refresh admits it.  reset != 0 clears the counters after reading, also when
 * there was nothing to move.  Outputs (HOST, any may be NULL): clusters
 * evicted, admitted and deferred; mean_hit_rate of the searches counted since
 * the last reset.  Nothing to move: IVF_OK and no migration is started.
 * IVF_EBUSY if a migration is in flight or an old mapping table is still being
 * read; IVF_ESTATE if no search has been counted since the last reset (the
 * counters then say nothing and the resident set is kept); IVF_EINVAL for
 * n_hot outside [0, nlist].  Synchronizes with searches already enqueued, like
 * ivf_hit_stats.
 */
int ivf_refresh_hot_set(ivf_index_t *index, int32_t n_hot, int reset, void *side_stream,
                        int32_t *n_evicted, int32_t *n_admitted, int32_t *n_deferred,
                        double *mean_hit_rate);

/*
 * Totals over migrations completed since creation (any output may be NULL):
 * bytes_copied as in ivf_migrate_poll; copy_ms = time between the first copy
 * and the last kernel of each migration on its side stream, from HIP events;
 * n_migrations = completed migrations.  All HOST pointers.
 */
int ivf_migrate_stats(ivf_index_t *index, uint64_t *bytes_copied, double *copy_ms,
                      uint64_t *n_migrations);

/* Number of currently resident clusters and vectors (either may be NULL). */
int ivf_resident_info(ivf_index_t *index, int32_t *n_clusters, int64_t *n_vectors);

/*
 * The published resident set (the mapping table of Section 4.1.4 read back):
 * ids of the resident clusters in ascending order into cluster_ids (HOST int32
 * [cap], may be NULL when cap = 0), their number into *n (HOST).  Clusters of a
 * migration still in flight are not in it.  IVF_EINVAL if cap is smaller than
 * the number of resident clusters (*n is still written, nothing else is).
 */
int ivf_resident_list(ivf_index_t *index, int32_t *cluster_ids, int32_t cap, int32_t *n);

/*
 * Which form of the CPU scan of non-resident clusters (Section 4.2.1) this
 * index uses: 0 = the plain loop over each vector's code bytes, 1 = the
 * byte-plane scan (CPUs with AVX-512 VBMI; the index then holds a column-major
 * copy of the codes, N * code-bytes more host memory, made at creation).  Both
 * add the same integers and return identical results.  The environment
 * variable IVF_HOST_SCAN=scalar, read by ivf_index_create, selects form 0.
 * Form 1 first bounds every vector's sum from below with two of the four byte
 * planes of a growing share of the columns and forms exact sums only for
 * vectors the bound does not rule out (same results; IVF_HOST_FILTER=0, read
 * at every search, turns the bound off).
 * Negative on error.
 */
int ivf_host_scan_form(const ivf_index_t *index);

/*
 * How cluster copies (ivf_index_load_partition, ivf_migrate_clusters; Section
 * 4.2.3) reach the device: 1 = the copy kernel reads the caller's codes and ids
 * itself, which needs both arrays in pinned host memory that the device can
 * address (hipHostMalloc, or a pinned torch tensor; codes 16-byte aligned) and
 * fewer than 2^31 vectors; 0 = runs of vectors are copied with hipMemcpyAsync
 * into the staging area and rearranged from there (any host memory; one copy
 * call per run of consecutive vectors, so scattered clusters copy slowly).
 * Decided by ivf_index_create; IVF_COPY_PATH=staged in its environment selects
 * 0.  The resulting tiles are identical.  Negative on error.
 */
int ivf_copy_form(const ivf_index_t *index);

/*
 * Tuning and instrumentation.  scan_slices: blocks per query in the ADC scan
 * (0 = automatic).  timing = 1 records HIP events around every stage of
 * subsequent searches on their stream, timing = 2 only around the ADC scan
 * (each recorded event costs a few microseconds of stream time), 0 none.
 * The events of a batch are held until ivf_stage_times() reads them; after
 * 8192 unread batches further batches are not timed.  Events are pooled:
 * turning timing on stocks the pool, ivf_stage_times() returns events to it.
 */
int ivf_set_tuning(ivf_index_t *index, int32_t scan_slices, int32_t timing);

/*
 * Kernel times accumulated since the last reset, from HIP events recorded on
 * the search stream.  ms: HOST double [IVF_N_STAGES] total milliseconds per
 * stage; launches: HOST uint64 [IVF_N_STAGES]; scan_bytes: HOST, sum over
 * (query, resident probe) pairs of M * list length, the bytes the ADC scan
 * must stream.  Synchronizes with recorded events.  reset != 0 clears.
 */
enum {
  IVF_STAGE_LUT = 0,           /* lookup tables (built first: they need the queries only) */
  IVF_STAGE_COARSE_GEMM = 1,
  IVF_STAGE_COARSE_SELECT = 2,
  IVF_STAGE_ROUTE = 3,
  IVF_STAGE_SCAN = 4,
  IVF_STAGE_MERGE = 5,
  IVF_N_STAGES = 6
};
int ivf_stage_times(ivf_index_t *index, double *ms, uint64_t *launches, uint64_t *scan_bytes,
                    int reset);

/*
 * Spread of the per-query hit rate over the searches counted since the last
 * reset (Section 3.3: the hit rate varies from query to query; Section 4.1.2
 * models its variance as 4 sigma_max^2 mean (1 - mean) with one profiled
 * constant).  mean = average over queries of (resident probes / probes) (equal
 * to ivf_hit_stats' mean_hit_rate when every query has the same number of
 * probes), variance = their population variance, sigma_max2 = variance /
 * (4 mean (1 - mean)), the constant that ivf_model_min_hit_rate and its
 * relatives take (NaN when the mean is 0 or 1: the model says nothing there;
 * the paper profiles it where the mean is near one half).  All outputs HOST,
 * any may be NULL.  Rates are accumulated in units of 2^-32.  Synchronizes with
 * searches already enqueued; cleared by ivf_hit_stats' / ivf_refresh_hot_set's
 * reset.
 */
int ivf_hit_rate_moments(ivf_index_t *index, double *mean, double *variance, double *sigma_max2,
                         uint64_t *n_queries);

/*
 * The hit rate weighted by size (Section 3.2's access-skew figure counts distance
 * computations, not clusters): of the code bytes that the probes counted since
 * the last reset scan (each probe of list c scans M * L_c bytes), the share
 * that falls into clusters of the resident set as it stands now.  rate and
 * probed_bytes (that total) are HOST, either may be NULL; rate is 0 when nothing
 * has been counted.  Equals what the device scanned over what was scanned in
 * all if the resident set has not changed since the reset.  Synchronizes with
 * searches already enqueued.
 */
int ivf_weighted_hit_rate(ivf_index_t *index, double *rate, double *probed_bytes);

/*
 * The access profile the partitioning model works on (Section 4.1.1: cluster
 * access frequencies collected over calibration queries; Section 3.2: their
 * cumulative distribution), taken from the router's per-cluster counters as
 * they stand (searches since the last reset; nothing is cleared).  Clusters are
 * ranked from the most to the least probed, equal counts by id.  All outputs
 * HOST, any may be NULL: ranked int32 [nlist], the cluster ids in that order;
 * hit_cdf double [nlist+1], hit_cdf[i] = share of all counted probes that fall
 * into the i hottest clusters (hit_cdf[0] = 0, hit_cdf[nlist] = 1); mem_index
 * double [nlist+1], device bytes of the i hottest clusters (code bytes + 8 id
 * bytes per vector, + 4 for residual codes under L2).  The two curves are the
 * hit_cdf / mem_index arguments of ivf_model_hitrate_to_coverage and
 * ivf_model_partition_point, whose rho, times nlist, is ivf_refresh_hot_set's
 * n_hot.  IVF_ESTATE if no probe has been counted.  Synchronizes with searches
 * already enqueued.
 */
int ivf_profile_curves(ivf_index_t *index, int32_t *ranked, double *hit_cdf, double *mem_index);

/*
 * ---- Partitioning point (Section 4.1): pure host functions ----
 *
 * ivf_latency_model_t: piecewise-linear CPU latency models of the two search
 * stages as functions of the batch size (Section 4.1.1), given by n_knots >= 1
 * profiled points with strictly increasing batch sizes; linear between knots
 * and beyond the outer ones.  All pointers HOST.
 */
typedef struct {
  int32_t n_knots;
  const double *batch; /* [n_knots] */
  const double *t_cq;  /* [n_knots] coarse-quantization latency */
  const double *t_lut; /* [n_knots] table build + scan latency */
} ivf_latency_model_t;

/* Eq. (1): latency of the hybrid index at batch size `batch` when the smallest
 * hit rate in the batch is eta.  NaN on a malformed model. */
double ivf_model_hybrid_latency(const ivf_latency_model_t *model, double batch, double eta);

/* Eq. (2): expected smallest per-query hit rate in a batch of `batch` queries,
 * hit rates ~ Beta with the given mean and variance 4 sigma_max2 mean (1 - mean)
 * (Section 4.1.2).  0 < sigma_max2 < 0.25, else NaN. */
double ivf_model_min_hit_rate(double mean_hit_rate, double sigma_max2, int32_t batch);

/* Inverse of Eq. (2) over a measured profile ("HitRate2Coverage"): the smallest
 * fraction of clusters (hottest first, whole clusters) whose expected smallest
 * hit rate in a batch reaches eta_min.  hit_cdf: HOST double [nlist+1],
 * hit_cdf[i] = share of all probes that fall into the i hottest clusters. */
double ivf_model_hitrate_to_coverage(const double *hit_cdf, int32_t nlist, double sigma_max2,
                                     int32_t batch, double eta_min);

/* Algorithm 1 (latency-bounded partitioning): binary search for the coverage rho
 * at which the coverage needed to hold tau_s = slo_search / (1 + eps), at the
 * batch size the remaining LLM throughput implies, equals the coverage spent.
 * mem_index: HOST double [nlist+1], bytes of the i hottest clusters; mem_kvcache:
 * KV-cache bytes with no index loaded; mu_llm0: LLM throughput then (requests per
 * unit of the latency model's time); delta: width at which the search stops.
 * Writes rho to *rho_out.  IVF_EINVAL on bad arguments. */
int ivf_model_partition_point(const ivf_latency_model_t *model, const double *hit_cdf,
                              const double *mem_index, int32_t nlist, double sigma_max2,
                              double slo_search, double eps, double mem_kvcache, double mu_llm0,
                              double delta, double *rho_out);

/*
 * Instrumentation aid: a plain streaming copy kernel (reads `bytes`, writes
 * `bytes`; DEVICE pointers, 16-byte aligned, bytes a multiple of 16) whose
 * known traffic calibrates hardware byte counters.  Asynchronous on `stream`.
 */
int ivf_calib_copy(const void *src, void *dst, size_t bytes, void *stream);

/*
 * Instrumentation aid: a plain streaming read of `bytes` from src (DEVICE,
 * 16-byte aligned, bytes a multiple of 16); sink is DEVICE scratch of
 * sink_bytes >= IVF_CALIB_SINK_BYTES that receives one word per launched thread
 * (a smaller sink returns IVF_EINVAL).  Its rate is the achievable read
 * bandwidth, the practical ceiling of the ADC scan.  Asynchronous on `stream`.
 */
#define IVF_CALIB_SINK_BYTES ((size_t)2 << 20)
int ivf_calib_read(const void *src, void *sink, size_t sink_bytes, size_t bytes, void *stream);

/* Message for the last error returned on this thread ("" if none). */
const char *ivf_last_error(void);

#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#ifdef __cplusplus
}
#endif
#endif /* IVFPQ_HOT_H */
