// Internal declarations shared by the host API and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ivfpq_hot.h"

namespace ivf {

constexpr int kTileVecs = 64;      // vectors per code tile (one wavefront)
constexpr int kMaxSlices = 256;    // scan blocks per query, upper bound (slices * k <= kMaxMergeCand)
constexpr int kMaxMergeCand = 8192;  // candidates the per-query merge holds in LDS (16 B each)
// Partial-result rows (one per scan block of a sliced query) the workspace holds:
// room for eight slices of every query of a full batch, and for kMaxSlices slices of
// the small batches that need them to fill the chip.
constexpr int64_t part_rows(int64_t max_nq) {
  return max_nq * 8 > 16 * (int64_t)kMaxSlices ? max_nq * 8 : 16 * (int64_t)kMaxSlices;
}
constexpr int kMaxK = 128;
constexpr int kMaxNprobe = 2048;
constexpr int kSelSplitMaxNq = 128;  // largest batch the split coarse selection serves
constexpr int kLutMaxParts = 512;   // per-query slots for partial table maxima
constexpr int kSplitPadBytes = 16384;  // tail padding of the split-fp16 operand arrays
constexpr int kWsSlots = 2;        // batches that may be in flight on different streams
// size of the file-scope device array behind ivf_coarse_probe_dev_noalloc
constexpr size_t kStaticScratchBytes = IVF_STATIC_SCRATCH_BYTES;

// Counters kept on the device next to the per-cluster hit counters.
enum {
  QS_RESIDENT_PROBES = 0,
  QS_PROBES = 1,
  QS_QUERIES = 2,
  QS_MIN_RATE_BITS = 3,  // float bits of the smallest per-query hit rate
  QS_SCAN_BYTES = 4,     // instrumentation, reset separately
  QS_RATE_SUM = 5,       // sum over queries of the hit rate, in units of 2^-32
  QS_RATE_SQ = 6,        // sum over queries of its square, in units of 2^-32
  QS_COUNT = 8
};

// One 64-vector tile to fill from staged raw codes/ids.
struct TileDesc {
  int32_t dst_tile;   // tile index in the cluster region
  int32_t src_vec;    // first vector: in the staging chunk, or in the caller's arrays (direct copy)
  int32_t n_valid;    // 1..64 (0 never emitted)
  int32_t pad;
};

// Per-batch workspace.  There are kWsSlots of them so that batches issued on
// different streams can be in flight together (one batch's coarse stage then
// overlaps another's scan).
struct BatchWs {
  void *q_parts;           // [max_nq][d] queries as a two-way fp16 split, 4 B per element
  int32_t *q_exp;          // [max_nq] power-of-two scale of each split row
  float *queries;          // [max_nq][d]
  float *scores;           // [max_nq][nlist]
  void *sel_split;         // workspace of the split coarse selection
  int32_t *probe;          // [max_nq][max_nprobe]
  int32_t *g_base;         // [max_nq][max_nprobe] first tile of each resident probe
  int32_t *g_len;          // [max_nq][max_nprobe] list length
  int32_t *g_prefix;       // [max_nq][max_nprobe+1] running tile count
  int32_t *g_n;            // [max_nq] resident probes
  int32_t *cold;           // [max_nq][max_nprobe] non-resident cluster ids
  int32_t *n_cold;         // [max_nq]
  float *lut;              // [max_nq][256][M], one column per code byte
  uint32_t *lutpart;       // [max_nq][kLutMaxParts] partial maxima, one slot per LUT-kernel wave
  uint32_t *lutmax;        // [max_nq] bits of the largest |entry| of the query's table
  int32_t *q_vecs;         // [max_nq] vectors in the query's resident probes
  int32_t *order;          // [max_nq] scan visiting order of the queries
  int32_t *heavy;          // [max_nq] the queries that get one more scan block than the others
  int32_t *hslot;          // [max_nq] position of a query in heavy[], or -1
  float *bias;             // [max_nq][max_nprobe] residual encoding: bias(q, probe), probe order
  float *g_bias;           // [max_nq][max_nprobe] the same for resident probes, work-list order
  float *qbmax;            // [max_nq] largest |bias| among the query's probes (0 if unused)
  int32_t *part_key;       // [part_rows(max_nq)][max_k]: row (q * slices + s) of a launch
  int64_t *part_id;
  int32_t *res_key;        // [max_nq][max_k] merged GPU partial (hybrid path)
  int64_t *res_id;
  int64_t *out_ids;        // [max_nq][max_k] host-API staging
  float *out_dists;
};

// Pointers into the device arena.
struct DevLayout {
  float *centroids;        // [nlist][d]
  float *cent_norm;        // [nlist] squared norms (L2 only)
  void *cent_parts;        // centroids as a two-way fp16 split, 4 B per element
  int32_t *cent_exp;       // [nlist] power-of-two scale of each split row
  float *cbT;              // [2^nbits][msub][dsub] transposed codebooks
  int32_t *clus_len;       // [nlist]
  int32_t *clus_tile[3];   // mapping table ring: first tile of a resident cluster, or -1
  unsigned long long *hits;    // [nlist]
  unsigned long long *qstats;  // [QS_COUNT]
  struct BatchWs ws[kWsSlots];  // per-batch workspaces: batches on different streams overlap
  uint8_t *staging;        // copy staging
  size_t staging_bytes;
  uint8_t *tile_codes;     // [cap_tiles][M*64]
  int64_t *tile_ids;       // [cap_tiles][64]
  float *tile_pv;          // [cap_tiles][64] per-vector term (residual-encoded L2), else NULL
  int64_t cap_tiles;
};

struct Shape {
  int d, nlist;
  int M;             // bytes per stored code = columns of the scan's lookup table
  int dsub, metric_ip;
  int by_residual;   // codes encode x - centroid
  float pv_max;      // largest |per-vector term| (residual-encoded L2), else 0
  int nbits;         // bits per code: 8, or 4 (two codes per byte)
  int msub;          // sub-quantizers: M for 8-bit codes, 2 M for 4-bit codes
  int lut_kind() const { return metric_ip ? 1 : (by_residual ? 2 : 0); }
  int scan_res() const { return by_residual ? (metric_ip ? 1 : 2) : 0; }
};

// ---- kernel launchers (kernels_*.hip).  All enqueue on `st` and return the
// HIP error of the launch. ----
hipError_t launch_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t st);

hipError_t launch_calib_copy(const void *src, void *dst, size_t bytes, hipStream_t st);
// sink: at least 2 MiB (one word per launched thread)
hipError_t launch_calib_read(const void *src, void *sink, size_t bytes, hipStream_t st);

hipError_t launch_cent_norms(const float *cent, int nlist, int d, float *out, hipStream_t st);

// fp32 [rows][d] -> two-way fp16 split of the rows scaled by 2^row_exp, 4 bytes per element
hipError_t launch_split_f16(const float *src, size_t rows, int d, void *dst, int32_t *row_exp,
                            hipStream_t st);

hipError_t launch_coarse_gemm(const Shape &sh, const void *q_parts, const int32_t *q_exp, int nq,
                              const void *cent_parts, const int32_t *cent_exp,
                              const float *cent_norm, float *scores, hipStream_t st);

// split_ws: coarse_select_split_bytes() of workspace (256-byte aligned), or NULL.  With it,
// batches of up to kSelSplitMaxNq queries over more than 16384 lists are selected by
// several blocks per query; the result is the same exact selection.  ordered != 0: best
// first throughout; ordered == 0: the best cluster first, the others in any order
// (selections of more than a thousand candidates are then not sorted).
hipError_t launch_coarse_select(const Shape &sh, const float *scores, int nq, int nprobe,
                                int probe_stride, int32_t *probe, void *split_ws, int ordered,
                                hipStream_t st);
size_t coarse_select_split_bytes();

// The coarse quantizer with its intermediates in the library's file-scope device array
// (kStaticScratchBytes per device) instead of a workspace.  static_scratch_for_device
// returns that array's address on `device`, which must be the current device the first
// time it is asked for; coarse_static_bytes is what a batch of nq queries needs of it.
hipError_t static_scratch_for_device(int device, void **ptr);
size_t coarse_static_bytes(const Shape &sh, int64_t nq);
hipError_t launch_coarse_probe_static(const Shape &sh, const float *queries, int nq, int nprobe,
                                      const void *cent_parts, const int32_t *cent_exp,
                                      const float *cent_norm, void *scratch_ptr, int32_t *out_probe,
                                      hipStream_t st);

// bias(q, probe) for every probe of every query (residual encoding)
hipError_t launch_bias(const Shape &sh, const float *q, int nq, const int32_t *probe, int nprobe,
                       int probe_stride, const float *centroids, float *bias, hipStream_t st);

// bias may be NULL (no residual encoding): g_bias is then untouched and qbmax set to 0.
// lut_parts > 0: also reduce each query's lut_parts partial table maxima into lutmax.
hipError_t launch_route(const int32_t *probe, int nq, int nprobe, int probe_stride, int nlist,
                        const int32_t *clus_tile, const int32_t *clus_len, int M, int32_t *g_base,
                        int32_t *g_len, int32_t *g_prefix, int32_t *g_n, int32_t *cold,
                        int32_t *n_cold, int32_t *q_vecs, const float *bias, float *g_bias,
                        float *qbmax, unsigned long long *hits, int count_stats,
                        const uint32_t *lutpart, int lut_parts, uint32_t *lutmax, hipStream_t st);

// Lookup tables of every query and, per query, *n_parts partial maxima in lutpart.
// With q_parts != NULL the launch also does launch_split_f16(q, nq, d, q_parts, q_exp).
hipError_t launch_lut(const Shape &sh, const float *q, int nq, const float *cbT, float *lut,
                      uint32_t *lutpart, int *n_parts, void *q_parts, int32_t *q_exp,
                      hipStream_t st);

// After the router: batch totals of the router counters, the scan's visiting order and,
// with extra > 0, the `extra` queries with the most resident vectors (W.heavy, W.hslot).
hipError_t launch_order(const BatchWs &W, int nq, int probe_stride, int M,
                        unsigned long long *qstats, int count_stats, int extra, hipStream_t st);

// Every query is scanned by `slices` blocks, the `extra` heaviest ones (launch_order) by
// slices + 1.  Returns hipErrorInvalidValue for an unsupported (M, k).  A query scanned
// by a single block gets its result written by that block, as launch_merge would (same
// meaning of out_ids / out_dists); with slices == 1 and extra == 0 launch_merge is not needed.
hipError_t launch_scan(const Shape &sh, const DevLayout &L, const BatchWs &W, int nq,
                       int probe_stride, int slices, int extra, int k, int64_t *out_ids,
                       float *out_dists, hipStream_t st);

// out_ids != NULL: write (id, dist) to out_ids/out_dists; else (key, id) to res_key/res_id.
hipError_t launch_merge(const Shape &sh, const BatchWs &W, int nq, int slices, int extra, int k,
                        int64_t *out_ids, float *out_dists, hipStream_t st);

// stage_pv / tile_pv may be NULL
hipError_t launch_interleave(const uint8_t *stage_codes, const int64_t *stage_ids,
                             const float *stage_pv, const TileDesc *descs, int n_tiles, int M,
                             uint8_t *tile_codes, int64_t *tile_ids, float *tile_pv,
                             hipStream_t st);
// the same, reading the caller's pinned host arrays directly (descs[].src_vec =
// index of the tile's first vector in those arrays)
hipError_t launch_interleave_direct(const uint8_t *host_codes, const int64_t *host_ids,
                                    const float *host_pv, const TileDesc *descs, int n_tiles, int M,
                                    uint8_t *tile_codes, int64_t *tile_ids, float *tile_pv,
                                    hipStream_t st);

bool scan_supports(int M, int k);
// scan blocks that fit one compute unit at a time (its LDS decides)
int scan_blocks_per_cu(int M, int k);

}  // namespace ivf
