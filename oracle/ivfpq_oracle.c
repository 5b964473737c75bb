/*
 * CPU oracle for IVF-PQ search.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, literal definition that the HIP library is checked
 * against.  Only tests/, the smoke check and the benchmark's cpu_baseline leg
 * may build or call it; the library never does, and the two share no code.
 *
 * What it computes follows the three-stage description of IVF-PQ search
 * (Section 2.2 "Search Operation in IVF Index" and the figure "Three stages of
 * vector search in IVF-based index"):
 *   (1) coarse quantization: score the query against every centroid and keep
 *       the nprobe best clusters;
 *   (2)+(3) for every code stored in those clusters, the aggregated distance
 *       between the query and the code's representative values, then the k
 *       best.  The lookup table of stage (2) only avoids recomputing partial
 *       distances; here each distance is computed directly from the decoded
 *       vector, which is the quantity the table sum equals term by term.
 * Arithmetic is double precision on the fp32 inputs.  Selection is a full
 * sort.  No table, no blocking, no partial selection.
 *
 * Readings where the paper is silent: PQ encodes the raw vector, or (by_residual)
 * the residual of the vector to its cluster centroid, in which case a stored
 * code decodes to centroid + representative values; L2 means squared L2; ties go to the smaller cluster id / vector id; missing
 * results are (-1, +inf for L2 | -inf for IP).
 *
 * Parity pins (tests/test_oracle_pins.py): exact brute-force kNN in flat mode,
 * exhaustive decoded scan at nprobe = nlist, a hand-computed ADC example,
 * sub-space separability of the distance, hit-rate conservation.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_L2 0
#define ORACLE_IP 1

typedef struct {
    double score;  /* smaller is better after sign handling in cmp */
    int64_t id;
} cand_t;

/* ascending score, ties to the smaller id */
static int cmp_asc(const void *a, const void *b) {
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->score < y->score) return -1;
    if (x->score > y->score) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

/* descending score, ties to the smaller id */
static int cmp_desc(const void *a, const void *b) {
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

/* Distance between a query and one fp32 vector, by the definition. */
static double pair_score(int metric, int d, const float *q, const float *x) {
    double s = 0.0;
    if (metric == ORACLE_L2) {
        for (int i = 0; i < d; ++i) {
            double t = (double)q[i] - (double)x[i];
            s += t * t;
        }
    } else {
        for (int i = 0; i < d; ++i) s += (double)q[i] * (double)x[i];
    }
    return s;
}

/* Same, against the vector a + b (the sum is formed in double, i.e. exactly). */
static double pair_score_sum(int metric, int d, const float *q, const float *a, const float *b) {
    double s = 0.0;
    if (metric == ORACLE_L2) {
        for (int i = 0; i < d; ++i) {
            double t = (double)q[i] - ((double)a[i] + (double)b[i]);
            s += t * t;
        }
    } else {
        for (int i = 0; i < d; ++i) s += (double)q[i] * ((double)a[i] + (double)b[i]);
    }
    return s;
}

/*
 * Stage (1).  For each query: score all nlist centroids, full sort, keep the
 * first min(nprobe, nlist).  out_probe: [nq][nprobe] (padded with -1),
 * out_score: [nq][nprobe] (NaN padded).  out_gap[q] = |score of the last kept
 * centroid - score of the first dropped one| (+inf when nothing is dropped):
 * the test harness uses it to recognise coarse near-ties.
 */
int oracle_coarse(int metric, int d, int nlist, const float *centroids,
                  int64_t nq, const float *queries, int nprobe,
                  int32_t *out_probe, double *out_score, double *out_gap) {
    if (d <= 0 || nlist <= 0 || nprobe <= 0 || nq < 0) return -1;
    int keep = nprobe < nlist ? nprobe : nlist;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t qi = 0; qi < nq; ++qi) {
        cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)nlist);
        if (!c) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        const float *q = queries + qi * d;
        for (int j = 0; j < nlist; ++j) {
            c[j].score = pair_score(metric, d, q, centroids + (size_t)j * d);
            c[j].id = j;
        }
        qsort(c, (size_t)nlist, sizeof(cand_t), metric == ORACLE_L2 ? cmp_asc : cmp_desc);
        for (int p = 0; p < nprobe; ++p) {
            out_probe[qi * nprobe + p] = p < keep ? (int32_t)c[p].id : -1;
            if (out_score) out_score[qi * nprobe + p] = p < keep ? c[p].score : NAN;
        }
        if (out_gap)
            out_gap[qi] = keep < nlist ? fabs(c[keep - 1].score - c[keep].score) : INFINITY;
        free(c);
    }
    return failed ? -2 : 0;
}

/*
 * Stages (2)+(3) over a given probe list (negative entries are skipped).
 * use_pq != 0: each stored code is decoded to its representative values,
 *   x_hat = concat_m codebooks[m][code[m]], and scored against the query.
 *   nbits = 8: one byte per sub-quantizer, 256 codewords each; nbits = 4: 16
 *   codewords each, two codes per byte (Section 2.2 describes fast-scan indexes
 *   with such short codes), codebooks [M][16][d/M].
 *   With residual_centroids != NULL ([nlist][d]) the codes encode residuals and
 *   x_hat = centroid of the list + concat_m codebooks[m][code[m]].
 * use_pq == 0 ("flat"): the raw fp32 vector (flat_vectors, same order as
 *   codes) is scored instead.
 * All candidates of the query are fully sorted; the first k are returned.
 */
int oracle_scan(int metric, int d, int M, int nbits, const float *codebooks,
                const int64_t *list_offsets, const uint8_t *codes,
                const int64_t *ids, const float *flat_vectors, int use_pq,
                const float *residual_centroids,
                int64_t nq, const float *queries, int nprobe,
                const int32_t *probe, int k, int64_t *out_ids, double *out_dist) {
    if (d <= 0 || k <= 0 || nprobe <= 0 || nq < 0) return -1;
    if (use_pq && (M <= 0 || d % M != 0)) return -1;
    if (use_pq && nbits != 8 && !(nbits == 4 && M % 2 == 0)) return -1;
    if (!use_pq && !flat_vectors) return -1;
    int dsub = use_pq ? d / M : 0;
    int ksub = 1 << nbits;                           /* codewords per sub-quantizer */
    size_t code_bytes = ((size_t)M * (size_t)nbits) / 8;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t qi = 0; qi < nq; ++qi) {
        const float *q = queries + qi * d;
        size_t total = 0;
        for (int p = 0; p < nprobe; ++p) {
            int32_t c = probe[qi * nprobe + p];
            if (c >= 0) total += (size_t)(list_offsets[c + 1] - list_offsets[c]);
        }
        cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (total ? total : 1));
        float *xhat = (float *)malloc(sizeof(float) * (size_t)d);
        if (!cand || !xhat) {
#pragma omp atomic write
            failed = 1;
            free(cand);
            free(xhat);
            continue;
        }
        size_t n = 0;
        for (int p = 0; p < nprobe; ++p) {
            int32_t c = probe[qi * nprobe + p];
            if (c < 0) continue;
            for (int64_t v = list_offsets[c]; v < list_offsets[c + 1]; ++v) {
                const float *x;
                if (use_pq) {
                    const uint8_t *code = codes + (size_t)v * code_bytes;
                    for (int m = 0; m < M; ++m) {
                        /* 4-bit codes: two per byte, the even sub-quantizer in the low half */
                        int j = nbits == 8 ? code[m] : (code[m >> 1] >> (4 * (m & 1))) & 15;
                        memcpy(xhat + (size_t)m * dsub,
                               codebooks + ((size_t)m * ksub + j) * dsub,
                               sizeof(float) * (size_t)dsub);
                    }
                    x = xhat;
                } else {
                    x = flat_vectors + (size_t)v * d;
                }
                if (use_pq && residual_centroids)
                    cand[n].score = pair_score_sum(metric, d, q,
                                                   residual_centroids + (size_t)c * d, x);
                else
                    cand[n].score = pair_score(metric, d, q, x);
                cand[n].id = ids[v];
                ++n;
            }
        }
        qsort(cand, n, sizeof(cand_t), metric == ORACLE_L2 ? cmp_asc : cmp_desc);
        for (int r = 0; r < k; ++r) {
            if ((size_t)r < n) {
                out_ids[qi * k + r] = cand[r].id;
                out_dist[qi * k + r] = cand[r].score;
            } else {
                out_ids[qi * k + r] = -1;
                out_dist[qi * k + r] = metric == ORACLE_L2 ? INFINITY : -INFINITY;
            }
        }
        free(cand);
        free(xhat);
    }
    return failed ? -2 : 0;
}

/*
 * Per-query hit rate as defined in Section 3.3 "Variance of Hit Rate across
 * Queries": the number of the query's probed clusters that fall inside the
 * cached (resident) set, over nprobe; plus per-cluster access counts
 * (Section 4.2.3, the router's counters).
 */
int oracle_hit_stats(int nlist, int64_t nq, int nprobe, const int32_t *probe,
                     const uint8_t *resident, uint64_t *per_cluster,
                     double *per_query_rate) {
    if (nlist <= 0 || nprobe <= 0 || nq < 0) return -1;
    for (int j = 0; j < nlist; ++j) per_cluster[j] = 0;
    for (int64_t qi = 0; qi < nq; ++qi) {
        int hit = 0, total = 0;
        for (int p = 0; p < nprobe; ++p) {
            int32_t c = probe[qi * nprobe + p];
            if (c < 0) continue;
            ++total;
            ++per_cluster[c];
            if (resident[c]) ++hit;
        }
        per_query_rate[qi] = total ? (double)hit / (double)total : 0.0;
    }
    return 0;
}

/* Limit the query loops to n threads (n >= 1); the arithmetic is untouched. */
void oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Threads the query loops run on (OpenMP over queries only). */
int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
