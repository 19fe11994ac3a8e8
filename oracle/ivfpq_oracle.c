/*
 * CPU oracle for IVF-PQ retrieval.  TEST INFRASTRUCTURE ONLY: it exists to
 * define what the GPU library must compute and is never part of the product
 * path.  Plain, slow, and written to be checked by eye.  It shares no code
 * with the HIP library.
 *
 * What it follows.  The paper states retrieval as: a query vector goes in,
 * the k closest database entries come out (Section 2, "Database
 * construction"); the index is IVF-PQ: the database is clustered into nlist
 * inverted lists, nprobe of them are scanned per query and the vectors inside
 * are compared with the query (Section 3.2, S3), database vectors being
 * stored as product-quantisation codes (Section 3.1, O3; Appendix
 * "Detailed Evaluation Setup", Software: 64-byte codes).  The paper defers
 * the construction to the product-quantisation method it cites; the
 * readings taken where it is silent are listed beside each function.
 *
 * Precision.  Inputs are fp32.  Every sum is accumulated in fp64 in index
 * order and rounded to fp32 once.  Every decision (argmin, top-nprobe,
 * top-k) compares those fp32 values; equal values are ordered by the lower
 * index / id.
 *
 * All pointers are host memory owned by the caller.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Squared L2 distances from one vector to K centres.
 * dist[j] = sum_t (x[t] - c_j[t])^2, accumulated over t = 0..d-1 in order.
 * The centres are passed coordinate-major (ct[t*K + j] = c_j[t]) so the
 * loop over j is the contiguous one; the per-pair summation order is the
 * plain definition's. */
static void sqdist_to_all(const float *x, const float *ct, int64_t K, int d, double *dist) {
    for (int64_t j = 0; j < K; ++j) dist[j] = 0.0;
    for (int t = 0; t < d; ++t) {
        const double xt = (double)x[t];
        const float *row = ct + (int64_t)t * K;
        for (int64_t j = 0; j < K; ++j) {
            const double diff = xt - (double)row[j];
            dist[j] += diff * diff;
        }
    }
}

static float *transpose_centres(const float *c, int64_t K, int d) {
    float *ct = (float *)malloc(sizeof(float) * (size_t)K * (size_t)d);
    for (int64_t j = 0; j < K; ++j)
        for (int t = 0; t < d; ++t) ct[(int64_t)t * K + j] = c[j * d + t];
    return ct;
}

/* Nearest-centre assignment (used by k-means and by encoding).
 * x: [n] rows of d floats, row stride ldx floats.  c: [K, d].
 * out_idx[i] = argmin_j fp32(dist(x_i, c_j)), lowest j on equal values.
 * out_dist (optional): that fp32 distance. */
void oracle_assign(const float *x, int64_t n, int d, int64_t ldx, const float *c, int64_t K,
                   int32_t *out_idx, float *out_dist) {
    float *ct = transpose_centres(c, K, d);
#pragma omp parallel
    {
        double *dist = (double *)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            sqdist_to_all(x + i * ldx, ct, K, d, dist);
            float best = (float)dist[0];
            int32_t arg = 0;
            for (int64_t j = 1; j < K; ++j) {
                const float v = (float)dist[j];
                if (v < best) { best = v; arg = (int32_t)j; }
            }
            out_idx[i] = arg;
            if (out_dist) out_dist[i] = best;
        }
        free(dist);
    }
    free(ct);
}

/* Nearest centre among a given subset of the centres (the same definition as
 * oracle_assign, restricted): cand[i*T + t], t < T, are centre numbers for row
 * i; negative entries are skipped; a row needs at least one valid entry.
 * out_idx[i] = the listed centre with the smallest fp32(dist(x_i, c_j)), the
 * lowest number on equal values (whatever the order of the entries).  With
 * every centre listed this is oracle_assign.  It serves tests that have first
 * ruled out, by other means and with a wide margin, the centres that are far. */
void oracle_assign_among(const float *x, int64_t n, int d, int64_t ldx, const float *c, const int32_t *cand, int T,
                         int32_t *out_idx, float *out_dist) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const float *xi = x + i * ldx;
        float best = 0.f;
        int32_t arg = -1;
        for (int t = 0; t < T; ++t) {
            const int32_t j = cand[i * T + t];
            if (j < 0) continue;
            const float *cj = c + (int64_t)j * d;
            double acc = 0.0;
            for (int u = 0; u < d; ++u) {
                const double diff = (double)xi[u] - (double)cj[u];
                acc += diff * diff;
            }
            const float v = (float)acc;
            if (arg < 0 || v < best || (v == best && j < arg)) { best = v; arg = j; }
        }
        out_idx[i] = arg;
        if (out_dist) out_dist[i] = best;
    }
}

/* ------------------------------------------------------------------ */
/* Lloyd k-means with a fixed iteration count (reading: the paper does not
 * say how the IVF lists or PQ codebooks are trained; Section 3.2 S3 only
 * says the database is clustered).
 *   init:   centre j = row init_rows[j] (K distinct rows drawn by the caller)
 *   repeat `iters` times: assign every row to its nearest centre, then set
 *           each centre to the mean of its rows, summed in row order in
 *           fp64 and rounded to fp32; a centre with no rows keeps its value.
 * x: [S] rows of d floats with stride ldx.  c_out: [K, d].
 * inertia_out (optional, [iters]): sum over rows of the fp32 distance to the
 * assigned centre, measured in each iteration's assignment step.
 * The result does not depend on the number of threads. */
void oracle_kmeans(const float *x, int64_t S, int d, int64_t ldx, int64_t K, int iters,
                   const int64_t *init_rows, float *c_out, double *inertia_out) {
    for (int64_t j = 0; j < K; ++j)
        memcpy(c_out + j * d, x + init_rows[j] * ldx, sizeof(float) * (size_t)d);
    int32_t *assign = (int32_t *)malloc(sizeof(int32_t) * (size_t)S);
    float *adist = (float *)malloc(sizeof(float) * (size_t)S);
    int64_t *count = (int64_t *)malloc(sizeof(int64_t) * (size_t)K);
    double *sum = (double *)malloc(sizeof(double) * (size_t)K * (size_t)d);
    for (int it = 0; it < iters; ++it) {
        oracle_assign(x, S, d, ldx, c_out, K, assign, adist);
        if (inertia_out) {
            double tot = 0.0;
            for (int64_t i = 0; i < S; ++i) tot += (double)adist[i];
            inertia_out[it] = tot;
        }
        memset(count, 0, sizeof(int64_t) * (size_t)K);
        memset(sum, 0, sizeof(double) * (size_t)K * (size_t)d);
        for (int64_t i = 0; i < S; ++i) {          /* row order */
            const int64_t j = assign[i];
            count[j] += 1;
            double *s = sum + j * d;
            const float *xi = x + i * ldx;
            for (int t = 0; t < d; ++t) s[t] += (double)xi[t];
        }
        for (int64_t j = 0; j < K; ++j) {
            if (count[j] == 0) continue;
            for (int t = 0; t < d; ++t) c_out[j * d + t] = (float)(sum[j * d + t] / (double)count[j]);
        }
    }
    free(assign); free(adist); free(count); free(sum);
}

/* ------------------------------------------------------------------ */
/* Encoding (database construction): which inverted list a vector joins and
 * its PQ code.  Reading: the code quantises the raw vector, not its residual
 * to the list centre.
 *   list_out[i]    = nearest coarse centre of x_i
 *   codes_out[i,m] = nearest of the ksub centres of sub-quantiser m to the
 *                    m-th slice (dsub = d / M coordinates) of x_i
 * coarse: [nlist, d]; pq: [M, ksub, dsub]; codes_out: [n, M] bytes. */
void oracle_encode(const float *x, int64_t n, int d, const float *coarse, int64_t nlist, const float *pq,
                   int M, int ksub, int32_t *list_out, uint8_t *codes_out) {
    const int dsub = d / M;
    if (list_out) oracle_assign(x, n, d, d, coarse, nlist, list_out, NULL);
    if (!codes_out) return;
    int32_t *col = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    for (int m = 0; m < M; ++m) {
        oracle_assign(x + m * dsub, n, dsub, d, pq + (int64_t)m * ksub * dsub, ksub, col, NULL);
        for (int64_t i = 0; i < n; ++i) codes_out[i * M + m] = (uint8_t)col[i];
    }
    free(col);
}

/* ------------------------------------------------------------------ */
/* Coarse quantiser search (the index-scan term of the retrieval latency
 * model, Section 3.2 S3): the nprobe lists whose centres are closest to the
 * query, ordered by (distance, list number).
 * probes_out: [nq, nprobe]; dist_out (optional): [nq, nprobe]. */
typedef struct { float d; int64_t id; } cand_t;

static int cand_less(const cand_t *a, const cand_t *b) {
    return a->d < b->d || (a->d == b->d && a->id < b->id);
}
static int cand_cmp(const void *pa, const void *pb) {
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    return cand_less(a, b) ? -1 : (cand_less(b, a) ? 1 : 0);
}

void oracle_coarse(const float *q, int64_t nq, int d, const float *coarse, int64_t nlist, int nprobe,
                   int32_t *probes_out, float *dist_out) {
    float *ct = transpose_centres(coarse, nlist, d);
#pragma omp parallel
    {
        double *dist = (double *)malloc(sizeof(double) * (size_t)nlist);
        cand_t *all = (cand_t *)malloc(sizeof(cand_t) * (size_t)nlist);
#pragma omp for schedule(static)
        for (int64_t qi = 0; qi < nq; ++qi) {
            sqdist_to_all(q + qi * d, ct, nlist, d, dist);
            for (int64_t j = 0; j < nlist; ++j) { all[j].d = (float)dist[j]; all[j].id = j; }
            qsort(all, (size_t)nlist, sizeof(cand_t), cand_cmp);
            for (int p = 0; p < nprobe; ++p) {
                probes_out[qi * nprobe + p] = (int32_t)all[p].id;
                if (dist_out) dist_out[qi * nprobe + p] = all[p].d;
            }
        }
        free(dist); free(all);
    }
    free(ct);
}

/* ------------------------------------------------------------------ */
/* Per-query lookup table of the asymmetric distance computation:
 *   lut[m][j] = sum_{t<dsub} (q[m*dsub+t] - pq[m][j][t])^2      (fp64)
 * lut: [M, ksub] doubles. */
static void build_lut(const float *q, const float *pq, int M, int ksub, int dsub, double *lut) {
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < ksub; ++j) {
            const float *c = pq + ((int64_t)m * ksub + j) * dsub;
            double acc = 0.0;
            for (int t = 0; t < dsub; ++t) {
                const double diff = (double)q[m * dsub + t] - (double)c[t];
                acc += diff * diff;
            }
            lut[m * ksub + j] = acc;
        }
}

/* Same table rounded to fp32, for checking the table by itself. */
void oracle_lut(const float *q, int64_t nq, int d, const float *pq, int M, int ksub, float *lut_out) {
    const int dsub = d / M;
    double *lut = (double *)malloc(sizeof(double) * (size_t)M * (size_t)ksub);
    for (int64_t qi = 0; qi < nq; ++qi) {
        build_lut(q + qi * d, pq, M, ksub, dsub, lut);
        for (int64_t e = 0; e < (int64_t)M * ksub; ++e) lut_out[qi * M * ksub + e] = (float)lut[e];
    }
    free(lut);
}

/* ------------------------------------------------------------------ */
/* Scan of the probed lists + k-selection for given probe lists.
 *   dist(q, x) = fp32( sum_{m<M} lut[m][code_x[m]] ), m in order
 *   result     = the k candidates smallest by (dist, id); slots beyond the
 *                number of candidates hold id -1, dist +inf.
 * Inverted lists: list l holds entries list_off[l] .. list_off[l+1]-1 of
 * codes ([ntotal, M] bytes) and ids ([ntotal]).
 * probes: [nq, nprobe] list numbers (a negative entry is skipped).
 * scanned_out (optional, [nq]): number of vectors compared per query. */
/* Scan of one query's probed lists: cstart[p] = number of candidates in probes before p (nprobe + 1
 * entries, filled here); returns a malloc'd array of all candidates in probe order. */
static cand_t *scan_probed_lists(const float *q_row, const float *pq, int M, int ksub, int dsub,
                                 const int64_t *list_off, const uint8_t *codes, const int64_t *ids,
                                 const int32_t *probes, int nprobe, int64_t *cstart) {
    double *lut = (double *)malloc(sizeof(double) * (size_t)M * (size_t)ksub);
    build_lut(q_row, pq, M, ksub, dsub, lut);
    cstart[0] = 0;
    for (int p = 0; p < nprobe; ++p) {
        const int32_t l = probes[p];
        cstart[p + 1] = cstart[p] + (l < 0 ? 0 : list_off[l + 1] - list_off[l]);
    }
    const int64_t ncand = cstart[nprobe];
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(ncand > 0 ? ncand : 1));
#pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < nprobe; ++p) {
        const int32_t l = probes[p];
        if (l < 0) continue;
        const int64_t a = list_off[l], len = list_off[l + 1] - a;
        for (int64_t i = 0; i < len; ++i) {
            const uint8_t *code = codes + (a + i) * M;
            double acc = 0.0;
            for (int m = 0; m < M; ++m) acc += lut[m * ksub + code[m]];
            cand[cstart[p] + i].d = (float)acc;
            cand[cstart[p] + i].id = ids[a + i];
        }
    }
    free(lut);
    return cand;
}

void oracle_search_with_probes(const float *q, int64_t nq, int d, const float *pq, int M, int ksub,
                               const int64_t *list_off, const uint8_t *codes, const int64_t *ids,
                               const int32_t *probes, int nprobe, int k, float *out_dist, int64_t *out_ids,
                               int64_t *scanned_out) {
    const int dsub = d / M;
    int nthreads = oracle_num_threads();
#pragma omp parallel for schedule(dynamic, 1) if (nq >= nthreads)
    for (int64_t qi = 0; qi < nq; ++qi) {
        int64_t *cstart = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nprobe + 1));
        cand_t *cand = scan_probed_lists(q + qi * d, pq, M, ksub, dsub, list_off, codes, ids, probes + qi * nprobe,
                                         nprobe, cstart);
        const int64_t ncand = cstart[nprobe];
        /* keep the k smallest by (dist, id): sorted insertion */
        cand_t *best = (cand_t *)malloc(sizeof(cand_t) * (size_t)k);
        int nb = 0;
        for (int64_t c = 0; c < ncand; ++c) {
            if (nb == k && !cand_less(&cand[c], &best[k - 1])) continue;
            int pos = nb < k ? nb : k - 1;
            while (pos > 0 && cand_less(&cand[c], &best[pos - 1])) { best[pos] = best[pos - 1]; --pos; }
            best[pos] = cand[c];
            if (nb < k) ++nb;
        }
        for (int r = 0; r < k; ++r) {
            out_dist[qi * k + r] = r < nb ? best[r].d : INFINITY;
            out_ids[qi * k + r] = r < nb ? best[r].id : -1;
        }
        if (scanned_out) scanned_out[qi] = ncand;
        free(best); free(cand); free(cstart);
    }
}

/* The same scan for one query, without the selection: distance and id of every candidate, in probe order
 * (out arrays sized for the sum of the probed lists' lengths).  Returns the number of candidates. */
int64_t oracle_scan_with_probes(const float *q_row, int d, const float *pq, int M, int ksub,
                                const int64_t *list_off, const uint8_t *codes, const int64_t *ids,
                                const int32_t *probes, int nprobe, float *out_dist, int64_t *out_ids) {
    int64_t *cstart = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nprobe + 1));
    cand_t *cand = scan_probed_lists(q_row, pq, M, ksub, d / M, list_off, codes, ids, probes, nprobe, cstart);
    const int64_t ncand = cstart[nprobe];
    for (int64_t c = 0; c < ncand; ++c) { out_dist[c] = cand[c].d; out_ids[c] = cand[c].id; }
    free(cand); free(cstart);
    return ncand;
}

/* Full search: coarse quantiser, then the scan above. */
void oracle_search(const float *q, int64_t nq, int d, const float *coarse, int64_t nlist, const float *pq,
                   int M, int ksub, const int64_t *list_off, const uint8_t *codes, const int64_t *ids,
                   int nprobe, int k, float *out_dist, int64_t *out_ids, int32_t *probes_out,
                   int64_t *scanned_out) {
    int32_t *probes = probes_out ? probes_out : (int32_t *)malloc(sizeof(int32_t) * (size_t)nq * (size_t)nprobe);
    oracle_coarse(q, nq, d, coarse, nlist, nprobe, probes, NULL);
    oracle_search_with_probes(q, nq, d, pq, M, ksub, list_off, codes, ids, probes, nprobe, k, out_dist,
                              out_ids, scanned_out);
    if (!probes_out) free(probes);
}

/* ------------------------------------------------------------------ */
/* Exact k nearest neighbours by squared L2 distance over raw vectors
 * (what IVF-PQ approximates; used for recall and for pinning the oracle). */
void oracle_brute_force_knn(const float *x, int64_t n, int d, const float *q, int64_t nq, int k,
                            float *out_dist, int64_t *out_ids) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t qi = 0; qi < nq; ++qi) {
        cand_t *best = (cand_t *)malloc(sizeof(cand_t) * (size_t)k);
        int nb = 0;
        for (int64_t i = 0; i < n; ++i) {
            double acc = 0.0;
            for (int t = 0; t < d; ++t) {
                const double diff = (double)q[qi * d + t] - (double)x[i * d + t];
                acc += diff * diff;
            }
            cand_t c = { (float)acc, i };
            if (nb == k && !cand_less(&c, &best[k - 1])) continue;
            int pos = nb < k ? nb : k - 1;
            while (pos > 0 && cand_less(&c, &best[pos - 1])) { best[pos] = best[pos - 1]; --pos; }
            best[pos] = c;
            if (nb < k) ++nb;
        }
        for (int r = 0; r < k; ++r) {
            out_dist[qi * k + r] = r < nb ? best[r].d : INFINITY;
            out_ids[qi * k + r] = r < nb ? best[r].id : -1;
        }
        free(best);
    }
}

/* Decoded vector of a code: the concatenation of the selected sub-centres. */
void oracle_decode(const uint8_t *codes, int64_t n, const float *pq, int M, int ksub, int dsub, float *x_out) {
    for (int64_t i = 0; i < n; ++i)
        for (int m = 0; m < M; ++m)
            memcpy(x_out + (i * M + m) * dsub, pq + ((int64_t)m * ksub + codes[i * M + m]) * dsub,
                   sizeof(float) * (size_t)dsub);
}

/* ================================================================== */
/* Residual variant (the inverted-file ADC of the product-quantisation
 * method the paper cites for its index, Section 3.2 S3): a database vector
 * x in list l is stored as the code of its residual x - c_l to the list
 * centre, and a query is compared with it through the residual of the
 * query to the same centre:
 *     dist(q, x) = sum_m | (q - c_l)_m - pq[m][code_x[m]] |^2 .
 * Everything else (lists, probes, k-selection, ties) is as above.  The
 * residual itself is the single fp32 subtraction x - c_l (it is an input of
 * the quantiser, which is defined on fp32 vectors); sums are fp64. */

/* residual_out[i] = x_i - coarse[lists[i]], one fp32 subtraction per coordinate. */
void oracle_residuals(const float *x, int64_t n, int d, const float *coarse, const int32_t *lists, float *residual_out) {
    for (int64_t i = 0; i < n; ++i) {
        const float *c = coarse + (int64_t)lists[i] * d;
        for (int t = 0; t < d; ++t) residual_out[i * d + t] = x[i * d + t] - c[t];
    }
}

/* list_out[i] = nearest coarse centre; codes_out[i] = code of the residual to it. */
void oracle_encode_residual(const float *x, int64_t n, int d, const float *coarse, int64_t nlist, const float *pq,
                            int M, int ksub, int32_t *list_out, uint8_t *codes_out) {
    oracle_assign(x, n, d, d, coarse, nlist, list_out, NULL);
    float *r = (float *)malloc(sizeof(float) * (size_t)n * (size_t)d);
    oracle_residuals(x, n, d, coarse, list_out, r);
    oracle_encode(r, n, d, coarse, nlist, pq, M, ksub, NULL, codes_out);
    free(r);
}

/* Scan of one query's probed lists, residual variant; same outputs as scan_probed_lists. */
static cand_t *scan_probed_lists_residual(const float *q_row, int d, const float *coarse, const float *pq, int M, int ksub,
                                          const int64_t *list_off, const uint8_t *codes, const int64_t *ids,
                                          const int32_t *probes, int nprobe, int64_t *cstart) {
    const int dsub = d / M;
    cstart[0] = 0;
    for (int p = 0; p < nprobe; ++p) {
        const int32_t l = probes[p];
        cstart[p + 1] = cstart[p] + (l < 0 ? 0 : list_off[l + 1] - list_off[l]);
    }
    const int64_t ncand = cstart[nprobe];
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(ncand > 0 ? ncand : 1));
#pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < nprobe; ++p) {
        const int32_t l = probes[p];
        if (l < 0) continue;
        /* the query's residual to this list's centre (fp32, like the stored vectors' residuals), its table */
        float *rq = (float *)malloc(sizeof(float) * (size_t)d);
        double *lut = (double *)malloc(sizeof(double) * (size_t)M * (size_t)ksub);
        for (int t = 0; t < d; ++t) rq[t] = q_row[t] - coarse[(int64_t)l * d + t];
        build_lut(rq, pq, M, ksub, dsub, lut);
        const int64_t a = list_off[l], len = list_off[l + 1] - a;
        for (int64_t i = 0; i < len; ++i) {
            const uint8_t *code = codes + (a + i) * M;
            double acc = 0.0;
            for (int m = 0; m < M; ++m) acc += lut[m * ksub + code[m]];
            cand[cstart[p] + i].d = (float)acc;
            cand[cstart[p] + i].id = ids[a + i];
        }
        free(lut); free(rq);
    }
    return cand;
}

void oracle_search_residual_with_probes(const float *q, int64_t nq, int d, const float *coarse, const float *pq, int M,
                                        int ksub, const int64_t *list_off, const uint8_t *codes, const int64_t *ids,
                                        const int32_t *probes, int nprobe, int k, float *out_dist, int64_t *out_ids) {
    for (int64_t qi = 0; qi < nq; ++qi) {
        int64_t *cstart = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nprobe + 1));
        cand_t *cand = scan_probed_lists_residual(q + qi * d, d, coarse, pq, M, ksub, list_off, codes, ids,
                                                  probes + qi * nprobe, nprobe, cstart);
        const int64_t ncand = cstart[nprobe];
        cand_t *best = (cand_t *)malloc(sizeof(cand_t) * (size_t)k);
        int nb = 0;
        for (int64_t c = 0; c < ncand; ++c) {
            if (nb == k && !cand_less(&cand[c], &best[k - 1])) continue;
            int pos = nb < k ? nb : k - 1;
            while (pos > 0 && cand_less(&cand[c], &best[pos - 1])) { best[pos] = best[pos - 1]; --pos; }
            best[pos] = cand[c];
            if (nb < k) ++nb;
        }
        for (int r = 0; r < k; ++r) {
            out_dist[qi * k + r] = r < nb ? best[r].d : INFINITY;
            out_ids[qi * k + r] = r < nb ? best[r].id : -1;
        }
        free(best); free(cand); free(cstart);
    }
}

/* The same scan for one query without the selection (every candidate, in probe order). */
int64_t oracle_scan_residual_with_probes(const float *q_row, int d, const float *coarse, const float *pq, int M, int ksub,
                                         const int64_t *list_off, const uint8_t *codes, const int64_t *ids,
                                         const int32_t *probes, int nprobe, float *out_dist, int64_t *out_ids) {
    int64_t *cstart = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nprobe + 1));
    cand_t *cand = scan_probed_lists_residual(q_row, d, coarse, pq, M, ksub, list_off, codes, ids, probes, nprobe, cstart);
    const int64_t ncand = cstart[nprobe];
    for (int64_t c = 0; c < ncand; ++c) { out_dist[c] = cand[c].d; out_ids[c] = cand[c].id; }
    free(cand); free(cstart);
    return ncand;
}
