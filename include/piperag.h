/*
 * piperag.h - C ABI of the MI355X IVF-PQ retrieval library.
 *
 * The library implements the retrieval step of retrieval-augmented generation as
 * the paper states it: a query vector goes in, the k closest database entries
 * (ids and distances) come out (Section 2, "Database construction").  The index
 * is IVF-PQ (Section 3.2, S3): the database is clustered into nlist inverted
 * lists, each vector is stored as a product-quantisation code of M bytes
 * (Section 3.1, O3; Appendix "Detailed Evaluation Setup", Software), and a query
 * scans the nprobe lists whose centres are closest to it.  nprobe is the knob
 * the paper's performance model tunes; piperag_latency_profile measures the
 * nprobe -> latency relation that model is fitted on.
 *
 * Conventions
 *   - Every function returns PIPERAG_OK (0) or a negative error code and never
 *     throws or aborts; piperag_last_error() gives a thread-local message.
 *   - Pointers named *_dev are device (HBM) memory owned by the caller, row-major,
 *     contiguous, 16-byte aligned.  Pointers named *_host are host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls that take a stream enqueue their work on it; unless stated otherwise
 *     they return without waiting, and results are valid once the caller has
 *     synchronised that stream.  The search calls allocate nothing.
 *   - Distance is squared L2 (no square root).  8 bits per sub-quantiser.  The PQ
 *     code quantises the raw vector, or, for an index created with residual = 1,
 *     the vector's residual to the centre of its list (the inverted-file ADC of
 *     the product-quantisation method the paper cites, Section 3.2, S3); the
 *     distance to a vector x of list l is then sum_m |(q - c_l)_m - pq[m][code_x[m]]|^2.
 *   - An index must not be searched from two streams at once: the search
 *     workspace belongs to the index.
 */
#ifndef PIPERAG_H
#define PIPERAG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PIPERAG_OK 0
#define PIPERAG_ERR_ARG (-1)   /* null pointer, size out of range, wrong state */
#define PIPERAG_ERR_OOM (-2)   /* device or host allocation failed */
#define PIPERAG_ERR_HIP (-3)   /* a HIP runtime call failed */
#define PIPERAG_ERR_FILE (-4)  /* unreadable, truncated or malformed index file */
#define PIPERAG_ERR_LIMIT (-5) /* nq / nprobe / k / ntotal beyond the limits given at creation */

typedef struct piperag_index piperag_index; /* opaque; owns its device memory and search workspace */

typedef struct piperag_params {
    int32_t d;          /* vector dimension, multiple of M */
    int32_t nlist;      /* number of inverted lists (coarse centres), 1 .. 2^20 */
    int32_t M;          /* sub-quantisers = bytes per code, 1 .. 128 */
    int32_t nbits;      /* bits per sub-quantiser; must be 8 */
    int64_t ntotal;     /* create: capacity in vectors (add fails beyond it); load: ignored */
    int32_t max_nq;     /* largest query batch a search call may pass (>= 1) */
    int32_t max_nprobe; /* largest nprobe (1 .. min(nlist, 1024)) */
    int32_t max_k;      /* largest k (1 .. 1024) */
    int32_t residual;   /* 0: the code quantises the vector itself; 1: its residual to the centre of its list */
} piperag_params;

/* ---- index life cycle ------------------------------------------------------------------- */

/* Reads an index file (layout below) into HBM and makes it searchable.  Only max_nq, max_nprobe and
 * max_k of `limits` are used.  File, little-endian: 64-byte header = "PRAGIVF1", u32 version (1), u32 d,
 * u32 nlist, u32 M, u32 nbits (8), u32 flags (bit 0: residual codes), u64 ntotal, zero padding; then centres f32 [nlist*d]; codebooks
 * f32 [M*256*(d/M)]; list lengths i64 [nlist]; codes u8 [ntotal*M], list after list; ids i64 [ntotal] in
 * the same order.  On success *out owns everything; free with piperag_ivf_free. */
int piperag_ivf_load(const char *path, const piperag_params *limits, piperag_index **out);

/* Creates an empty index from trained parameters (Section 3.2, S3: the clustering into nlist lists; the
 * product quantiser of Section 3.1, O3).  centroids_host: f32 [nlist*d]; pq_codebook_host: f32
 * [M*256*(d/M)], sub-quantiser-major.  Both are copied. */
int piperag_ivf_create(const piperag_params *params, const float *centroids_host, const float *pq_codebook_host,
                       piperag_index **out);

/* Index training.  The paper does not say how the lists and codebooks are trained (Section 3.2, S3 only
 * states that the database is clustered into nlist lists); this is Lloyd's k-means with a fixed number of
 * iterations: centre j starts as row init_rows_host[j] of x; each iteration assigns every row to its
 * nearest centre (as piperag_ivf_add does, see there; lower index on equal values) and replaces each centre by the
 * mean of its rows (coordinate sums are exact 2^-24 fixed-point integers, so the result does not depend on
 * summation order; coordinates must stay below 2^15 in magnitude); a centre without rows keeps its value.
 * x_dev f32: n rows of d coordinates, row stride ldx floats (a column slice of a wider matrix trains one
 * sub-quantiser).  centroids_out_dev f32 [K*d].  inertia_out_host f64 [iters] or NULL: sum of
 * row-to-centre distances seen by each iteration's assignment.  Allocates scratch; synchronises `stream`. */
int piperag_kmeans(const float *x_dev, int64_t n, int32_t d, int64_t ldx, int32_t K, int32_t iters,
                   const int64_t *init_rows_host, float *centroids_out_dev, double *inertia_out_host, void *stream);

/* Database construction (Section 2; Appendix, Software: each vector becomes a list number and M code
 * bytes): encodes n vectors x_dev f32 [n*d] on the GPU and appends them.  list(x) = nearest centre,
 * code[m] = nearest of the 256 centres of sub-quantiser m to the m-th slice of x; on equal distances the
 * lower index.  Arithmetic of the decision: with 128 lists or more and d >= 64, |c|^2 - 2 <x, c> from a
 * matrix-core product whose operands are carried as two fp16 parts each (22 significant bits: every product is
 * as accurate as an fp32 multiplication) shortlists the two best centres, and the fp32 direct-form distances
 * sum_t (x_t - c_t)^2 to those two decide; the result can differ from the exact nearest centre only where a
 * third centre lies within the expanded form's fp32 rounding error (a few 2^-24 |x||c|) of the best.  Smaller
 * shapes use the direct form throughout.  Codes: fp32 |p|^2 - 2 <x_m, p> on the matrix
 * cores (direct form when d/M < 4).  ids_dev: i64 [n] or NULL for consecutive ids continuing from the number already added.
 * Enqueues on `stream`; x_dev and ids_dev must stay valid until the stream has passed the call. */
int piperag_ivf_add(piperag_index *index, const float *x_dev, int64_t n, const int64_t *ids_dev, void *stream);

/* Appends n already-encoded vectors: lists_dev i32 [n] (each in 0..nlist-1, checked), codes_dev u8 [n*M],
 * ids_dev i64 [n] or NULL.  Synchronises `stream` (for the check). */
int piperag_ivf_add_encoded(piperag_index *index, const int32_t *lists_dev, const uint8_t *codes_dev,
                            const int64_t *ids_dev, int64_t n, void *stream);

/* Two-pass build, for databases whose per-vector staging area (M + 12 bytes per vector until finalize) would not
 * fit beside the finished index: the caller presents the database twice, in the same order (any tiling).
 *   pass 1  piperag_ivf_count(index, x_dev, n, stream)        assigns the n vectors to their lists, keeps the list
 *                                                             numbers (4 bytes per vector) and counts the lists;
 *           piperag_ivf_reserve(index, stream)                sizes the lists and allocates the index (synchronises);
 *   pass 2  piperag_ivf_place(index, x_dev, n, ids_dev, stream)  computes the codes of the next n vectors and puts
 *                                                             them, in order, straight into their lists;
 *           piperag_ivf_finalize(index, stream)               as below; every counted vector must have been placed.
 * The result is identical to that of piperag_ivf_add + finalize on the same sequence.  ids_dev NULL numbers the
 * vectors by position.  A build uses either piperag_ivf_add / add_encoded or count / place, not both
 * (PIPERAG_ERR_ARG).  Peak memory is the index plus 4 bytes per vector. */
int piperag_ivf_count(piperag_index *index, const float *x_dev, int64_t n, void *stream);
int piperag_ivf_reserve(piperag_index *index, void *stream);
int piperag_ivf_place(piperag_index *index, const float *x_dev, int64_t n, const int64_t *ids_dev, void *stream);

/* Groups everything added so far into inverted lists (inside a list: order of addition) and builds the
 * scan layout.  Synchronises `stream`; allocates.  Afterwards the index is searchable and closed to adds. */
int piperag_ivf_finalize(piperag_index *index, void *stream);

/* Writes a finalized index in the file layout of piperag_ivf_load. */
int piperag_ivf_save(const piperag_index *index, const char *path);

void piperag_ivf_free(piperag_index *index);

/* ---- search ----------------------------------------------------------------------------- */

/* Batched IVF-PQ search (Section 3.2, S3: nprobe of the nlist lists are selected and the vectors inside
 * them are compared with the query; Section 2: the k closest are returned).
 *   queries_dev f32 [nq*d];  out_dist_dev f32 [nq*k];  out_ids_dev i64 [nq*k].
 * Per query: ascending by (distance, id); distance = sum over m of the squared distance between the
 * query's m-th slice and the centre the code selects; when the probed lists hold fewer than k vectors
 * the remaining slots are id -1, distance +inf.  Which vectors are returned when more of them share the
 * k-th distance, bit for bit, than there are places left: those stored first in the index (the scan
 * selects by (distance, position), deterministically); only the order of the returned rows is by id.  1 <= nq <= max_nq, 1 <= nprobe <= min(nlist,
 * max_nprobe), 1 <= k <= max_k, else PIPERAG_ERR_LIMIT / PIPERAG_ERR_ARG.  nq == 0 is a no-op. */
int piperag_ivfpq_search(const piperag_index *index, const float *queries_dev, int32_t nq, int32_t nprobe,
                         int32_t k, float *out_dist_dev, int64_t *out_ids_dev, void *stream);

/* For callers that cannot allocate device memory or create streams and events (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it): the same search as piperag_ivfpq_search, same kernels, same
 * results, but every intermediate (coarse distances, probe tables, lookup tables, partial results, counters)
 * lives in a static device array of PIPERAG_STATIC_SCRATCH_BYTES that the library's code object brings with it
 * (each GPU the library runs on holds its own copy until the process ends).  The call allocates nothing and ignores the index's
 * max_nq / max_nprobe / max_k: it is limited by the array instead - the scratch needed grows with nq * nlist,
 * nq * 256 * M and (512 + 10 * nq) * (k + 64); a call that needs more returns PIPERAG_ERR_LIMIT (e.g. nq = 16,
 * nprobe = 128, k = 100 on 65,536 lists with 64-byte codes needs 7 MiB).  The index must have been created in
 * this process (creation sets up the array's address on the index's device).  All calls on one GPU share that
 * GPU's array: two such calls that overlap in time on one GPU, from any streams or indexes, race; calls on one
 * stream are safe.  piperag_search_stats afterwards reports this call.  Stage timing and graph replay do not
 * apply. */
#define PIPERAG_STATIC_SCRATCH_BYTES (16u << 20)
int piperag_ivfpq_search_static(const piperag_index *index, const float *queries_dev, int32_t nq, int32_t nprobe,
                                int32_t k, float *out_dist_dev, int64_t *out_ids_dev, void *stream);

/* The performance model's retrieval side (Section 3.2, S3: search latency is modelled by linear
 * regression on nprobe): runs the search above for each nprobes_host[i] (`reps` timed repetitions after
 * two warm-up runs, HIP events on `stream`), writes the median latency in milliseconds to
 * out_p50_ms_host[i] and the least-squares line latency = fit[0] + fit[1]*nprobe to out_fit_host[2].
 * Synchronises `stream`.  Scratch outputs for the searches are taken from the index workspace. */
int piperag_latency_profile(const piperag_index *index, const float *queries_dev, int32_t nq,
                            const int32_t *nprobes_host, int32_t n_nprobes, int32_t k, int32_t reps,
                            float *out_p50_ms_host, float *out_fit_host, void *stream);

/* ---- performance model (host arithmetic, no GPU work) -------------------------------------- */

/* Inversion of the retrieval performance model (Section 3.2, S3: given the time T(C) it takes to generate
 * the next token chunk, derive the maximal nprobe whose predicted retrieval latency stays within it).
 * fit_host[2] = the line latency_ms = fit[0] + fit[1]*nprobe (as written by piperag_latency_profile);
 * overhead_ms = the part of the retrieval latency outside the search (network, query encoding; >= 0).
 * *out_nprobe = the largest nprobe in 1..nprobe_cap with overhead_ms + fit[0] + fit[1]*nprobe <= budget_ms;
 * when even nprobe = 1 does not fit, *out_nprobe = 1 and *out_fits = 0 (a retrieval is always made),
 * otherwise *out_fits = 1.  A slope <= 0 (latency does not grow with nprobe) gives nprobe_cap if nprobe = 1
 * fits.  out_predicted_ms (optional) = the predicted latency at the chosen nprobe, overhead included.
 * PIPERAG_ERR_ARG for NULL pointers, nprobe_cap < 1 or non-finite inputs. */
int piperag_max_nprobe(const float *fit_host, float overhead_ms, float budget_ms, int32_t nprobe_cap,
                       int32_t *out_nprobe, int32_t *out_fits, float *out_predicted_ms);

/* End-to-end generation latency projected for faster retrieval or inference hardware (Appendix
 * "Performance Modeling for Future Hardware").  inference_ms_host[c], retrieval_ms_host[c]: measured
 * latency of generating token chunk c and of the retrieval issued for it, c = 0..nchunks-1; each is divided
 * by its speed-up factor (> 0).  Sequential generation (the baseline that waits for every retrieval) takes
 * the sum of all inference and retrieval times; pipelined generation takes inference + retrieval for the
 * first chunk, where the pipeline is not yet active, and max(inference, retrieval) for every later chunk.
 * Sums are accumulated in double precision in chunk order.  nchunks >= 1. */
int piperag_project_latency(const float *inference_ms_host, const float *retrieval_ms_host, int32_t nchunks,
                            float inference_speedup, float retrieval_speedup, double *out_sequential_ms,
                            double *out_pipelined_ms);

/* A stream whose kernels run only on compute units first_cu .. first_cu + ncu - 1 of the current device
 * (numbered as the driver's compute-unit mask numbers them; on this GPU consecutive numbers go round the XCDs),
 * at the default priority.  The paper hides the retrieval behind the generation of the next tokens by running it
 * on a server of its own (Section 3.2, S1); on one GPU the same is had by giving the search such a stream and the
 * generation a stream on the remaining compute units: every call of this library that takes a stream then runs
 * in that slice (a search is launched on the given stream only).  piperag_latency_profile on the same stream
 * gives the latency line of the slice.  *out_stream is a hipStream_t; destroy it with piperag_stream_destroy. */
int piperag_stream_create_cu_slice(int32_t first_cu, int32_t ncu, void **out_stream);
int piperag_stream_destroy(void *stream);

/* ---- stage taps (each step of the search path by itself, for checking) ------------------- */

/* Coarse quantiser (the index-scan term of the latency model, Section 3.2, S3): the nprobe closest
 * centres per query ordered by (distance, list).  out_lists_dev i32 [nq*nprobe]; out_dist_dev f32
 * [nq*nprobe] or NULL. */
int piperag_ivf_coarse(const piperag_index *index, const float *queries_dev, int32_t nq, int32_t nprobe,
                       int32_t *out_lists_dev, float *out_dist_dev, void *stream);

/* Per-query lookup tables: out_lut_dev f32 [nq*M*256], entry [q][m][j] = squared distance between the
 * m-th slice of query q and centre j of sub-quantiser m. */
int piperag_ivf_lut(const piperag_index *index, const float *queries_dev, int32_t nq, float *out_lut_dev,
                    void *stream);

/* Search with the probe lists given by the caller instead of the coarse quantiser: probes_dev i32
 * [nq*nprobe]; an entry outside 0..nlist-1, or equal to an earlier entry of the same query, is skipped. */
int piperag_ivfpq_search_probes(const piperag_index *index, const float *queries_dev, int32_t nq,
                                const int32_t *probes_dev, int32_t nprobe, int32_t k, float *out_dist_dev,
                                int64_t *out_ids_dev, void *stream);

/* Encoder by itself (no append): out_lists_dev i32 [n], out_codes_dev u8 [n*M]; either may be NULL. */
int piperag_ivf_encode(const piperag_index *index, const float *x_dev, int64_t n, int32_t *out_lists_dev,
                       uint8_t *out_codes_dev, void *stream);

/* Copies one inverted list to the host in canonical form (row i = the M code bytes of its i-th vector).
 * *len_out receives the length; codes_host (u8 [len*M]) and ids_host (i64 [len]) may be NULL to query
 * the length only.  Synchronous. */
int piperag_ivf_get_list(const piperag_index *index, int32_t list, int64_t *len_out, uint8_t *codes_host,
                         int64_t *ids_host);

/* Lengths of all lists: out_host i64 [nlist].  Synchronous. */
int piperag_ivf_list_lengths(const piperag_index *index, int64_t *out_host);

/* Work done by the most recent search call on this index (valid after its stream has been
 * synchronised): vectors compared and their code bytes (vectors * M). */
int piperag_search_stats(const piperag_index *index, int64_t *scanned_vectors, int64_t *scanned_code_bytes);

/* Per-stage timing of the retrieval latency model's terms (Section 3.2, S3: index scan + vector scan).
 * When enabled, every search call records HIP events around its stages on its stream;
 * piperag_stage_times synchronises on them and writes the most recent call's milliseconds:
 * [0] coarse quantiser, [1] top-nprobe selection, scan plan and work sharing, [2] lookup
 * tables, [3] list scan with k-selection, merge of
 * the query's partial results and id gather (one kernel).  Stages [0]+[1] are the index-scan term,
 * [2]+[3] the vector-scan term. */
#define PIPERAG_NSTAGES 4
int piperag_set_stage_timing(piperag_index *index, int enable);
int piperag_stage_times(const piperag_index *index, float *out_ms_host /* [PIPERAG_NSTAGES] */);

/* Graph replay of repeated search calls (off by default).  For callers that issue one search at a time
 * and wait for it (the paper's serving loop retrieves for one sequence between generation steps, Section
 * 3.1): when enabled, a search call whose arguments (query, probe and output pointers, nq, nprobe, k)
 * repeat an earlier call's is captured into a HIP graph the second time it is seen and replayed with a
 * single launch from then on: one host call per search instead of four, for callers whose host thread is
 * the scarce resource.  It does not shorten the search itself (on an MI355X a waited-for single query took
 * 93 us replayed against 89 us launched plainly, and back-to-back calls lose about 10 us each).  The buffers'
 * contents may change between calls; their addresses must stay valid while replay is enabled.  Up to 8
 * distinct calls are remembered (least recently used is dropped).  Disabling destroys the cached graphs.
 * Stage timing bypasses replay. */
int piperag_set_graph_replay(piperag_index *index, int enable);

/* How the scan reads the code blocks (Section 3.2, S3: the vector-scan term of the latency).  mode < 0
 * (default): by the shape of the index - indexes with 4 GiB of codes or more whose lists average less than
 * 4 MiB of codes are read with non-temporal loads, because nothing a search reads is still cached when it
 * is needed again and streaming the codes past the caches is then faster (measured); other indexes are
 * read with ordinary loads so that lists probed by several queries of a batch, or again by the next call,
 * are found in the caches.  mode = 0: always
 * ordinary loads; mode > 0: always non-temporal loads.  Results do not depend on the mode.  Cached graphs
 * of repeated calls are dropped. */
int piperag_set_scan_streaming(piperag_index *index, int mode);

/* Compute units the searches on this index may use: ncu <= 0 (default) all of the device's, else that many -
 * for searches given a stream from piperag_stream_create_cu_slice.  The selection and scan launches are sized to
 * it (two scan workgroups per compute unit; 512 workgroups on a 32-unit slice would run in eight rounds, each
 * paying the launch's fixed costs).  Results do not depend on it.  Cached graphs of repeated calls are dropped. */
int piperag_set_compute_units(piperag_index *index, int32_t ncu);

/* Number of vectors in the index. */
int64_t piperag_ivf_ntotal(const piperag_index *index);

const char *piperag_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PIPERAG_H */
