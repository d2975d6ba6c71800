/*
 * lorann.h - C ABI of the MI355X (gfx950) implementation of LoRANN's query phase.
 *
 * LoRANN (arXiv 2410.18926) is clustering-based approximate nearest-neighbour search whose score computation
 * is reduced-rank regression: for a query q routed to cluster c, the inner products with the cluster's
 * points are estimated as (q'^T A_c) B_c with q' = P^T q (Sec. 3.2, 4.1), evaluated as two 8-bit integer
 * products with absmax scales (Sec. 3.3), followed by candidate selection and an exact re-rank (Sec. 2.2).
 *
 * Conventions shared by every entry point
 *   - Pointers may be host or device pointers unless stated otherwise; the library finds out which with
 *     hipPointerGetAttributes.  Device pointers must belong to the current HIP device.
 *   - The library never keeps a caller pointer: lorann_load_index copies everything it needs into device
 *     memory it owns; search inputs/outputs are only used during the call.
 *   - Return value: LORANN_OK (0) or a negative error code; on error the outputs are untouched and
 *     lorann_last_error() describes the problem (thread-local string, valid until the next failing call).
 *   - One search at a time per lane of an index (each lane owns a workspace; the plain entry points use lane 0).
 *     Calls on one index must come from one host thread at a time.  Distinct indexes are independent.
 *   - Work is enqueued on the index's stream (default: the null stream, see lorann_set_stream) and
 *     lorann_search returns after the results are complete (it synchronises that stream).
 */
#ifndef LORANN_H
#define LORANN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lorann_index lorann_index;   /* opaque; owns device memory */

/* Dissimilarity measures of Sec. 2.1.  Returned distances: LORANN_IP  -> -<q, c>,
 * LORANN_L2 -> squared Euclidean distance |q - c|^2, LORANN_COS -> 1 - <q, c> / |q| (corpus rows are
 * expected to be unit-norm, Sec. 3.1). */
enum { LORANN_IP = 0, LORANN_L2 = 1, LORANN_COS = 2 };

enum {
    LORANN_OK = 0,
    LORANN_E_INVAL = -1,        /* bad argument (NULL, size, range, layout) */
    LORANN_E_NOMEM = -2,        /* device or host allocation failed */
    LORANN_E_DEVICE = -3,       /* a HIP call failed, or no gfx950 device */
    LORANN_E_UNSUPPORTED = -4   /* valid request outside the implemented limits */
};

/* Limits of this implementation. */
#define LORANN_MAX_W 256         /* clusters probed per query */
#define LORANN_MAX_M 4096        /* candidates re-ranked per query */
#define LORANN_MAX_R 64          /* RRR rank (multiple of 8) */
#define LORANN_MAX_DP 1024       /* reduced dimension d' (multiple of 16) */
#define LORANN_LANES 4           /* searches of one index that can be in flight at once (lorann_search_lane) */

/*
 * lorann_load_index - copy an index to the GPU (Sec. 2.2 partition, Sec. 3.2-3.3 quantized factors,
 * Sec. 4.1 projection and d'-dimensional centroids) and prepare it for searching.
 *
 *   metric           LORANN_IP / LORANN_L2 / LORANN_COS
 *   n, d             corpus size (1 <= n < 2^31) and dimension (d >= 1)
 *   dp               reduced dimension d' (the paper's s); multiple of 16, <= LORANN_MAX_DP
 *   r                rank of the factors; multiple of 8, <= LORANN_MAX_R
 *   L                number of clusters (>= 1)
 *   centroids        [L][dp] float, row-major: cluster centroids in the projected space
 *   P                [d][dp] float, row-major: projection matrix (the paper's W_s, any rotation already
 *                    folded in); NULL means identity and requires dp == d
 *   A                [L][r][dp] int8: A_c transposed, i.e. element (c, j, i) is A_c[i][j]
 *   B                [n][r] int8: one r-byte code per corpus row (column of B_c), rows in cluster order
 *   scale_A, scale_B [L] float each: absmax step sizes, real A_c ~= scale_A[c] * A, same for B
 *   cluster_offsets  [L+1] int64: cluster c owns rows [cluster_offsets[c], cluster_offsets[c+1]);
 *                    non-decreasing, first 0, last n.  Empty clusters are allowed.
 *   corpus           [n][d] float, row-major, rows in the same cluster order (kept for the re-rank)
 *   ids              [n] int64 caller id of each row, or NULL (then the row number is returned)
 *
 * On success *out receives the index (release it with lorann_free_index).  Errors: LORANN_E_INVAL for NULL
 * or inconsistent arguments (including non-monotone offsets), LORANN_E_UNSUPPORTED beyond the limits above,
 * LORANN_E_NOMEM / LORANN_E_DEVICE from the runtime.  Nothing is allocated on failure.
 */
int lorann_load_index(lorann_index **out, int32_t metric, int64_t n, int32_t d, int32_t dp, int32_t r, int32_t L,
                      const float *centroids, const float *P, const int8_t *A, const int8_t *B,
                      const float *scale_A, const float *scale_B, const int64_t *cluster_offsets,
                      const float *corpus, const int64_t *ids);

/*
 * lorann_load_index_file - the same from a serialized index (the file the CPU reference implementation reads
 * too; the harness writes it).  Little-endian; every array starts at a multiple of 64 bytes:
 *   offset 0  char[8] "LRNIDX01";  8 int32 metric;  12 int32 d;  16 int32 dp;  20 int32 r;  24 int32 L;
 *   28 int32 flags (bit 0: P present, bit 1: ids present);  32 int64 n;  zero padding up to 64;
 *   then cluster_offsets, ids (if present), centroids, P (if present), A, B, scale_A, scale_B, corpus, with
 *   the element types and layouts of lorann_load_index.
 * `path` is a host string.  Errors: LORANN_E_INVAL for a missing, foreign or truncated file, otherwise those
 * of lorann_load_index.
 */
int lorann_load_index_file(lorann_index **out, const char *path);

/*
 * lorann_search - the query phase (Sec. 2.2 template with the score computation of Sec. 3.2-3.3, 4.1):
 * project each query, route it to its w nearest centroids, estimate the scores of all points of those
 * clusters with the 8-bit reduced-rank model, keep the m best (the paper's t), re-rank them with the exact
 * dissimilarity to the original query and return the k best.
 *
 *   queries    [nq][d] float, row-major
 *   nq         number of queries (0 is allowed and does nothing)
 *   k, w, m    1 <= k <= m <= LORANN_MAX_M;  1 <= w <= min(L, LORANN_MAX_W)
 *   out_ids    [nq][k] int64: ids of the neighbours, nearest first; ties by distance go to the lower id;
 *              slots beyond the number of scored points hold -1
 *   out_dists  [nq][k] float: their dissimilarities (see the metric enum), ascending; +inf where id is -1
 *
 * All selections break ties toward the lower index (cluster id, corpus row, returned id).  m larger than the
 * number of points in the selected clusters is legal: all of them become candidates.
 */
int lorann_search(lorann_index *ix, const float *queries, int64_t nq, int32_t k, int32_t w, int32_t m,
                  int64_t *out_ids, float *out_dists);

/*
 * lorann_search_async - lorann_search without the wait: the work is enqueued on the index's stream and the call
 * returns; out_ids / out_dists are complete once that stream has been synchronised (by the caller, or by any later
 * synchronous call on this index).  queries, out_ids and out_dists must be device pointers and must stay valid
 * until then.  Calls on one index execute in the order they were made (they share its workspace through the
 * stream), so a serving loop can enqueue the next batch while the GPU finishes the current one.
 * Errors: those of lorann_search, plus LORANN_E_INVAL for a host pointer.
 */
int lorann_search_async(lorann_index *ix, const float *queries, int64_t nq, int32_t k, int32_t w, int32_t m,
                        int64_t *out_ids, float *out_dists);

/*
 * lorann_search_lane - lorann_search_async on lane `lane` (0 <= lane < LORANN_LANES) of the index.  Every lane owns a
 * workspace; lane 0 runs on the index's stream (lorann_search_lane(ix, 0, ...) IS lorann_search_async), each other lane
 * on a stream the library creates for it (default priority).  Searches enqueued on different lanes run concurrently
 * on the GPU: the re-rank of one batch is bound by HBM, the stages before it mostly are not, so two or three batches
 * in flight raise the throughput of a serving loop.  Ordering: a lane starts a search only after everything enqueued
 * on the index's stream at the time of the call (where the caller produced the queries) has finished, and runs its own
 * searches in the order they were enqueued.  Results are complete on the index's stream after lorann_lane_join.
 * The index's data is shared and read-only; lorann_set_rerank, lorann_set_column_scales, lorann_profile_* and
 * lorann_free_index wait for all lanes first.  Errors: those of lorann_search_async, LORANN_E_INVAL for a bad lane.
 */
int lorann_search_lane(lorann_index *ix, int32_t lane, const float *queries, int64_t nq, int32_t k, int32_t w, int32_t m,
                       int64_t *out_ids, float *out_dists);

/*
 * lorann_search_noalloc - lorann_search_async for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and ordering as lorann_search_async (device
 * pointers only; enqueues on the index's stream and returns), but the call allocates nothing - no device memory, no
 * events, no streams: every intermediate buffer of the search (projected queries, codes, approximate centroid scores,
 * the counting-sort tables, the pairs' vectors and scales, candidate lists, the row unions and distances of the
 * re-rank) is a slice of ONE fixed region of LORANN_NOALLOC_SCRATCH_BYTES that is part of the library's device code;
 * each GPU the library runs on holds that region until the process ends.
 *   - A search whose buffers do not fit is refused with LORANN_E_UNSUPPORTED before anything is enqueued; the message
 *     states the bytes needed.  (The need grows with nq * (L + w * (r + 24) + m * (8 * 2 + 22)) roughly: 32 MiB hold
 *     about 2000 queries at L = 1024, w = 32, m = 200, or 256 queries at L = 16384, w = 64, m = 200.)
 *   - All indexes on a GPU share the region and it keeps the previous call's contents; the kernels clear what
 *     must start at zero.  Calls that overlap on one GPU (other streams, other indexes, other threads) race: run
 *     them one after the other on one stream, and not beside lorann_search_lane traffic that has not been joined.
 *   - Not available while profiling is enabled (LORANN_E_INVAL).  The current device must be the index's.
 */
#define LORANN_NOALLOC_SCRATCH_BYTES (32u << 20)
int lorann_search_noalloc(lorann_index *ix, const float *queries, int64_t nq, int32_t k, int32_t w, int32_t m,
                          int64_t *out_ids, float *out_dists);

/* Make the index's stream wait (on the device; the host does not block) for everything enqueued so far on `lane`.
 * After it, work enqueued on the index's stream - or a synchronisation of that stream - sees the lane's results. */
int lorann_lane_join(lorann_index *ix, int32_t lane);

/* The re-rank gather of one batch alone saturates HBM, so by default the gathers of different lanes take turns (each
 * waits, on the device, for the previous lane's gather) while all other stages of the lanes overlap freely; every
 * gather then runs at its full rate.  on = 0 lets gathers overlap as well: each launch takes longer, the throughput of
 * a loop over several lanes was measured a few percent higher.  Waits for all lanes first. */
int lorann_set_gather_turns(lorann_index *ix, int32_t on);

/* Release an index and its workspaces.  NULL is ignored. */
void lorann_free_index(lorann_index *ix);

/* Message of the last failing call on this thread ("" if none). */
const char *lorann_last_error(void);

/* Use `hip_stream` (a hipStream_t, e.g. the caller framework's current stream) for all later work of this
 * index.  NULL selects the null stream.  The stream must stay valid while the index uses it. */
int lorann_set_stream(lorann_index *ix, void *hip_stream);

/* Candidate selection normally runs batched by cluster (each cluster's codes are read once per batch) and
 * hands the rare queries it cannot finish to an exact per-query kernel; cluster selection (Sec. 2.2) normally
 * evaluates approximate centroid scores for all clusters and exact ones for a provably sufficient short list.
 * on != 0 makes every query take the per-query kernel, evaluates every centroid score exactly and re-ranks one
 * query at a time (same results, much slower); used to verify one path against the other. */
int lorann_set_exact_selection(lorann_index *ix, int32_t on);

/* How the approximate centroid scores of the screening (Sec. 2.2 routing; the result is the same exact ranking in
 * every mode) reach the selection:
 *   LORANN_SCREEN_MATRIX  all nq x L values are written to device memory and read back by the selection;
 *   LORANN_SCREEN_DIGEST  the bf16 product is computed twice and only digests are kept (minima of 256 disjoint
 *                         subsets of the clusters, then the values at or below a per-query threshold); needs
 *                         d' of 128, 192 or 256, L >= 1024 and w <= 128, otherwise the matrix route is taken;
 *   LORANN_SCREEN_AUTO    (default) digests for launches of at least 6144 queries over at least 4096 clusters.
 * Waits for the index's searches in flight.  Errors: LORANN_E_INVAL for an unknown mode. */
enum { LORANN_SCREEN_AUTO = 0, LORANN_SCREEN_MATRIX = 1, LORANN_SCREEN_DIGEST = 2 };
int lorann_set_screen_mode(lorann_index *ix, int32_t mode);

/*
 * lorann_set_column_scales - column-wise quantization, as Sec. 3.3 prints it: absmax quantization applied to EACH
 * COLUMN of A_c and of B_c, instead of the one step size per cluster and matrix that lorann_load_index takes.
 *   scale_A_columns  [L][r] float: real A_c[i][j] ~= scale_A_columns[c][j] * A[c][j][i]
 *   scale_B_points   [n] float: real code of corpus row t ~= scale_B_points[t] * B[t][:] (a column of B_c)
 * The codes given at load time must have been produced with these step sizes; scale_A / scale_B are then ignored.
 * The arithmetic of the first product's re-quantization changes with it (the step sizes no longer cancel):
 *   rho_j = R_j * (Delta_x * scale_A_columns[c][j]);  z = rint(rho * (127 / |rho|_inf)), clamped to +-127;
 *   sigma = |rho|_inf / 127;  score of point t = fma(Y_t, sigma' * scale_B_points[t], -bias_t)  with sigma' = sigma
 *   (2 sigma for LORANN_L2) - each operation one IEEE float operation in the order written.
 * NULL, NULL returns to the per-cluster step sizes.  The arrays are copied (host or device pointers).
 * Errors: LORANN_E_INVAL for one NULL of two or a negative / non-finite step size (index unchanged).
 */
int lorann_set_column_scales(lorann_index *ix, const float *scale_A_columns, const float *scale_B_points);

/*
 * lorann_set_first_rows - mixed-precision decomposition (Sec. 4.2): the first component of the projected query and
 * the first row of every A_c and B_c are not quantized.  Needs the column-wise step sizes (lorann_set_column_scales).
 *   first_row_A  [L][r] float: A_c[0][j], the row that meets the query's first component q'_0
 *   first_row_B  [n] float: B_c[0][t] for the column of B_c that belongs to corpus row t
 * The codes' first components (A[c][j][0], B[t][0]) are then not read, and the step sizes must have been formed
 * from the remaining components.  Arithmetic, each operation one IEEE float operation in the order written:
 *   codes of q' from q'_1.. alone (absmax over them; code 0 in position 0), Delta_x likewise;
 *   rho_j = fma(q'_0, first_row_A[c][j], R_j * (Delta_x * scale_A_columns[c][j]))  for every j;
 *   rho_0 stays a float;  z_0 = 0, (z_1..) = rint(rho * (127 / |rho_1..|_inf)),  sigma = |rho_1..|_inf / 127;
 *   score of point t = fma(rho_0', first_row_B[t], fma(Y_t, sigma' * scale_B_points[t], -bias_t))
 *   with (rho_0', sigma') = (rho_0, sigma), doubled for LORANN_L2.
 * NULL, NULL switches the decomposition off (so does lorann_set_column_scales(ix, NULL, NULL)).  The arrays are
 * copied (host or device pointers).
 * Errors: LORANN_E_INVAL for one NULL of two, a non-finite value, or when the index has no column-wise step sizes
 * (index unchanged).
 */
int lorann_set_first_rows(lorann_index *ix, const float *first_row_A, const float *first_row_B);

/*
 * lorann_set_rerank - choose what the last step of later searches reads (Sec. 2.2 re-ranking; default F32).
 *   LORANN_RERANK_F32   the float corpus given at load time;
 *   LORANN_RERANK_F16   a half-precision (IEEE binary16, round to nearest even) copy of it, half the bytes of the
 *                       step that dominates the search (Sec. 4.3: 16-bit floating point on the GPU).  Each stored
 *                       value is widened exactly and the arithmetic stays in float, so the result is the plain
 *                       re-rank over the rounded rows; candidates are unaffected.  The copy (2*n*d bytes) is made by
 *                       the first call that selects this mode and lives as long as the index.  LORANN_E_UNSUPPORTED
 *                       if a corpus value is not finite or exceeds 65504 in magnitude (mode unchanged).
 *   LORANN_RERANK_NONE  no re-ranking step (Sec. 7.1 memory usage, App. D.3): the k points of highest estimated
 *                       score are returned (ties at the boundary toward the lower corpus row), nearest first by
 *                       out_dists = -score (for LORANN_L2 the score is 2<q', x'> - |x|^2 as estimated, i.e. the
 *                       |q|^2 term is left out), ties toward the lower id.  The search's m argument is then taken
 *                       to be k, also for the layouts of lorann_search_stages.
 * Errors: LORANN_E_INVAL for an unknown mode, LORANN_E_NOMEM / LORANN_E_DEVICE from the runtime.
 */
enum { LORANN_RERANK_F32 = 0, LORANN_RERANK_F16 = 1, LORANN_RERANK_NONE = 2 };
int lorann_set_rerank(lorann_index *ix, int32_t mode);

/*
 * Intermediate results of one search, for verification against a reference implementation.  Every pointer
 * may be NULL (skipped) and may be a host or device pointer.  Layouts, with slot = query * w + rank:
 */
typedef struct lorann_stages {
    float *qproj;          /* [nq][dp]      projected queries q' (Sec. 4.1)                               */
    int8_t *q8;            /* [nq][dp]      absmax codes of q' (Sec. 3.3)                                 */
    float *dx;             /* [nq]          step size of each query's codes                               */
    int32_t *sel;          /* [nq][w]       selected clusters, nearest centroid first (Sec. 2.2)          */
    int8_t *z;             /* [nq][w][r]    re-quantized intermediate vectors of each pair (Sec. 3.3)     */
    float *sigma;          /* [nq][w]       combined scale of each pair: score = sigma * integer score    */
    int32_t *cand_rows;    /* [nq][m]       candidate corpus rows, unordered, -1 padded (Sec. 2.2)        */
    float *tau;            /* [nq]          estimated score of the m-th candidate found by the batched    */
                           /*               selection (-inf: fewer than m points); untouched otherwise    */
    int32_t *n_survivors;  /* [nq]          scores the batched selection still held when it finished      */
                           /*               (-1: the query was finished by the exact per-query kernel)    */
    const int64_t *y_off;  /* [nq*w + 1]    caller-chosen offsets into y (needs sel known beforehand)     */
    int32_t *y;            /* [y_off[nq*w]] int32 score accumulators of every point of every pair, in     */
                           /*               cluster row order: y[y_off[slot] + t] (Sec. 3.3, 4.2); written */
                           /*               by the batched matrix-core scoring kernel (by the per-query   */
                           /*               kernel when exact selection is forced)                        */
    float *rho0;           /* [nq][w]       unquantized first component of each pair's intermediate vector */
                           /*               (zeros unless lorann_set_first_rows is in force; Sec. 4.2)     */
    float *pmax;           /* [nq][w]       highest estimated score among the points of each pair's        */
                           /*               cluster, as the batched matrix-core scoring kernel found it    */
                           /*               (-inf: empty cluster); untouched when exact selection is forced */
} lorann_stages;

/* lorann_search that also exports the intermediate results named in `st`.  Same arguments and errors as
 * lorann_search; y_off[slot+1] - y_off[slot] must equal the size of the slot's cluster. */
int lorann_search_stages(lorann_index *ix, const float *queries, int64_t nq, int32_t k, int32_t w, int32_t m,
                         int64_t *out_ids, float *out_dists, const lorann_stages *st);

/*
 * Per-kernel timing of the searches of one index, taken with HIP events on the index's stream.
 * lorann_profile_enable(ix, 1) starts recording every kernel (and clears the totals), 2 records only the
 * re-rank gather kernel (two events per batch: negligible overhead inside a timed run), 3 only the int8
 * matrix-core scoring kernel (the B_c product), 0 stops.
 * lorann_profile_get writes up to `cap` records and returns how many kernels exist (or a negative error code).
 */
typedef struct lorann_kernel_time {
    char name[48];      /* kernel name */
    double ms;          /* total time of its launches since profiling was enabled */
    int64_t launches;
} lorann_kernel_time;

int lorann_profile_enable(lorann_index *ix, int32_t on);
int lorann_profile_get(lorann_index *ix, lorann_kernel_time *out, int32_t cap);
/* Number of queries that the batched selection handed to the exact per-query kernel since profiling was
 * enabled (-1 if ix is NULL). */
int64_t lorann_profile_fallback_queries(lorann_index *ix);

/* Corpus rows the re-rank of the latest batch on lane 0 actually fetched (Sec. 2.2 re-ranking): queries that are
 * neighbours in the visiting order share candidate rows and a shared row is fetched once per group, so this is
 * at most nq * m and at least the number of distinct candidate rows of the batch.  Multiply by the row size for the
 * bytes the gather kernel requests.  Waits for all work on the index.  -1: ix is NULL, or the latest batch did not
 * take the grouped re-rank. */
int64_t lorann_profile_gather_rows(lorann_index *ix);

#ifdef __cplusplus
}
#endif
#endif /* LORANN_H */
