/*
 * knng.h -- C ABI of libknng: single-GPU k-nearest-neighbour-graph construction
 * for AMD MI355X (gfx950), after the local kNNG construction of SOLANET
 * (paper Sec. 3.1 "NN-Descent" and Sec. 3.1.1 "Lock-Free GPU-based NN-Descent"),
 * and the local building blocks of its refinement across partitions.
 *
 *   knng_build_knn_graph[_u8|_f16]  approximate k-NN graph            (Sec. 3.1, 3.1.1)
 *   knng_brute_knn                  exact k-NN rows                    (Sec. 2.1, 5.3.1)
 *   knng_graph_recall               recall of one graph against another (Sec. 2.1, 5.4.3)
 *   knng_merge_graphs               rows updated with search results   (Sec. 4.3, 4.4)
 *   knng_optimize_graph             k-NN graph -> search graph          (Sec. 3.3)
 *   knng_graph_search[_u8]          graph search for query points      (Sec. 3.2)
 *
 * Conventions for every entry point
 *   - Pointers named *_dev are DEVICE pointers (hipMalloc-class memory, as the
 *     paper passes its dataset: Sec. 5.3.1); pointers named *_host are HOST
 *     pointers.  The caller owns every buffer; the library never frees or keeps
 *     a caller pointer after the call returns.
 *   - The dataset is n feature vectors of equal dimensionality d, a row-major
 *     fp32 matrix points[n][d] (Sec. 2.1).  It is read-only and never copied.
 *   - A graph is two row-major matrices ids[rows][k] (int32) and
 *     dists[rows][k] (fp32), exactly k entries per row, rows ascending under
 *     (distance, id) (Sec. 2.1: G_id and G_dis).
 *   - Distances (Sec. 2.1: sigma >= 0, smaller = more similar):
 *       KNNG_METRIC_L2SQ     sum_t (a_t - b_t)^2
 *       KNNG_METRIC_IP_UNIT  max(0, 1 - <a,b>); the caller guarantees unit rows
 *       KNNG_METRIC_COSINE   max(0, 1 - <a,b> / sqrt(|a|^2 |b|^2)) for rows of any length (a
 *                            similarity turned into a dissimilarity, Sec. 2.1); a zero row is at
 *                            distance 1 from every row.  <a,b>, |a|^2 and |b|^2 are each
 *                            accumulated as below; quotient and root in fp64.  Accepted by
 *                            knng_build_knn_graph and knng_brute_knn[_base] (fp32 rows); the
 *                            build needs n*d*4 more bytes of workspace for unit-length copies
 *                            of the rows, which the joins work on.
 *     Every distance WRITTEN to an output is accumulated in fp64 over
 *     t = 0..d-1 in index order with fused multiply-add and rounded once to
 *     fp32.  Inputs must be finite; NaN/Inf inputs give unspecified ordering
 *     (never a fault).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it; each call has completed on return.
 *   - Return value: 0 (KNNG_OK) or a negative KNNG_E* code; knng_strerror()
 *     gives text.  On KNNG_EINVAL / KNNG_EWORKSPACE nothing has been written.
 *   - n <= 2^31 - 1; all byte offsets are 64-bit.
 *   - Calls that overlap in time must not share a workspace.
 */
#ifndef KNNG_H
#define KNNG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KNNG_VERSION 2

enum {
    KNNG_OK = 0,
    KNNG_EINVAL = -1,      /* bad argument (null pointer, n < 2, k < 1, k > n-1, ...) */
    KNNG_EWORKSPACE = -2,  /* workspace missing or smaller than knng_*_workspace_bytes */
    KNNG_EHIP = -3,        /* a HIP call failed; knng_strerror(KNNG_EHIP) has its text */
    KNNG_ETOOLARGE = -4,   /* more input than an entry point with fixed scratch memory takes */
    KNNG_ECHECK = -5       /* knng_params_t.check_rows: a row broke an invariant (a bug in the
                              library); the outputs are written all the same                  */
};

enum { KNNG_METRIC_L2SQ = 0, KNNG_METRIC_IP_UNIT = 1, KNNG_METRIC_COSINE = 2 };

#define KNNG_MAX_K 64            /* largest k / k_build / cand_cap */
#define KNNG_STATS_MAX_ITERS 128 /* per-iteration records kept in knng_stats_t */

/* Filled by knng_build_knn_graph when params->stats_host != NULL (host memory). */
typedef struct knng_stats {
    int32_t iterations;        /* refinement iterations run                        */
    int32_t converged;         /* 1: stopped by updates < delta*K*n; 0: max_iters  */
    uint64_t updates[KNNG_STATS_MAX_ITERS]; /* accepted updates per iteration       */
    float join_ms[KNNG_STATS_MAX_ITERS];    /* local-join kernel time per iteration */
    uint64_t join_rows[KNNG_STATS_MAX_ITERS]; /* vectors gathered by that launch    */
    float ms_init, ms_sample, ms_join, ms_merge, ms_finalize; /* summed kernel ms   */
    float ms_total;            /* first enqueue to last completion                  */
    uint64_t offers;           /* candidates offered to candidate lists (atomics), whole build */
    uint64_t pairs;            /* pairs the local joins had to evaluate (new x new unordered
                                  plus new x old per joined point), whole build      */
    uint64_t cand_kept;        /* candidate slots the merges found occupied, whole build.
                                  offers - cand_kept offers did not survive in their slot:
                                  the same neighbour offered again by another join, or a
                                  different neighbour that shares the slot and is closer --
                                  the second kind is a dropped candidate (Sec. 3.1.1: a
                                  fixed-size list may drop true neighbours), so the
                                  difference bounds the drops from above                */
    uint64_t joined;           /* local joins done (points with a new member around them), whole build */
    uint64_t rejoined;         /* joins done twice, whole build: points whose join in reduced
                                  precision (long fp32 rows, or samples above 16: the Gram
                                  block on bf16 halves) chose a partner far closer to a member
                                  than both are to the point, and was repeated in fp32        */
    uint64_t row_violations;   /* knng_params_t.check_rows: invariants found broken, whole build */
} knng_stats_t;

/*
 * Parameters of the build (Sec. 3.1: k, delta, rho; Sec. 5.3.1: iteration cap and
 * a build degree larger than the target k).  Zero in a numeric field selects the
 * default.  struct_size must be sizeof(knng_params_t) (ABI check).
 */
typedef struct knng_params {
    uint32_t struct_size;
    int32_t k_build;          /* K: internal degree, k <= K <= min(n-1, KNNG_MAX_K); default k.
                                 The result is the nearest k of the K (Sec. 5.3.1).           */
    float rho;                /* sampling rate in (0,1]; default 0.5 (Sec. 3.1, 5.4)           */
    float delta;              /* stop when an iteration accepts < delta*K*n updates;
                                 default 1e-4; negative = never stop early (Sec. 3.1)          */
    int32_t max_iters;        /* default 100 (Sec. 5.3.1); negative = 0 iterations             */
    int32_t cand_cap;         /* slots of each point's fixed-size candidate list
                                 (Sec. 3.1.1), 1..KNNG_MAX_K; default min(2K, KNNG_MAX_K): a
                                 slot is a lane of the merging wavefront, so K = 64 has K
                                 slots, not 2K                                                 */
    uint64_t seed;
    const int32_t *init_ids_dev; /* optional warm start [n][K] (device); entries that are out
                                 of range, self or repeated are replaced by random ids; NULL =
                                 random initial graph (Sec. 3.1)                              */
    void *stream;             /* hipStream_t; NULL = default stream                            */
    void *workspace_dev;      /* device scratch, >= knng_build_workspace_bytes(), 256-B aligned */
    uint64_t workspace_bytes;
    knng_stats_t *stats_host; /* optional                                                      */
    void *pinned_host;        /* optional: 64 bytes of page-locked host memory (hipHostMalloc
                                 class, 8-byte aligned) for the convergence counter the host
                                 reads once per iteration; NULL = the call allocates and frees
                                 its own, which costs a page-locked allocation per build       */
    uint32_t check_rows;      /* debug mode, nonzero: after every merge a kernel checks every
                                 point's state -- row sorted by (distance, id), ids distinct,
                                 in range and not the point, distances real and >= 0, the
                                 row's farthest distance as the join will read it, candidate
                                 slots empty again, sample sizes <= ceil(rho K), sampled ids in
                                 range, every id of the row in the row's signature (the joins
                                 rely on it: Sec. 3.1.1's single owner leaves the row itself
                                 race-free, these are what the lock-free parts must keep).
                                 A violation makes the call return KNNG_ECHECK.  Slow.          */
    uint32_t reserved;        /* 0 */
} knng_params_t;

/* Device scratch needed by knng_build_knn_graph for these sizes (0 on bad arguments).
 * For KNNG_METRIC_COSINE add knng_build_cosine_extra_bytes(n, d). */
uint64_t knng_build_workspace_bytes(int64_t n, int32_t d, int32_t k, const knng_params_t *params);
uint64_t knng_build_cosine_extra_bytes(int64_t n, int32_t d);

/*
 * Approximate k-NN graph of the n points (Sec. 3.1, 3.1.1).
 *
 * Random initial graph; then per iteration: per-point sampling of new and old
 * neighbours (rate rho) with reverse edges; a local join per point that
 * evaluates the distances among its sampled neighbours; every close pair is
 * offered, lock-free, to the two points' fixed-size candidate lists when it
 * beats their current farthest neighbour; one owner per point folds its list
 * into its row and clears it.  Iterates until an iteration accepts fewer than
 * delta*K*n updates or max_iters is reached (reaching max_iters is a normal
 * return).  Finally every kept (point, neighbour) distance is recomputed in
 * the fp64 recipe above, rows are sorted by (distance, id) and cut to k.
 *
 * points_dev [n][d] fp32 (device, read-only); ids_out_dev [n][k] int32 and
 * dists_out_dev [n][k] fp32 (device, written in full on success).
 * Errors: KNNG_EINVAL for null pointers, n < 2, d < 1, k < 1, K < k,
 * K > min(n-1, KNNG_MAX_K), rho outside (0,1], cand_cap outside [1, KNNG_MAX_K],
 * unknown metric, wrong struct_size; KNNG_EWORKSPACE; KNNG_EHIP.
 * Host-synchronises `stream` once per iteration (the convergence test).
 */
int knng_build_knn_graph(const float *points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                         const knng_params_t *params, int32_t *ids_out_dev, float *dists_out_dev);

/*
 * The same build for points stored as uint8 (Sec. 5.2, dataset table: the SIFT sets the paper scales
 * to are 8-bit; a quarter of the bytes the joins gather).  points_dev [n][d] uint8
 * (device, read-only, 4-byte aligned; rows are 16-byte pieces when d % 16 == 0 and
 * the pointer is 16-byte aligned, else 4-byte words).  The values are taken as they
 * are: every distance is the exact integer sum of squared differences, rounded once
 * to fp32, which is what the fp64 recipe gives on the same values stored as fp32 --
 * the result obeys the same definition as knng_build_knn_graph on that fp32 copy.
 * Workspace: knng_build_workspace_bytes (the same).  Everything else as above.
 * Additional KNNG_EINVAL cases: metric other than KNNG_METRIC_L2SQ, d % 4 != 0,
 * d > 65536 (32-bit integer sums), pointer not 4-byte aligned.
 */
int knng_build_knn_graph_u8(const uint8_t *points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                            const knng_params_t *params, int32_t *ids_out_dev, float *dists_out_dev);

/*
 * The same build for points stored as IEEE half precision (compact element types
 * halve the bytes the joins gather; Sec. 5.2 lists the element types of the paper's
 * sets).  points_dev [n][d] fp16 (device, read-only, 4-byte aligned; 16-byte pieces
 * when d % 8 == 0 and the pointer is 16-byte aligned, else 4-byte words).  The values
 * are taken as they are: the result obeys the definition of knng_build_knn_graph on
 * the same values converted to fp32 (every written distance is the fp64 recipe on
 * them).  During the search the joins centre rows in fp16, so candidates are compared
 * at a relative precision of about 1e-3; this affects which neighbours are found, not
 * what is written about them.  Workspace: knng_build_workspace_bytes (the same).
 * Additional KNNG_EINVAL cases: metric other than KNNG_METRIC_L2SQ, d % 2 != 0,
 * pointer not 4-byte aligned.
 */
int knng_build_knn_graph_f16(const uint16_t *points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                             const knng_params_t *params, int32_t *ids_out_dev, float *dists_out_dev);

/* Device scratch needed by knng_brute_knn (0 on bad arguments). */
uint64_t knng_brute_workspace_bytes(int64_t n, int32_t d, int32_t k, int64_t nq);

/*
 * Exact k-NN rows by brute force (Sec. 2.1: the exact graph recall is measured
 * against; Sec. 5.3.1: the ground truth of the single-GPU experiments).
 *
 * For query q the source point is r = query_rows_dev ? query_rows_dev[q] : q;
 * every j != r is scored and the k smallest under (fp32 distance, id) are
 * written ascending to ids_out_dev[q][0..k) / dists_out_dev[q][0..k).
 * nq rows are produced (nq = n and query_rows_dev = NULL gives the whole graph);
 * nq = 0 is a no-op.  k <= min(n-1, KNNG_MAX_K).  Results are deterministic.
 */
int knng_brute_knn(const float *points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                   const int32_t *query_rows_dev, int64_t nq,
                   int32_t *ids_out_dev, float *dists_out_dev,
                   void *workspace_dev, uint64_t workspace_bytes, void *stream);

/*
 * Recall of a test graph against a reference graph over the nearest at_k
 * entries of each row (Sec. 5.3.1), rows ascending in both.
 *   mode 0 (Sec. 2.1): share of the test neighbours whose id also appears in
 *          the reference row.  Needs the two id matrices.
 *   mode 1 (Sec. 5.4.3): the reference row's at_k-th distance is a threshold;
 *          share of the test neighbours with distance <= it.  Needs the two
 *          distance matrices.
 * test_* are [rows][k_test], ref_* are [rows][k_ref] (device); at_k <= both.
 * A row holds each id at most once; an entry with id < 0 is padding and a miss.
 * The matrices a mode does not need may be NULL.  *recall_out_host (host)
 * receives hits / (rows * at_k).  Allocates and frees 8 bytes of device memory.
 */
int knng_graph_recall(const int32_t *test_ids_dev, const float *test_dists_dev, int32_t k_test,
                      const int32_t *ref_ids_dev, const float *ref_dists_dev, int32_t k_ref,
                      int64_t rows, int32_t at_k, int32_t mode,
                      double *recall_out_host, void *stream);

/*
 * knng_graph_recall for callers that cannot allocate or wait: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same recall,
 * bit for bit, but the call allocates nothing, copies nothing to the host and does
 * not synchronise: it enqueues two kernels on `stream` and returns; *recall_out_dev
 * (DEVICE memory, one double, 8-byte aligned) holds hits / (rows * at_k) once they
 * have run.  The per-workgroup partial counts live in a fixed 64 KiB device array
 * inside the library (every GPU the library runs on holds it until the process
 * ends); its address is looked up on the first call on a device.  Nothing in it has
 * to start at zero, and no memset is enqueued.
 * Limits: rows * at_k <= KNNG_RECALL_STATIC_MAX_ENTRIES, else KNNG_ETOOLARGE and
 * nothing is enqueued.  All calls on one GPU share the array: calls that overlap in
 * time on one GPU (different streams, different threads) race and must be ordered by
 * the caller.  Other arguments and errors as knng_graph_recall.
 */
#define KNNG_RECALL_STATIC_MAX_ENTRIES (1ll << 36)
int knng_graph_recall_static(const int32_t *test_ids_dev, const float *test_dists_dev, int32_t k_test,
                             const int32_t *ref_ids_dev, const float *ref_dists_dev, int32_t k_ref,
                             int64_t rows, int32_t at_k, int32_t mode,
                             double *recall_out_dev, void *stream);

/*
 * Update of a graph's rows with neighbour candidates found elsewhere: the local
 * half of the refinement step (Sec. 4.3 step 4: a rank updates its graph with the
 * candidates per point found on a remote graph; Sec. 4.4: G_{0->0} becomes
 * G_{0->0:1} using the search results R_{0->1}, which have the layout of a graph:
 * an id matrix and a distance matrix, one row per query point).
 *
 * Row i of the result = the k_out smallest entries under (distance, id) of row i
 * of A and row i of B taken together, one entry per id (of several entries with
 * one id the smallest stays).  Entries with id < 0 are padding and ignored; a row
 * with fewer than k_out distinct ids is filled with id -1 / distance +inf.
 * Distances are non-negative (as everywhere in this library).
 *
 * ids_a_dev/dists_a_dev [n][ka], ids_b_dev/dists_b_dev [n][kb], outputs
 * [n][k_out] (all device; outputs must not overlap inputs).  0 <= ka, kb <=
 * KNNG_MAX_K, ka + kb >= 1, 1 <= k_out <= 2*KNNG_MAX_K.  Asynchronous on `stream`;
 * allocates nothing.  Errors: KNNG_EINVAL, KNNG_EHIP.
 */
int knng_merge_graphs(const int32_t *ids_a_dev, const float *dists_a_dev, int32_t ka,
                      const int32_t *ids_b_dev, const float *dists_b_dev, int32_t kb,
                      int64_t n, int32_t k_out, int32_t *ids_out_dev, float *dists_out_dev,
                      void *stream);

/*
 * The same with the candidates restricted to the first n_base of the n points:
 * the exact neighbours, in one partition, of points that may lie in another (the
 * ground truth for the cross-partition search of Sec. 4.3).  Query rows are any
 * of the n points; for row r every j < n_base, j != r, is scored.
 * 2 <= n_base <= n, k <= min(n_base - 1, KNNG_MAX_K); workspace:
 * knng_brute_workspace_bytes(n, d, k, nq).  Everything else as knng_brute_knn.
 */
int knng_brute_knn_base(const float *points_dev, int64_t n, int64_t n_base, int32_t d, int32_t k,
                        int32_t metric, const int32_t *query_rows_dev, int64_t nq,
                        int32_t *ids_out_dev, float *dists_out_dev,
                        void *workspace_dev, uint64_t workspace_bytes, void *stream);

/* Device scratch needed by knng_optimize_graph (0 on bad arguments). */
uint64_t knng_optimize_workspace_bytes(int64_t n, int32_t k, int32_t d_out);

/*
 * Search graph G^s from a k-NN graph G (Sec. 3.3: edges that can be bypassed via
 * shorter paths are removed, reverse edges added; ranks only, no distance data).
 * The section names the technique; the steps are fixed here as follows.
 *
 * ids_dev [n][k] int32 (device, read-only): row u lists u's neighbours nearest
 * first (what knng_build_knn_graph writes), so the column is the rank.  An entry
 * is valid if it lies in [0,n), is not u and does not repeat an earlier entry of
 * its row; any other entry is padding.
 *   1. c(u,j) = number of neighbours w of u at a rank i < j whose own row holds
 *      u's j-th neighbour at a rank r < j (the edge u -> that neighbour can be
 *      bypassed through w); padding entries get c = k.
 *   2. P(u) = the d_out entries of row u with the smallest (c, rank), in that
 *      order (padding as -1).
 *   3. Every edge u -> v at position p of P(u) hands (p, u) to v; R(v) = what v
 *      received, ascending by (p, u).
 *   4. Row v of the result = the first d_out - d_out/2 entries of P(v); then R(v)
 *      in order, then the remaining entries of P(v) in order, are appended,
 *      skipping -1 and ids the row already holds, until it has d_out entries; a
 *      row that runs out of candidates is padded with -1.
 * ids_out_dev [n][d_out] int32 (device, written in full on success; must not
 * overlap ids_dev).  1 <= d_out <= k <= KNNG_MAX_K.  The result is deterministic.
 * Errors: KNNG_EINVAL (null pointers, sizes out of range), KNNG_EWORKSPACE, KNNG_EHIP.
 */
int knng_optimize_graph(const int32_t *ids_dev, int64_t n, int32_t k, int32_t d_out,
                        int32_t *ids_out_dev, void *workspace_dev, uint64_t workspace_bytes,
                        void *stream);

/*
 * Graph-based approximate nearest-neighbour search for query points (Sec. 3.2: the
 * search starts from selected points of the graph and greedily explores it by
 * visiting neighbours of previously visited points, until no closer neighbours are
 * found or a stopping criterion is met; k_s neighbours per query).  The bookkeeping,
 * which the section leaves open, is fixed as follows.
 *
 * Per query a list of at most itopk entries (distance, id, expanded or not) is kept
 * ascending by (fp32 distance, id), ids distinct.  "Offer x": if x is a valid id (in
 * [0,n)) that is not in the list, sigma(query, x) is evaluated (the fp64 recipe
 * above) and the itopk smallest of the list and x are kept.
 *   start:     starts_dev[q][0 .. n_starts) are offered in order;
 *   iteration: the first `width` entries of the list that are not yet expanded are
 *              marked expanded (none: the search ends), then the graph row of each
 *              is offered, in list order and row order; at most max_iters iterations.
 * Result: the first k_s entries of the list, padded with id -1 / distance +inf.
 * The start points are an input: the caller draws them (the paper picks them at
 * random), so the result is a function of the arguments alone.
 *
 * points_dev [n][d] fp32, graph_dev [n][deg] int32 (a k-NN graph or a search graph;
 * entries outside [0,n) are ignored), queries_dev [nq][d] fp32, starts_dev
 * [nq][n_starts] int32: device, read-only.  ids_out_dev [nq][k_s] int32,
 * dists_out_dev [nq][k_s] fp32: device, written in full.  iters_out_dev [nq] int32
 * and evals_out_dev [nq] int32 (optional, NULL to skip): iterations performed and
 * distances evaluated per query.  A row (or the start ids) is offered as one batch:
 * the ids of the batch that are valid, distinct and not in the list before the batch
 * are evaluated, which is never more than offering them one at a time evaluates.
 * 1 <= k_s <= itopk <= KNNG_MAX_K; deg, n_starts, width in [1, KNNG_MAX_K];
 * max_iters >= 0; d <= 8192; nq = 0 is a no-op.  Needs no workspace.
 * Errors: KNNG_EINVAL, KNNG_EHIP.
 */
int knng_graph_search(const float *points_dev, int64_t n, int32_t d, int32_t metric,
                      const int32_t *graph_dev, int32_t deg,
                      const float *queries_dev, int64_t nq,
                      const int32_t *starts_dev, int32_t n_starts,
                      int32_t k_s, int32_t itopk, int32_t width, int32_t max_iters,
                      int32_t *ids_out_dev, float *dists_out_dev, int32_t *iters_out_dev,
                      int32_t *evals_out_dev, void *stream);

/*
 * The same search for points and queries stored as uint8 (squared L2 only; the 8-bit
 * sets of Sec. 5.2): every distance is the exact integer sum of squared differences
 * rounded once to fp32, i.e. the result is that of knng_graph_search on the same
 * values stored as fp32.  points_dev [n][d] and queries_dev [nq][d] uint8, 4-byte
 * aligned, d % 4 == 0, d <= 65536; everything else as above.
 */
int knng_graph_search_u8(const uint8_t *points_dev, int64_t n, int32_t d, int32_t metric,
                         const int32_t *graph_dev, int32_t deg,
                         const uint8_t *queries_dev, int64_t nq,
                         const int32_t *starts_dev, int32_t n_starts,
                         int32_t k_s, int32_t itopk, int32_t width, int32_t max_iters,
                         int32_t *ids_out_dev, float *dists_out_dev, int32_t *iters_out_dev,
                         int32_t *evals_out_dev, void *stream);

/* Text for a return code; for KNNG_EHIP the text of the last HIP failure on this thread. */
const char *knng_strerror(int code);

/* KNNG_VERSION the library was built from. */
int knng_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KNNG_H */
