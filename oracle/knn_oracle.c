/*
 * knn_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow CPU statement of what the k-NN-graph path computes.  It exists
 * so that the tests, the smoke check and the CPU-baseline leg of the benchmark
 * have something independent to compare the GPU library against.  Nothing in
 * the product path may include, link or call this file, and this file includes
 * nothing from the GPU sources.
 *
 * Contents (paper passages each one follows are named at the function):
 *   oracle_distance      sigma(p1,p2): the distance recipes            (Sec. 2.1)
 *   oracle_brute_knn     the exact k-NN graph by brute force           (Sec. 2.1)
 *   oracle_graph_recall  recall of one graph against another           (Sec. 2.1, 5.3.1, 5.4.3)
 *   oracle_check_graph   row invariants of a k-NN graph                (Sec. 2.1)
 *   oracle_nn_descent    NN-Descent with candidate lists and a
 *                        single-owner merge, step by step              (Sec. 3.1, 3.1.1)
 *   oracle_merge_rows    a graph's rows updated with search results R  (Sec. 4.3 step 4, 4.4)
 *   oracle_optimize_graph  k-NN graph G -> search graph G^s            (Sec. 3.3)
 *   oracle_graph_search  greedy graph search for query points           (Sec. 3.2)
 *
 * Pin status: every function is pinned by tests that do not go through this
 * file (closed forms, exhaustive enumeration in numpy on tiny inputs, integer
 * data where all arithmetic is exact, the K = n-1 special case; for
 * oracle_nn_descent also a restatement of its sampling, reverse lists,
 * neighbour check and merge as set statements in Python, checked against the
 * lists oracle_nn_descent_trace writes out).  What stays
 * "parity unpinned" is agreement with the outputs of the paper's own
 * implementation: the paper prints no worked example or per-dataset numbers
 * for this path.
 *
 * Arithmetic: inputs are fp32; every distance is accumulated in IEEE double,
 * coordinates taken in index order t = 0..d-1 with an explicit fma and no
 * reassociation, then rounded once to fp32.  Build with -ffp-contract=off.
 * All orderings are lexicographic on (fp32 distance, id).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_L2SQ = 0, ORACLE_IP_UNIT = 1, ORACLE_COSINE = 2 };

/* ------------------------------------------------------------------------ */
/* sigma: non-negative, smaller = more similar (Sec. 2.1).                   */
/*   L2SQ    : sum_t (a_t - b_t)^2                                           */
/*   IP_UNIT : max(0, 1 - <a,b>)       rows are unit length by contract      */
/*   COSINE  : max(0, 1 - <a,b>/(|a||b|)); a zero vector is at distance 1    */
/* ------------------------------------------------------------------------ */
float oracle_distance(const float *a, const float *b, int32_t d, int32_t metric)
{
    double acc = 0.0;
    if (metric == ORACLE_L2SQ) {
        for (int32_t t = 0; t < d; ++t) {
            double df = (double)a[t] - (double)b[t];
            acc = fma(df, df, acc);
        }
        return (float)acc;
    }
    for (int32_t t = 0; t < d; ++t)
        acc = fma((double)a[t], (double)b[t], acc);
    if (metric == ORACLE_IP_UNIT) {
        double r = 1.0 - acc;
        if (r < 0.0) r = 0.0;
        return (float)r;
    }
    /* ORACLE_COSINE */
    double na = 0.0, nb = 0.0;
    for (int32_t t = 0; t < d; ++t) na = fma((double)a[t], (double)a[t], na);
    for (int32_t t = 0; t < d; ++t) nb = fma((double)b[t], (double)b[t], nb);
    if (na == 0.0 || nb == 0.0) return 1.0f;
    double r = 1.0 - acc / sqrt(na * nb);
    if (r < 0.0) r = 0.0;
    return (float)r;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* (dist, id) lexicographic "less than" */
static int key_less(float da, int32_t ia, float db, int32_t ib)
{
    return (da < db) || (da == db && ia < ib);
}

/* ------------------------------------------------------------------------ */
/* Exact k-NN graph (Sec. 2.1: the graph recall is measured against, found   */
/* by scoring every pair; k neighbours per source point, no more, no fewer). */
/* For query row r (= query_rows[q]                                          */
/* or q when query_rows is NULL) every j != r is scored with sigma and the k */
/* smallest under (fp32 dist, id) are written in ascending order.            */
/* The only parallelism is one query row per OpenMP iteration.               */
/* Returns 0, or -1 on bad arguments.                                        */
/* ------------------------------------------------------------------------ */
/* oracle_brute_knn_base: the same with the candidates restricted to the first */
/* n_base points (the exact neighbours of one partition's points in another     */
/* partition: Sec. 4.3); query rows may be any of the n points.                 */
int oracle_brute_knn_base(const float *points, int64_t n, int64_t n_base, int32_t d, int32_t k, int32_t metric,
                          const int32_t *query_rows, int64_t nq, int32_t *ids_out, float *dists_out);

int oracle_brute_knn(const float *points, int64_t n, int32_t d, int32_t k, int32_t metric,
                     const int32_t *query_rows, int64_t nq,
                     int32_t *ids_out, float *dists_out)
{
    return oracle_brute_knn_base(points, n, n, d, k, metric, query_rows, nq, ids_out, dists_out);
}

int oracle_brute_knn_base(const float *points, int64_t n, int64_t n_base, int32_t d, int32_t k, int32_t metric,
                          const int32_t *query_rows, int64_t nq, int32_t *ids_out, float *dists_out)
{
    if (!points || !ids_out || !dists_out || n < 2 || n_base < 2 || n_base > n || d < 1 || k < 1 ||
        k > n_base - 1 || metric < 0 || metric > 2 || nq < 0)
        return -1;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t q = 0; q < nq; ++q) {
        int64_t r = query_rows ? (int64_t)query_rows[q] : q;
        const float *x = points + r * (int64_t)d;
        int32_t *oi = ids_out + q * (int64_t)k;
        float *od = dists_out + q * (int64_t)k;
        int32_t cnt = 0;
        for (int64_t j = 0; j < n_base; ++j) {
            if (j == r) continue;
            float l = oracle_distance(x, points + j * (int64_t)d, d, metric);
            if (cnt == k && !key_less(l, (int32_t)j, od[k - 1], oi[k - 1])) continue;
            int32_t p = (cnt < k) ? cnt : k - 1;   /* slot that is free or dropped */
            while (p > 0 && key_less(l, (int32_t)j, od[p - 1], oi[p - 1])) {
                od[p] = od[p - 1];
                oi[p] = oi[p - 1];
                --p;
            }
            od[p] = l;
            oi[p] = (int32_t)j;
            if (cnt < k) ++cnt;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Recall of a test graph against a reference graph, over the nearest at_k   */
/* entries of each (Sec. 5.3.1: take the nearest 32 of a k >= 32 graph).     */
/*   mode 0 (Sec. 2.1): fraction of test neighbours whose id also appears in */
/*           the reference row.                                              */
/*   mode 1 (Sec. 5.4.3): the reference row's at_k-th distance is a          */
/*           threshold; fraction of test neighbours at distance <= it.       */
/* Rows of both graphs are ascending and hold each id at most once; an entry */
/* with id < 0 is padding (a row with fewer than k neighbours) and counts as  */
/* a miss.  Returns the recall, or -1.0 on bad arguments.                    */
/* ------------------------------------------------------------------------ */
double oracle_graph_recall(const int32_t *test_ids, const float *test_dists, int32_t k_test,
                           const int32_t *ref_ids, const float *ref_dists, int32_t k_ref,
                           int64_t n, int32_t at_k, int32_t mode)
{
    if (n < 1 || at_k < 1 || at_k > k_test || at_k > k_ref || mode < 0 || mode > 1) return -1.0;
    if (mode == 0 && (!test_ids || !ref_ids)) return -1.0;
    if (mode == 1 && (!test_dists || !ref_dists)) return -1.0;
    int64_t hits = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (mode == 0) {
            const int32_t *t = test_ids + i * (int64_t)k_test;
            const int32_t *r = ref_ids + i * (int64_t)k_ref;
            for (int32_t a = 0; a < at_k; ++a) {
                if (t[a] < 0) continue;             /* padding is no neighbour */
                for (int32_t b = 0; b < at_k; ++b)
                    if (t[a] == r[b]) { ++hits; break; }
            }
        } else {
            const float *t = test_dists + i * (int64_t)k_test;
            float thr = ref_dists[i * (int64_t)k_ref + (at_k - 1)];
            for (int32_t a = 0; a < at_k; ++a)
                if (t[a] <= thr) ++hits;
        }
    }
    return (double)hits / ((double)n * (double)at_k);
}

/* ------------------------------------------------------------------------ */
/* Row invariants of a k-NN graph (Sec. 2.1: exactly k neighbours per source */
/* point, each entry an id and its distance from the source point).          */
/* violations[0] id out of [0,n)      violations[1] self loop                */
/* violations[2] duplicate id in row  violations[3] row not ascending under  */
/*                                                  (dist, id)               */
/* violations[4] |dist - sigma| > rel_tol*sigma + 1e-30                      */
/* violations[5] negative or non-finite distance                             */
/* Returns the total number of violations, or -1 on bad arguments.           */
/* ------------------------------------------------------------------------ */
int64_t oracle_check_graph(const float *points, int64_t n, int32_t d, int32_t metric,
                           const int32_t *ids, const float *dists, int32_t k,
                           double rel_tol, int64_t violations[6])
{
    if (!points || !ids || !dists || !violations || n < 2 || d < 1 || k < 1) return -1;
    int64_t v0 = 0, v1 = 0, v2 = 0, v3 = 0, v4 = 0, v5 = 0;
#pragma omp parallel for schedule(static) reduction(+ : v0, v1, v2, v3, v4, v5)
    for (int64_t i = 0; i < n; ++i) {
        const int32_t *ri = ids + i * (int64_t)k;
        const float *rd = dists + i * (int64_t)k;
        for (int32_t a = 0; a < k; ++a) {
            int32_t id = ri[a];
            if (!(rd[a] >= 0.0f) || isinf(rd[a])) ++v5;
            if (id < 0 || (int64_t)id >= n) { ++v0; continue; }
            if ((int64_t)id == i) ++v1;
            for (int32_t b = 0; b < a; ++b)
                if (ri[b] == id) { ++v2; break; }
            if (a > 0 && !key_less(rd[a - 1], ri[a - 1], rd[a], id)) ++v3;
            double s = (double)oracle_distance(points + i * (int64_t)d,
                                               points + (int64_t)id * d, d, metric);
            if (fabs((double)rd[a] - s) > rel_tol * s + 1e-30) ++v4;
        }
    }
    violations[0] = v0; violations[1] = v1; violations[2] = v2;
    violations[3] = v3; violations[4] = v4; violations[5] = v5;
    return v0 + v1 + v2 + v3 + v4 + v5;
}

/* ======================================================================== */
/* NN-Descent with per-point candidate lists (Sec. 3.1 and 3.1.1).           */
/* ======================================================================== */

/* The oracle's own stateless random numbers: a 64-bit mix of a counter.     */
static uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
typedef struct { uint64_t key, ctr; } rng_t;
static rng_t rng_make(uint64_t seed, uint64_t a, uint64_t b)
{
    rng_t r;
    r.key = mix64(mix64(seed ^ 0x6A09E667F3BCC908ull) + mix64(a * 0x100000001B3ull + b));
    r.ctr = 0;
    return r;
}
static uint64_t rng_next(rng_t *r) { return mix64(r->key + (r->ctr++) * 0xD1342543DE82EF95ull); }
/* uniform integer in [0, m), m >= 1 (rejection, unbiased) */
static uint64_t rng_below(rng_t *r, uint64_t m)
{
    uint64_t lim = UINT64_MAX - (UINT64_MAX % m);
    uint64_t x;
    do { x = rng_next(r); } while (x >= lim);
    return x % m;
}
/* keep a uniformly random subset of size min(want,cnt) in a[0..], return its size */
static int32_t choose_uniform(int32_t *a, int32_t cnt, int32_t want, rng_t *r)
{
    int32_t m = cnt < want ? cnt : want;
    for (int32_t i = 0; i < m; ++i) {
        int32_t j = i + (int32_t)rng_below(r, (uint64_t)(cnt - i));
        int32_t t = a[i]; a[i] = a[j]; a[j] = t;
    }
    return m;
}

typedef struct { int32_t id; float dist; } cand_t;
typedef struct { cand_t *v; int32_t cnt, cap; } candlist_t;

typedef struct {
    int64_t n; int32_t K;
    int32_t *ids; float *dist; uint8_t *isnew;     /* [n][K], rows ascending */
    candlist_t *cand; int32_t cand_cap;            /* 0 = unbounded */
    int64_t dropped;
} graph_t;

/* Offer (l, b) to point a: appended iff closer than a's current farthest     */
/* neighbour (Sec. 3.1.1); the list has a fixed size, a full list drops.      */
static void offer(graph_t *g, int32_t a, int32_t b, float l)
{
    const int32_t K = g->K;
    const float *rd = g->dist + (int64_t)a * K;
    const int32_t *ri = g->ids + (int64_t)a * K;
    if (!key_less(l, b, rd[K - 1], ri[K - 1])) return;
    candlist_t *c = &g->cand[a];
    if (g->cand_cap > 0 && c->cnt >= g->cand_cap) { ++g->dropped; return; }
    if (c->cnt == c->cap) {
        int32_t nc = c->cap ? 2 * c->cap : 16;
        if (g->cand_cap > 0 && nc > g->cand_cap) nc = g->cand_cap;
        c->v = (cand_t *)realloc(c->v, sizeof(cand_t) * (size_t)nc);
        c->cap = nc;
    }
    c->v[c->cnt].id = b;
    c->v[c->cnt].dist = l;
    ++c->cnt;
}

/* One owner per point folds its candidate list into its row (Sec. 3.1.1).   */
/* Returns the number of accepted updates for this row.                      */
static int64_t merge_row(graph_t *g, int64_t a)
{
    const int32_t K = g->K;
    int32_t *ri = g->ids + a * K;
    float *rd = g->dist + a * K;
    uint8_t *rf = g->isnew + a * K;
    candlist_t *c = &g->cand[a];
    int64_t acc = 0;
    for (int32_t e = 0; e < c->cnt; ++e) {
        int32_t id = c->v[e].id;
        float l = c->v[e].dist;
        if (!key_less(l, id, rd[K - 1], ri[K - 1])) continue;
        int dup = 0;
        for (int32_t p = 0; p < K; ++p)
            if (ri[p] == id) { dup = 1; break; }
        if (dup) continue;
        int32_t p = K - 1;
        while (p > 0 && key_less(l, id, rd[p - 1], ri[p - 1])) {
            rd[p] = rd[p - 1]; ri[p] = ri[p - 1]; rf[p] = rf[p - 1];
            --p;
        }
        rd[p] = l; ri[p] = id; rf[p] = 1;
        ++acc;
    }
    c->cnt = 0;       /* the list is cleared after the update */
    return acc;
}

static void append_unique(int32_t *dst, int32_t *cnt, int32_t id)
{
    for (int32_t i = 0; i < *cnt; ++i)
        if (dst[i] == id) return;
    dst[(*cnt)++] = id;
}

/*
 * oracle_nn_descent
 *
 *  1. G starts with K distinct random neighbours != v per point, with their
 *     true distances, rows ascending, every entry flagged new.   (Sec. 3.1)
 *  2. Per iteration and point: up to s = ceil(rho*K) new-flagged entries,
 *     chosen uniformly, form the forward new sample (their flags are cleared);
 *     up to s entries that were not new, chosen uniformly, form the forward
 *     old sample.  rho = 1 samples everything.                   (Sec. 3.1)
 *  3. Reverse samples: for each u, up to s uniformly chosen v that hold u in
 *     their forward new (old) sample.  NEW[v] = forward + reverse new, without
 *     repeats; OLD[v] likewise, minus anything in NEW[v].
 *  4. Neighbour check: for every point v, every unordered pair in NEW[v] and
 *     every pair NEW[v] x OLD[v]: l = sigma(u1,u2); u2 is appended to u1's
 *     candidate list if it is closer than u1's current farthest neighbour,
 *     and u1 to u2's.  Lists hold cand_cap entries (0 = unbounded); a full
 *     list drops.                                                (Sec. 3.1.1)
 *  5. Each point's list is folded into its row by one owner: ids already
 *     present and entries no longer closer than the farthest are rejected,
 *     the rest inserted in order, flagged new, and counted as accepted
 *     updates; the list is cleared.                              (Sec. 3.1.1)
 *  6. Stop when the accepted updates of an iteration are < delta*K*n, or
 *     after max_iters iterations.                                (Sec. 3.1, 5.3.1)
 *  7. The first k of the K entries of every row are the result.  (Sec. 5.3.1)
 *
 * The distance evaluations of step 4 are computed for a batch of points at a
 * time with one OpenMP iteration per pair; the offers are then made in the
 * sequential enumeration order, so results do not depend on the thread count.
 *
 * stats (optional, int64[3 + max_iters]): [0] iterations run, [1] distance
 * evaluations, [2] candidates dropped by full lists, [3+i] accepted updates
 * of iteration i.  Returns 0, -1 on bad arguments, -2 on allocation failure.
 *
 * oracle_nn_descent_trace is the same function with the intermediate lists of the
 * LAST iteration it ran written out, so that tests can check steps 2 and 3 against
 * their definitions from outside (no arithmetic differs).  Every pointer may be
 * NULL.  With s = the sample size and the last iteration's lists:
 *   tr_fwd  int32 [2][n][s]   forward new sample, forward old sample     (step 2)
 *   tr_rev  int32 [2][n][s]   reverse new sample, reverse old sample     (step 3)
 *   tr_cnt  int32 [n][4]      their lengths: fwd new, fwd old, rev new, rev old
 *   tr_full int32 [2][n][2s]  NEW[v], OLD[v] as the neighbour check uses them
 *   tr_fcnt int32 [n][2]      |NEW[v]|, |OLD[v]|
 *   flags_out uint8 [n][K]    the new-flags of the final rows (all K entries)
 *   rows_out int32 [n][K]     the ids of the final rows (all K entries)
 */
int oracle_nn_descent_trace(const float *points, int64_t n, int32_t d, int32_t k, int32_t metric,
                            int32_t K, double rho, double delta, int32_t max_iters,
                            int32_t cand_cap, uint64_t seed,
                            int32_t *ids_out, float *dists_out, int64_t *stats,
                            int32_t *tr_fwd, int32_t *tr_rev, int32_t *tr_cnt,
                            int32_t *tr_full, int32_t *tr_fcnt, uint8_t *flags_out, int32_t *rows_out)
{
    if (!points || !ids_out || !dists_out || n < 2 || d < 1 || k < 1 || K < k ||
        (int64_t)K > n - 1 || metric < 0 || metric > 2 || !(rho > 0.0) || rho > 1.0 ||
        delta < 0.0 || max_iters < 0 || cand_cap < 0)
        return -1;
    int32_t s = (int32_t)ceil(rho * (double)K);
    if (s > K) s = K;
    if (s < 1) s = 1;

    graph_t g;
    g.n = n; g.K = K; g.cand_cap = cand_cap; g.dropped = 0;
    g.ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * K);
    g.dist = (float *)malloc(sizeof(float) * (size_t)n * K);
    g.isnew = (uint8_t *)malloc((size_t)n * K);
    g.cand = (candlist_t *)calloc((size_t)n, sizeof(candlist_t));
    /* forward samples [n][s] + counts; full lists [n][2s] + counts */
    int32_t *newf = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * s);
    int32_t *oldf = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * s);
    int32_t *newf_cnt = (int32_t *)calloc((size_t)n, sizeof(int32_t));
    int32_t *oldf_cnt = (int32_t *)calloc((size_t)n, sizeof(int32_t));
    int32_t *NEW = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * 2 * s);
    int32_t *OLD = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * 2 * s);
    int32_t *NEW_cnt = (int32_t *)calloc((size_t)n, sizeof(int32_t));
    int32_t *OLD_cnt = (int32_t *)calloc((size_t)n, sizeof(int32_t));
    int64_t *rev_off = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    int32_t *rev_src = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * s);
    if (!g.ids || !g.dist || !g.isnew || !g.cand || !newf || !oldf || !newf_cnt || !oldf_cnt ||
        !NEW || !OLD || !NEW_cnt || !OLD_cnt || !rev_off || !rev_src)
        return -2;

    int64_t n_eval = 0;

    /* ---- step 1: random initial graph ---- */
#pragma omp parallel for schedule(static) reduction(+ : n_eval)
    for (int64_t v = 0; v < n; ++v) {
        rng_t r = rng_make(seed, 1, (uint64_t)v);
        int32_t *ri = g.ids + v * K;
        float *rd = g.dist + v * K;
        if ((int64_t)K * 2 > n - 1) {
            /* dense case: partial shuffle of all other points */
            int32_t *all = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n - 1));
            int32_t m = 0;
            for (int64_t j = 0; j < n; ++j) if (j != v) all[m++] = (int32_t)j;
            choose_uniform(all, m, K, &r);
            memcpy(ri, all, sizeof(int32_t) * (size_t)K);
            free(all);
        } else {
            int32_t c = 0;
            while (c < K) {
                int32_t id = (int32_t)rng_below(&r, (uint64_t)n);
                if (id == v) continue;
                int dup = 0;
                for (int32_t p = 0; p < c; ++p) if (ri[p] == id) { dup = 1; break; }
                if (!dup) ri[c++] = id;
            }
        }
        for (int32_t p = 0; p < K; ++p)
            rd[p] = oracle_distance(points + v * (int64_t)d, points + (int64_t)ri[p] * d, d, metric);
        n_eval += K;
        /* ascending by (dist, id): insertion sort */
        for (int32_t p = 1; p < K; ++p) {
            float l = rd[p]; int32_t id = ri[p]; int32_t q = p;
            while (q > 0 && key_less(l, id, rd[q - 1], ri[q - 1])) {
                rd[q] = rd[q - 1]; ri[q] = ri[q - 1]; --q;
            }
            rd[q] = l; ri[q] = id;
        }
        memset(g.isnew + v * K, 1, (size_t)K);
    }

    /* pair buffers for one batch of points */
    const int64_t BATCH = 1024;
    const int64_t max_pairs_pt = (int64_t)(2 * s) * (2 * s - 1) / 2 + (int64_t)(2 * s) * (2 * s);
    int32_t *pa = (int32_t *)malloc(sizeof(int32_t) * (size_t)(BATCH * max_pairs_pt));
    int32_t *pb = (int32_t *)malloc(sizeof(int32_t) * (size_t)(BATCH * max_pairs_pt));
    float *pl = (float *)malloc(sizeof(float) * (size_t)(BATCH * max_pairs_pt));
    if (!pa || !pb || !pl) return -2;

    int32_t it = 0;
    for (; it < max_iters; ++it) {
        /* ---- step 2: forward samples ---- */
        for (int64_t v = 0; v < n; ++v) {
            rng_t r = rng_make(seed, 2 + 4 * (uint64_t)it, (uint64_t)v);
            int32_t posn[K > 0 ? K : 1], poso[K > 0 ? K : 1];
            int32_t cn = 0, co = 0;
            for (int32_t p = 0; p < K; ++p) {
                if (g.isnew[v * K + p]) posn[cn++] = p; else poso[co++] = p;
            }
            int32_t mn = choose_uniform(posn, cn, s, &r);
            int32_t mo = choose_uniform(poso, co, s, &r);
            for (int32_t i = 0; i < mn; ++i) {
                newf[v * s + i] = g.ids[v * K + posn[i]];
                g.isnew[v * K + posn[i]] = 0;
            }
            for (int32_t i = 0; i < mo; ++i) oldf[v * s + i] = g.ids[v * K + poso[i]];
            newf_cnt[v] = mn; oldf_cnt[v] = mo;
        }
        /* ---- step 3: reverse samples, then the full lists ---- */
        for (int pass = 0; pass < 2; ++pass) {
            const int32_t *fwd = pass == 0 ? newf : oldf;
            const int32_t *fcnt = pass == 0 ? newf_cnt : oldf_cnt;
            int32_t *FULL = pass == 0 ? NEW : OLD;
            int32_t *FCNT = pass == 0 ? NEW_cnt : OLD_cnt;
            memset(rev_off, 0, sizeof(int64_t) * (size_t)(n + 1));
            for (int64_t v = 0; v < n; ++v)
                for (int32_t i = 0; i < fcnt[v]; ++i) ++rev_off[fwd[v * s + i] + 1];
            for (int64_t u = 0; u < n; ++u) rev_off[u + 1] += rev_off[u];
            {
                int64_t *cur = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
                if (!cur) return -2;
                memcpy(cur, rev_off, sizeof(int64_t) * (size_t)n);
                for (int64_t v = 0; v < n; ++v)
                    for (int32_t i = 0; i < fcnt[v]; ++i) rev_src[cur[fwd[v * s + i]]++] = (int32_t)v;
                free(cur);
            }
            for (int64_t u = 0; u < n; ++u) {
                rng_t r = rng_make(seed, 3 + pass + 4 * (uint64_t)it, (uint64_t)u);
                int32_t *dst = FULL + u * 2 * s;
                int32_t c = 0;
                for (int32_t i = 0; i < fcnt[u]; ++i) {
                    int32_t id = fwd[u * s + i];
                    int skip = 0;
                    if (pass == 1)      /* OLD excludes what is in NEW */
                        for (int32_t j = 0; j < NEW_cnt[u]; ++j)
                            if (NEW[u * 2 * s + j] == id) { skip = 1; break; }
                    if (!skip) append_unique(dst, &c, id);
                }
                int32_t rc = (int32_t)(rev_off[u + 1] - rev_off[u]);
                int32_t *src = rev_src + rev_off[u];
                int32_t m = choose_uniform(src, rc, s, &r);
                if (tr_rev) memcpy(tr_rev + ((int64_t)pass * n + u) * s, src, sizeof(int32_t) * (size_t)m);
                if (tr_cnt) tr_cnt[u * 4 + 2 + pass] = m;
                for (int32_t i = 0; i < m; ++i) {
                    int32_t id = src[i];
                    int skip = 0;
                    if (pass == 1)
                        for (int32_t j = 0; j < NEW_cnt[u]; ++j)
                            if (NEW[u * 2 * s + j] == id) { skip = 1; break; }
                    if (!skip) append_unique(dst, &c, id);
                }
                FCNT[u] = c;
            }
        }
        if (tr_fwd) {
            memcpy(tr_fwd, newf, sizeof(int32_t) * (size_t)n * s);
            memcpy(tr_fwd + n * s, oldf, sizeof(int32_t) * (size_t)n * s);
        }
        if (tr_cnt) for (int64_t v = 0; v < n; ++v) { tr_cnt[v * 4] = newf_cnt[v]; tr_cnt[v * 4 + 1] = oldf_cnt[v]; }
        if (tr_full) {
            memcpy(tr_full, NEW, sizeof(int32_t) * (size_t)n * 2 * s);
            memcpy(tr_full + n * 2 * s, OLD, sizeof(int32_t) * (size_t)n * 2 * s);
        }
        if (tr_fcnt) for (int64_t v = 0; v < n; ++v) { tr_fcnt[v * 2] = NEW_cnt[v]; tr_fcnt[v * 2 + 1] = OLD_cnt[v]; }
        /* ---- step 4: neighbour check, offers into candidate lists ---- */
        for (int64_t v0 = 0; v0 < n; v0 += BATCH) {
            int64_t v1 = v0 + BATCH < n ? v0 + BATCH : n;
            int64_t np = 0;
            for (int64_t v = v0; v < v1; ++v) {
                const int32_t *nw = NEW + v * 2 * s; int32_t cn = NEW_cnt[v];
                const int32_t *ol = OLD + v * 2 * s; int32_t co = OLD_cnt[v];
                for (int32_t i = 0; i < cn; ++i) {
                    for (int32_t j = i + 1; j < cn; ++j) { pa[np] = nw[i]; pb[np] = nw[j]; ++np; }
                    for (int32_t j = 0; j < co; ++j) { pa[np] = nw[i]; pb[np] = ol[j]; ++np; }
                }
            }
#pragma omp parallel for schedule(static)
            for (int64_t e = 0; e < np; ++e)
                pl[e] = oracle_distance(points + (int64_t)pa[e] * d, points + (int64_t)pb[e] * d, d, metric);
            n_eval += np;
            for (int64_t e = 0; e < np; ++e) {
                offer(&g, pa[e], pb[e], pl[e]);
                offer(&g, pb[e], pa[e], pl[e]);
            }
        }
        /* ---- step 5: single-owner merge, count accepted updates ---- */
        int64_t c = 0;
        for (int64_t a = 0; a < n; ++a) c += merge_row(&g, a);
        if (stats) stats[3 + it] = c;
        /* ---- step 6: convergence ---- */
        if ((double)c < delta * (double)K * (double)n) { ++it; break; }
    }
    if (stats) { stats[0] = it; stats[1] = n_eval; stats[2] = g.dropped; }

    /* ---- step 7: truncate to k ---- */
    for (int64_t v = 0; v < n; ++v) {
        memcpy(ids_out + v * k, g.ids + v * K, sizeof(int32_t) * (size_t)k);
        memcpy(dists_out + v * k, g.dist + v * K, sizeof(float) * (size_t)k);
    }
    if (flags_out) memcpy(flags_out, g.isnew, (size_t)n * K);
    if (rows_out) memcpy(rows_out, g.ids, sizeof(int32_t) * (size_t)n * K);
    for (int64_t a = 0; a < n; ++a) free(g.cand[a].v);
    free(g.cand); free(g.ids); free(g.dist); free(g.isnew);
    free(newf); free(oldf); free(newf_cnt); free(oldf_cnt);
    free(NEW); free(OLD); free(NEW_cnt); free(OLD_cnt);
    free(rev_off); free(rev_src); free(pa); free(pb); free(pl);
    return 0;
}

int oracle_nn_descent(const float *points, int64_t n, int32_t d, int32_t k, int32_t metric,
                      int32_t K, double rho, double delta, int32_t max_iters,
                      int32_t cand_cap, uint64_t seed,
                      int32_t *ids_out, float *dists_out, int64_t *stats)
{
    return oracle_nn_descent_trace(points, n, d, k, metric, K, rho, delta, max_iters, cand_cap, seed,
                                   ids_out, dists_out, stats, NULL, NULL, NULL, NULL, NULL, NULL, NULL);
}

/* ------------------------------------------------------------------------ */
/* Update of a k-NN graph's rows with neighbour candidates found elsewhere   */
/* (Sec. 4.3 step 4: a rank brings its own graph up to date with the k       */
/* candidates per point it found on a remote graph; Sec. 4.4: the search     */
/* result R_{0->1} turns G_{0->0} into G_{0->0:1}).  R has the layout of a   */
/* graph: ids and distances per query point (Sec. 4.4).                      */
/* Row i of the result = the k_out smallest entries under (distance, id) of  */
/* row i of A and row i of B taken together, one entry per id (of several    */
/* entries with one id the smallest stays); entries with id < 0 are padding  */
/* and ignored; missing entries are written as id -1, distance +inf.         */
/* Plain statement: concatenate, selection sort, skip repeated ids.          */
/* Returns 0, or -1 on bad arguments.                                        */
/* ------------------------------------------------------------------------ */
int oracle_merge_rows(const int32_t *ids_a, const float *dists_a, int32_t ka,
                      const int32_t *ids_b, const float *dists_b, int32_t kb,
                      int64_t n, int32_t k_out, int32_t *ids_out, float *dists_out)
{
    if (n < 0 || ka < 0 || kb < 0 || k_out < 1 || ka + kb < 1) return -1;
    if ((ka && (!ids_a || !dists_a)) || (kb && (!ids_b || !dists_b)) || !ids_out || !dists_out) return -1;
    int32_t m = ka + kb;
    int32_t *id = (int32_t *)malloc((size_t)m * sizeof(int32_t));
    float *ds = (float *)malloc((size_t)m * sizeof(float));
    char *used = (char *)malloc((size_t)m);
    if (!id || !ds || !used) { free(id); free(ds); free(used); return -1; }
    for (int64_t i = 0; i < n; ++i) {
        for (int32_t j = 0; j < ka; ++j) { id[j] = ids_a[i * ka + j]; ds[j] = dists_a[i * ka + j]; }
        for (int32_t j = 0; j < kb; ++j) { id[ka + j] = ids_b[i * kb + j]; ds[ka + j] = dists_b[i * kb + j]; }
        for (int32_t j = 0; j < m; ++j) used[j] = id[j] < 0;
        int32_t w = 0;
        while (w < k_out) {
            int32_t best = -1;
            for (int32_t j = 0; j < m; ++j)
                if (!used[j] && (best < 0 || key_less(ds[j], id[j], ds[best], id[best]))) best = j;
            if (best < 0) break;
            ids_out[i * k_out + w] = id[best];
            dists_out[i * k_out + w] = ds[best];
            ++w;
            for (int32_t j = 0; j < m; ++j)          /* every other entry with this id is larger */
                if (id[j] == id[best]) used[j] = 1;
        }
        for (; w < k_out; ++w) { ids_out[i * k_out + w] = -1; dists_out[i * k_out + w] = INFINITY; }
    }
    free(id); free(ds); free(used);
    return 0;
}

/* ======================================================================== */
/* Search-graph optimisation G -> G^s (Sec. 3.3): drop edges that a shorter  */
/* two-hop path bypasses, then add reverse edges; ids only, no distances.    */
/* The section names the technique and its properties (rank-based, needs no  */
/* distance data); the steps below are this build's reading of it.           */
/*                                                                           */
/* ids [n][k]: row u lists u's neighbours nearest first, so the column is the */
/* rank.  An entry is *valid* if it lies in [0,n), is not u and does not      */
/* repeat an earlier entry of the row; other entries are padding.            */
/* 1. Detours.  The edge u -> v at rank j can be bypassed through a          */
/*    neighbour w of u if both hops rank before it: w at rank i < j in u's   */
/*    row and v at some rank r < j in w's row.  c(u,j) = number of such w.   */
/*    Padding entries get c = k (more than any count).                       */
/* 2. Prune.  P(u) = the d_out entries of row u with the smallest (c, rank), */
/*    in that order; padding is written as -1.                               */
/* 3. Reverse.  Every edge u -> v at position p of P(u) hands (p, u) to v;   */
/*    R(v) = what v received, ascending by (p, u).                           */
/* 4. Merge, with h = d_out / 2: the row of v in G^s starts with the first   */
/*    d_out - h entries of P(v); then R(v) in order, then the rest of P(v)   */
/*    in order, are appended, skipping -1 and ids the row already holds,     */
/*    until it has d_out entries (at most h come from R(v) unless P(v) runs  */
/*    out); if everything runs out the row is padded with -1.                */
/* Returns 0, or -1 on bad arguments (n < 1, k < 1, d_out < 1, d_out > k).   */
/* ------------------------------------------------------------------------ */
typedef struct { int32_t p, u; } rev_t;
static int rev_cmp(const void *a, const void *b)
{
    const rev_t *x = (const rev_t *)a, *y = (const rev_t *)b;
    if (x->p != y->p) return x->p < y->p ? -1 : 1;
    return x->u < y->u ? -1 : (x->u > y->u ? 1 : 0);
}

int oracle_optimize_graph(const int32_t *ids, int64_t n, int32_t k, int32_t d_out, int32_t *out)
{
    if (!ids || !out || n < 1 || k < 1 || d_out < 1 || d_out > k) return -1;
    int32_t *P = (int32_t *)malloc((size_t)n * d_out * sizeof(int32_t));
    int64_t *start = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
    if (!P || !start) { free(P); free(start); return -1; }

    /* steps 1 and 2 */
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t u = 0; u < n; ++u) {
        const int32_t *row = ids + u * k;
        int32_t c[1024], valid[1024], order[1024];
        int32_t *cc = c, *vv = valid, *oo = order;
        if (k > 1024) { cc = malloc(3 * (size_t)k * sizeof(int32_t)); vv = cc + k; oo = vv + k; }
        for (int32_t j = 0; j < k; ++j) {
            int ok = row[j] >= 0 && (int64_t)row[j] < n && (int64_t)row[j] != u;
            for (int32_t i = 0; ok && i < j; ++i) if (row[i] == row[j]) ok = 0;
            vv[j] = ok;
        }
        for (int32_t j = 0; j < k; ++j) {
            if (!vv[j]) { cc[j] = k; continue; }
            int32_t cnt = 0;
            for (int32_t i = 0; i < j; ++i) {
                if (!vv[i]) continue;
                const int32_t *wrow = ids + (int64_t)row[i] * k;
                int found = 0;
                for (int32_t r = 0; r < j && !found; ++r) found = wrow[r] == row[j];
                cnt += found;
            }
            cc[j] = cnt;
        }
        /* stable selection by (count, rank) */
        for (int32_t j = 0; j < k; ++j) oo[j] = j;
        for (int32_t a = 1; a < k; ++a) {
            int32_t x = oo[a], b = a;
            while (b > 0 && cc[oo[b - 1]] > cc[x]) { oo[b] = oo[b - 1]; --b; }
            oo[b] = x;
        }
        for (int32_t p = 0; p < d_out; ++p) P[u * d_out + p] = vv[oo[p]] ? row[oo[p]] : -1;
        if (cc != c) free(cc);
    }

    /* step 3: what every point received, ascending by (p, u) */
    for (int64_t u = 0; u < n; ++u)
        for (int32_t p = 0; p < d_out; ++p)
            if (P[u * d_out + p] >= 0) ++start[P[u * d_out + p] + 1];
    for (int64_t v = 0; v < n; ++v) start[v + 1] += start[v];
    rev_t *R = (rev_t *)malloc((size_t)(start[n] > 0 ? start[n] : 1) * sizeof(rev_t));
    int64_t *fill = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    if (!R || !fill) { free(P); free(start); free(R); free(fill); return -1; }
    memcpy(fill, start, (size_t)n * sizeof(int64_t));
    for (int64_t u = 0; u < n; ++u)
        for (int32_t p = 0; p < d_out; ++p) {
            const int32_t v = P[u * d_out + p];
            if (v >= 0) { R[fill[v]].p = p; R[fill[v]].u = (int32_t)u; ++fill[v]; }
        }
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n; ++v)
        qsort(R + start[v], (size_t)(start[v + 1] - start[v]), sizeof(rev_t), rev_cmp);

    /* step 4 */
    const int32_t h = d_out / 2;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n; ++v) {
        int32_t *o = out + v * d_out;
        const int32_t *pv = P + v * d_out;
        int32_t m = 0;
        for (int32_t p = 0; p < d_out - h; ++p) if (pv[p] >= 0) o[m++] = pv[p];
        for (int64_t e = start[v]; e < start[v + 1] && m < d_out; ++e) {
            int dup = 0;
            for (int32_t t = 0; t < m; ++t) dup |= o[t] == R[e].u;
            if (!dup) o[m++] = R[e].u;
        }
        for (int32_t p = d_out - h; p < d_out && m < d_out; ++p) {
            if (pv[p] < 0) continue;
            int dup = 0;
            for (int32_t t = 0; t < m; ++t) dup |= o[t] == pv[p];
            if (!dup) o[m++] = pv[p];
        }
        while (m < d_out) o[m++] = -1;
    }
    free(P); free(start); free(R); free(fill);
    return 0;
}

/* ======================================================================== */
/* Graph-based ANN search (Sec. 3.2): start from given points of the graph,  */
/* greedily explore by visiting neighbours of points already visited, until  */
/* no closer neighbours turn up or the iteration cap is reached; k_s results */
/* per query.  The section describes the search in these words and leaves    */
/* the bookkeeping open; this is the build's reading of it:                  */
/*                                                                           */
/* Per query a list of at most L entries (distance, id, expanded?) is kept   */
/* ascending by (fp32 distance, id), ids distinct.  "Offer x" means: if x is */
/* a valid id (in [0,n)) not in the list, evaluate sigma(query, x) and keep  */
/* the L smallest of the list and x.                                         */
/*   start: offer starts[q][0 .. n_starts) in order.                         */
/*   iteration (at most max_iters): take the first `width` entries of the    */
/*   list that are not yet expanded (stop if there is none), mark them       */
/*   expanded, then for each of them in list order offer its graph row in    */
/*   row order.                                                              */
/* Result: the first k_s entries (padded with id -1 and distance +inf).      */
/* iters_out, evals_out (optional): iterations performed per query, and how   */
/* often "offer x" evaluated sigma for it.  (An implementation that offers a   */
/* whole row at once may skip a repeat inside the row, or an id the row itself */
/* has just pushed out of the list: it evaluates at most this many.)           */
/* Returns 0, or -1 on bad arguments.                                        */
/* ------------------------------------------------------------------------ */
int oracle_graph_search(const float *points, int64_t n, int32_t d, int32_t metric,
                        const int32_t *graph, int32_t deg,
                        const float *queries, int64_t nq,
                        const int32_t *starts, int32_t n_starts,
                        int32_t k_s, int32_t L, int32_t width, int32_t max_iters,
                        int32_t *ids_out, float *dists_out, int32_t *iters_out, int32_t *evals_out)
{
    if (!points || !graph || (!queries && nq > 0) || !starts || !ids_out || !dists_out) return -1;
    if (n < 1 || d < 1 || deg < 1 || nq < 0 || n_starts < 1 || k_s < 1 || L < k_s || width < 1 || max_iters < 0)
        return -1;
    if (metric != ORACLE_L2SQ && metric != ORACLE_IP_UNIT && metric != ORACLE_COSINE) return -1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t q = 0; q < nq; ++q) {
        const float *qv = queries + q * d;
        int32_t *lid = (int32_t *)malloc((size_t)L * sizeof(int32_t));
        float *ld = (float *)malloc((size_t)L * sizeof(float));
        char *lex = (char *)malloc((size_t)L);
        int32_t *par = (int32_t *)malloc((size_t)width * sizeof(int32_t));
        int32_t len = 0, iters = 0, evals = 0;
#define ORACLE_OFFER(x)                                                                     \
        do {                                                                                    \
            const int32_t x_ = (x);                                                             \
            if (x_ < 0 || (int64_t)x_ >= n) break;                                              \
            int in_ = 0;                                                                        \
            for (int32_t t_ = 0; t_ < len; ++t_) in_ |= lid[t_] == x_;                          \
            if (in_) break;                                                                     \
            const float dx_ = oracle_distance(qv, points + (int64_t)x_ * d, d, metric);         \
            ++evals;                                                                            \
            int32_t pos_ = len;                                                                 \
            while (pos_ > 0 && key_less(dx_, x_, ld[pos_ - 1], lid[pos_ - 1])) --pos_;          \
            if (pos_ >= L) break;                                                               \
            const int32_t last_ = len < L ? len : L - 1;                                        \
            for (int32_t t_ = last_; t_ > pos_; --t_) { lid[t_] = lid[t_ - 1]; ld[t_] = ld[t_ - 1]; lex[t_] = lex[t_ - 1]; } \
            lid[pos_] = x_; ld[pos_] = dx_; lex[pos_] = 0;                                      \
            if (len < L) ++len;                                                                 \
        } while (0)
        for (int32_t t = 0; t < n_starts; ++t) ORACLE_OFFER(starts[q * n_starts + t]);
        for (; iters < max_iters; ++iters) {
            int32_t np = 0;
            for (int32_t t = 0; t < len && np < width; ++t)
                if (!lex[t]) { lex[t] = 1; par[np++] = lid[t]; }
            if (np == 0) break;
            for (int32_t a = 0; a < np; ++a)
                for (int32_t j = 0; j < deg; ++j) ORACLE_OFFER(graph[(int64_t)par[a] * deg + j]);
        }
#undef ORACLE_OFFER
        for (int32_t t = 0; t < k_s; ++t) {
            ids_out[q * k_s + t] = t < len ? lid[t] : -1;
            dists_out[q * k_s + t] = t < len ? ld[t] : INFINITY;
        }
        if (iters_out) iters_out[q] = iters;
        if (evals_out) evals_out[q] = evals;
        free(lid); free(ld); free(lex); free(par);
    }
    return 0;
}
