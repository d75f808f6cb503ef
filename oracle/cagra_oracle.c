/*
 * CPU oracle for CAGRA graph construction and greedy graph search.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the method computes; the HIP library is checked against it.  It shares no
 * code with the HIP path and the product never calls it.
 *
 * Everything follows the paper's own order of steps:
 *   - k-NNS definition and recall:                Sec. II-A, Eq. 1, Eq. 2
 *   - reachability measures (2-hop count, CC):     Sec. III-A
 *   - initial k-NN graph, rows sorted by distance: Sec. III-B.1 (exact, or NN-descent in
 *                                                  synchronous rounds)
 *   - rank-based detour count, reorder, prune:     Sec. III-B.2, Eq. 3
 *   - distance-based detour count (the variant the paper compares with):
 *                                                  Sec. III-B.2, Eq. 3 with distances
 *   - reversed graph and interleaved merge:        Sec. III-B.2
 *   - search steps 0..3, termination, output:      Sec. IV-A
 *   - forgettable visited-set management:          Sec. IV-B.3
 *   - parent flag:                                 Sec. IV-B.4
 *   - several workers per query (multi-CTA):       Sec. IV-C.2
 *
 * Readings of the paper where it is silent (each also listed in the design
 * notes of the repository):
 *   T   every (distance, id) comparison is lexicographic: smaller fp32
 *       distance first, then smaller id.  Dummy entries are
 *       (FLT_MAX, 0xFFFFFFFF) and therefore last.
 *   D   distances are fp32 (the paper stores them as float, Sec. IV-A),
 *       accumulated one dimension after the other with a fused multiply-add:
 *       L2 is the squared norm of the difference (no root), inner product
 *       "distance" is 0 - <x, y>.
 *   S4  "top-M indices unchanged" is read on the stored index words, which
 *       include the parent flag (Sec. IV-B.4): the search stops when step 2
 *       finds no entry that has not been a parent yet, or at I_max passes.
 *
 * Pins (tests/test_oracle_*.py): brute force in float64 on integer-valued
 * data where every formula is exact, hand-computable 1-D layouts, the literal
 * definition of Eq. 3 re-derived from set membership, graph invariants,
 * BFS-closure equivalence of the search when M >= N, complete-graph search =
 * exact top-k, forgetting-independence of the result, published SplitMix64
 * outputs for the seed generator.  The multi-worker search: one worker equals
 * the single search; lists longer than the dataset on a strongly connected
 * graph give the float64 brute-force answer with every node in exactly one
 * list; a one-pass run followed by hand (seed slots per worker, ownership in
 * worker order, distance count); the result recomputed as the first k of the
 * union of the returned, disjoint worker lists.
 * parity unpinned: the worked example of Fig. 2 (the figure's ranks are not
 * recoverable).  The lock-step order of the workers is this oracle's reading;
 * a GPU interleaves them differently, so against the GPU only what does not
 * depend on the order is compared id for id.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_INVALID_ID 0xFFFFFFFFu
#define ORACLE_L2 0
#define ORACLE_IP 1

typedef struct {
    float dist;
    uint32_t id;
    int parent; /* Sec. IV-B.4: has this entry been a source of step 2 already */
} entry_t;

/* ---- reading D: the distance ------------------------------------------------ */

static float oracle_dist(const float *x, const float *y, int dim, int metric)
{
    float acc = 0.0f;
    if (metric == ORACLE_L2) {
        for (int j = 0; j < dim; ++j) {
            float t = x[j] - y[j];
            acc = fmaf(t, t, acc);
        }
        return acc;
    }
    for (int j = 0; j < dim; ++j) acc = fmaf(x[j], y[j], acc);
    return 0.0f - acc;
}

float oracle_distance(const float *x, const float *y, int32_t dim, int32_t metric)
{
    return oracle_dist(x, y, dim, metric);
}

/* ---- reading T: the total order --------------------------------------------- */

static int key_less(float da, uint32_t ia, float db, uint32_t ib)
{
    if (da < db) return 1;
    if (da > db) return 0;
    return ia < ib;
}

static int entry_cmp(const void *pa, const void *pb)
{
    const entry_t *a = (const entry_t *)pa, *b = (const entry_t *)pb;
    if (key_less(a->dist, a->id, b->dist, b->id)) return -1;
    if (key_less(b->dist, b->id, a->dist, a->id)) return 1;
    return 0;
}

/* Keep the K smallest (dist, id) seen so far, sorted ascending. */
static void topk_offer(float *bd, uint32_t *bi, int *n, int K, float d, uint32_t id)
{
    if (*n == K && !key_less(d, id, bd[K - 1], bi[K - 1])) return;
    int pos = (*n < K) ? (*n)++ : K - 1;
    while (pos > 0 && key_less(d, id, bd[pos - 1], bi[pos - 1])) {
        bd[pos] = bd[pos - 1];
        bi[pos] = bi[pos - 1];
        --pos;
    }
    bd[pos] = d;
    bi[pos] = id;
}

/* ---- Eq. 1: exact k nearest rows of X for each row of Q --------------------- */
/* exclude_self != 0: Q is X itself addressed through rows[], and row r is not
 * its own neighbour (Sec. III-B.1: the initial k-NN graph has no self edge). */
static int exact_topk(const float *X, int64_t N, int32_t dim, int32_t metric,
                      const float *Q, const int64_t *rows, int64_t B, int32_t K,
                      int exclude_self, uint32_t *ids, float *dists)
{
    if (!X || !Q || !ids || N < 1 || dim < 1 || K < 1 || B < 0) return -1;
    int err = 0;
#pragma omp parallel
    {
        float *bd = (float *)malloc(sizeof(float) * (size_t)K);
        uint32_t *bi = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)K);
        if (!bd || !bi) {
#pragma omp atomic write
            err = 1;
        } else {
#pragma omp for schedule(dynamic, 4)
            for (int64_t b = 0; b < B; ++b) {
                int64_t r = rows ? rows[b] : b;
                const float *q = Q + (size_t)r * (size_t)dim;
                int n = 0;
                for (int64_t y = 0; y < N; ++y) {
                    if (exclude_self && y == r) continue;
                    float d = oracle_dist(q, X + (size_t)y * (size_t)dim, dim, metric);
                    topk_offer(bd, bi, &n, K, d, (uint32_t)y);
                }
                for (int t = 0; t < K; ++t) {
                    ids[(size_t)b * K + t] = t < n ? bi[t] : ORACLE_INVALID_ID;
                    if (dists) dists[(size_t)b * K + t] = t < n ? bd[t] : FLT_MAX;
                }
            }
        }
        free(bd);
        free(bi);
    }
    return err ? -2 : 0;
}

int oracle_exact_search(const float *X, int64_t N, int32_t dim, int32_t metric,
                        const float *Q, int64_t B, int32_t k, uint32_t *ids, float *dists)
{
    return exact_topk(X, N, dim, metric, Q, NULL, B, k, 0, ids, dists);
}

/* Sec. III-B.1 with exact neighbours: rows of the initial graph for the listed
 * nodes (rows == NULL: all N nodes), each sorted ascending under T. */
int oracle_knn_graph(const float *X, int64_t N, int32_t dim, int32_t metric,
                     const int64_t *rows, int64_t n_rows, int32_t d_init,
                     uint32_t *g0, float *g0_dist)
{
    if (d_init >= N) return -1;
    return exact_topk(X, N, dim, metric, X, rows, rows ? n_rows : N, d_init, 1, g0, g0_dist);
}

/* ---- Sec. III-B.1 with NN-descent instead of exact neighbours ------------------ */
/* The paper builds the initial graph with NN-descent (Dong et al., 2011) and
 * gives no details.  Reading taken here (listed in the design notes): the
 * algorithm's principle -- a neighbour of a neighbour is likely a neighbour --
 * in synchronous rounds, every node pulling candidates, so that the result
 * does not depend on the order in which nodes are processed:
 *   round 0   L_0(x) = the k best of k pseudo-random nodes (slot j of node x is
 *             the step-0 generator of the search applied to (seed, x, j));
 *   round t   F(x) = the s entries of L_{t-1}(x) from rank w_t on, with the
 *                    window w_t = min(((t-1) mod ceil(k/s)) * s, k - s) moving
 *                    through the list from round to round (every entry gets to
 *                    propose its own neighbours once per cycle),
 *             R(x) = up to s nodes y with x in F(y), ordered by (rank of x in
 *                    F(y), y)  (reverse neighbours matter: a node nobody
 *                    lists would never be proposed to anyone),
 *             L_t(x) = the k best under T of L_{t-1}(x) and every entry of
 *                    L_{t-1}(v), v in F(x) then R(x), each node once, x left out.
 * Distances are the canonical fp32 ones; those of kept entries are carried. */
int oracle_nn_descent(const float *X, int64_t N, int32_t dim, int32_t metric, int32_t k,
                      int32_t rounds, int32_t s, uint64_t seed, uint32_t *ids, float *dists);

uint32_t oracle_seed_id(uint64_t seed, uint64_t query, uint64_t slot, uint64_t N);

/* k best under T of the entries in e[0..n) with repeated ids and the node `self` dropped;
 * unused slots become dummies */
static void keep_k_best(entry_t *e, int n, int k, uint32_t self, uint32_t *out_id, float *out_d)
{
    qsort(e, (size_t)n, sizeof(entry_t), entry_cmp);
    int m = 0;
    for (int i = 0; i < n && m < k; ++i) {
        if (e[i].id == ORACLE_INVALID_ID || e[i].id == self) continue;
        int dup = 0;
        for (int j = 0; j < m; ++j) dup |= (out_id[j] == e[i].id);   /* same node, same distance: adjacent anyway */
        if (dup) continue;
        out_id[m] = e[i].id;
        out_d[m] = e[i].dist;
        ++m;
    }
    for (; m < k; ++m) { out_id[m] = ORACLE_INVALID_ID; out_d[m] = FLT_MAX; }
}

int oracle_nn_descent(const float *X, int64_t N, int32_t dim, int32_t metric, int32_t k,
                      int32_t rounds, int32_t s, uint64_t seed, uint32_t *ids, float *dists)
{
    if (!X || !ids || !dists || N < 2 || k < 1 || k >= N || rounds < 0 || s < 1 || s > k) return -1;
    uint32_t *prev_id = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N * k);
    float *prev_d = (float *)malloc(sizeof(float) * (size_t)N * k);
    uint32_t *rev = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N * s);
    uint32_t *rev_len = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N);
    if (!prev_id || !prev_d || !rev || !rev_len) { free(prev_id); free(prev_d); free(rev); free(rev_len); return -2; }
    /* round 0 */
#pragma omp parallel
    {
        entry_t *e = (entry_t *)malloc(sizeof(entry_t) * (size_t)k);
#pragma omp for schedule(static)
        for (int64_t x = 0; x < N; ++x) {
            for (int j = 0; j < k; ++j) {
                uint32_t c = oracle_seed_id(seed, (uint64_t)x, (uint64_t)j, (uint64_t)N);
                e[j].id = c; e[j].parent = 0;
                e[j].dist = c == (uint32_t)x ? FLT_MAX : oracle_dist(X + (size_t)x * dim, X + (size_t)c * dim, dim, metric);
            }
            keep_k_best(e, k, k, (uint32_t)x, ids + (size_t)x * k, dists + (size_t)x * k);
        }
        free(e);
    }
    for (int t = 1; t <= rounds; ++t) {
        memcpy(prev_id, ids, sizeof(uint32_t) * (size_t)N * k);
        memcpy(prev_d, dists, sizeof(float) * (size_t)N * k);
        const int n_win = (k + s - 1) / s;
        int win = ((t - 1) % n_win) * s;
        if (win > k - s) win = k - s;
        /* reverse sample: sources in order of (rank, source id), at most s per node */
        memset(rev_len, 0, sizeof(uint32_t) * (size_t)N);
        for (int r = 0; r < s; ++r)
            for (int64_t y = 0; y < N; ++y) {
                uint32_t x = prev_id[(size_t)y * k + win + r];
                if (x != ORACLE_INVALID_ID && rev_len[x] < (uint32_t)s) rev[(size_t)x * s + rev_len[x]++] = (uint32_t)y;
            }
#pragma omp parallel
        {
            const int cap = k + 2 * s * k;
            entry_t *e = (entry_t *)malloc(sizeof(entry_t) * (size_t)cap);
            uint8_t *seen = (uint8_t *)calloc((size_t)N, 1);
#pragma omp for schedule(dynamic, 64)
            for (int64_t x = 0; x < N; ++x) {
                int n = 0;
                seen[x] = 1;
                for (int j = 0; j < k; ++j) {
                    uint32_t c = prev_id[(size_t)x * k + j];
                    e[n].id = c; e[n].dist = prev_d[(size_t)x * k + j]; e[n].parent = 0; ++n;
                    if (c != ORACLE_INVALID_ID) seen[c] = 1;
                }
                const int n_own = n;
                for (int pass = 0; pass < 2; ++pass) {
                    const int np = pass == 0 ? s : (int)rev_len[x];
                    for (int i = 0; i < np; ++i) {
                        uint32_t v = pass == 0 ? prev_id[(size_t)x * k + win + i] : rev[(size_t)x * s + i];
                        if (v == ORACLE_INVALID_ID) continue;
                        for (int j = 0; j < k; ++j) {
                            uint32_t c = prev_id[(size_t)v * k + j];
                            if (c == ORACLE_INVALID_ID || seen[c]) continue;
                            seen[c] = 1;
                            e[n].id = c; e[n].parent = 0;
                            e[n].dist = oracle_dist(X + (size_t)x * dim, X + (size_t)c * dim, dim, metric);
                            ++n;
                        }
                    }
                }
                seen[x] = 0;
                for (int i = 0; i < n; ++i) if (e[i].id != ORACLE_INVALID_ID) seen[e[i].id] = 0;
                (void)n_own;
                keep_k_best(e, n, k, (uint32_t)x, ids + (size_t)x * k, dists + (size_t)x * k);
            }
            free(e);
            free(seen);
        }
    }
    free(prev_id); free(prev_d); free(rev); free(rev_len);
    return 0;
}

/* ---- Sec. III-B.2, Eq. 3 with ranks as weights ------------------------------ */
/* count[X][j] = number of two-hop routes X -> Z -> Y (Y = G0[X][j]) with
 * max(rank of Z in X's list, rank of Y in Z's list) < j. */
/* rows == NULL: all N nodes, count[N][d_init]; else count[n_rows][d_init] for the listed nodes. */
int oracle_detour_count(const uint32_t *g0, int64_t N, int32_t d_init, const int64_t *rows,
                        int64_t n_rows, uint32_t *count)
{
    if (!g0 || !count || N < 1 || d_init < 1) return -1;
    if (!rows) n_rows = N;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < n_rows; ++t) {
        const int64_t x = rows ? rows[t] : t;
        const uint32_t *lx = g0 + (size_t)x * d_init;
        for (int j = 0; j < d_init; ++j) {
            uint32_t y = lx[j];
            uint32_t c = 0;
            for (int i = 0; i < j; ++i) {               /* w(X->Z) = i < j */
                const uint32_t *lz = g0 + (size_t)lx[i] * d_init;
                for (int l = 0; l < j; ++l) {           /* w(Z->Y) = l < j */
                    if (lz[l] == y) { ++c; break; }
                }
            }
            count[(size_t)t * d_init + j] = c;
        }
    }
    return 0;
}

/* ---- Sec. III-B.2, Eq. 3 with distances as weights --------------------------- */
/* The distance-based variant: count[X][j] = number of two-hop routes
 * X -> Z -> Y (Y = G0[X][j], Z in X's list, Y in Z's list) with
 * max(dist(X, Z), dist(Z, Y)) < dist(X, Y), the distances being those stored
 * with the initial graph (g0_dist[N][d_init], the table the paper speaks of). */
int oracle_detour_count_distance(const uint32_t *g0, const float *g0_dist, int64_t N,
                                 int32_t d_init, const int64_t *rows, int64_t n_rows,
                                 uint32_t *count)
{
    if (!g0 || !g0_dist || !count || N < 1 || d_init < 1) return -1;
    if (!rows) n_rows = N;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < n_rows; ++t) {
        const int64_t x = rows ? rows[t] : t;
        const uint32_t *lx = g0 + (size_t)x * d_init;
        const float *dx = g0_dist + (size_t)x * d_init;
        for (int j = 0; j < d_init; ++j) {
            const uint32_t y = lx[j];
            const float wxy = dx[j];
            uint32_t c = 0;
            for (int i = 0; i < d_init; ++i) {
                if (!(dx[i] < wxy)) continue;                     /* w(X->Z) < w(X->Y) */
                const uint32_t *lz = g0 + (size_t)lx[i] * d_init;
                const float *dz = g0_dist + (size_t)lx[i] * d_init;
                for (int l = 0; l < d_init; ++l)
                    if (lz[l] == y) {                             /* the edge Z -> Y exists */
                        if (dz[l] < wxy) ++c;                     /* w(Z->Y) < w(X->Y) */
                        break;
                    }
            }
            count[(size_t)t * d_init + j] = c;
        }
    }
    return 0;
}

/* Reorder each list by (count, initial rank) ascending and keep the first d. */
int oracle_prune(const uint32_t *g0, const uint32_t *count, int64_t N, int32_t d_init,
                 int32_t d, uint32_t *pruned)
{
    if (!g0 || !count || !pruned || d < 1 || d > d_init) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t x = 0; x < N; ++x) {
        const uint32_t *lx = g0 + (size_t)x * d_init;
        const uint32_t *cx = count + (size_t)x * d_init;
        int taken = 0;
        /* selection in ascending (count, j): counts are at most d_init - 1 */
        for (uint32_t c = 0; c < (uint32_t)d_init && taken < d; ++c)
            for (int j = 0; j < d_init && taken < d; ++j)
                if (cx[j] == c) pruned[(size_t)x * d + taken++] = lx[j];
    }
    return 0;
}

/* Reversed graph: node Y lists the sources X of edges X -> Y of the pruned
 * graph, ordered by the edge's rank in X's pruned list (then by X), at most d. */
int oracle_reverse(const uint32_t *pruned, int64_t N, int32_t d, uint32_t *rev,
                   uint32_t *rev_len)
{
    if (!pruned || !rev || !rev_len) return -1;
    memset(rev_len, 0, sizeof(uint32_t) * (size_t)N);
    for (int r = 0; r < d; ++r)
        for (int64_t x = 0; x < N; ++x) {
            uint32_t y = pruned[(size_t)x * d + r];
            if (rev_len[y] < (uint32_t)d) rev[(size_t)y * d + rev_len[y]++] = (uint32_t)x;
        }
    return 0;
}

/* Interleave: even slots from the pruned list, odd slots from the reversed
 * list while it lasts (at most d/2 of them), duplicates skipped on both sides,
 * the pruned list fills whatever the reversed list cannot. */
int oracle_merge(const uint32_t *pruned, const uint32_t *rev, const uint32_t *rev_len,
                 int64_t N, int32_t d, uint32_t *graph)
{
    if (!pruned || !rev || !rev_len || !graph || d < 2 || (d & 1)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t y = 0; y < N; ++y) {
        const uint32_t *p = pruned + (size_t)y * d;
        const uint32_t *r = rev + (size_t)y * d;
        uint32_t *out = graph + (size_t)y * d;
        int nr = (int)rev_len[y], ip = 0, ir = 0, nrev = 0;
        for (int slot = 0; slot < d; ++slot) {
            int done = 0;
            if ((slot & 1) && nrev < d / 2) {
                for (; ir < nr; ++ir) {
                    int dup = 0;
                    for (int t = 0; t < slot; ++t) dup |= (out[t] == r[ir]);
                    if (!dup) break;
                }
                if (ir < nr) { out[slot] = r[ir++]; ++nrev; done = 1; }
            }
            if (!done) {
                for (;; ++ip) {
                    int dup = 0;
                    for (int t = 0; t < slot; ++t) dup |= (out[t] == p[ip]);
                    if (!dup) break;
                }
                out[slot] = p[ip++];
            }
        }
    }
    return 0;
}

/* Whole optimisation: initial sorted k-NN graph -> CAGRA graph of degree d.
 * g0_dist == NULL: rank-based reordering (what CAGRA adopts); else distance-based. */
int oracle_optimize_ex(const uint32_t *g0, const float *g0_dist, int64_t N, int32_t d_init,
                       int32_t d, uint32_t *graph);

int oracle_optimize(const uint32_t *g0, int64_t N, int32_t d_init, int32_t d, uint32_t *graph)
{
    return oracle_optimize_ex(g0, NULL, N, d_init, d, graph);
}

int oracle_optimize_ex(const uint32_t *g0, const float *g0_dist, int64_t N, int32_t d_init,
                       int32_t d, uint32_t *graph)
{
    if (!g0 || !graph || N < 1 || d < 2 || (d & 1) || d > d_init) return -1;
    uint32_t *count = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N * d_init);
    uint32_t *pruned = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N * d);
    uint32_t *rev = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N * d);
    uint32_t *rev_len = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N);
    int rc = -2;
    if (count && pruned && rev && rev_len) {
        rc = g0_dist ? oracle_detour_count_distance(g0, g0_dist, N, d_init, NULL, N, count)
                     : oracle_detour_count(g0, N, d_init, NULL, N, count);
        if (!rc) rc = oracle_prune(g0, count, N, d_init, d, pruned);
        if (!rc) rc = oracle_reverse(pruned, N, d, rev, rev_len);
        if (!rc) rc = oracle_merge(pruned, rev, rev_len, N, d, graph);
    }
    free(count); free(pruned); free(rev); free(rev_len);
    return rc;
}

/* reorder: 0 rank-based, 1 distance-based */
int oracle_build_ex(const float *X, int64_t N, int32_t dim, int32_t metric, int32_t d,
                    int32_t d_init, int32_t reorder, uint32_t *graph)
{
    if (d_init == 0) d_init = 2 * d;
    if (!X || !graph || N < 2 || d_init >= N || reorder < 0 || reorder > 1) return -1;
    uint32_t *g0 = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N * d_init);
    float *gd = reorder ? (float *)malloc(sizeof(float) * (size_t)N * d_init) : NULL;
    int rc = -2;
    if (g0 && (gd || !reorder)) {
        rc = oracle_knn_graph(X, N, dim, metric, NULL, N, d_init, g0, gd);
        if (!rc) rc = oracle_optimize_ex(g0, gd, N, d_init, d, graph);
    }
    free(g0);
    free(gd);
    return rc;
}

int oracle_build(const float *X, int64_t N, int32_t dim, int32_t metric, int32_t d,
                 int32_t d_init, uint32_t *graph)
{
    return oracle_build_ex(X, N, dim, metric, d, d_init, 0, graph);
}

/* ---- Sec. III-A: how reachability of a graph is measured ---------------------- */
/* 2-hop node count of X: the number of nodes other than X that can be reached
 * from X in one or two steps (at most d + d^2). */
int oracle_two_hop_counts(const uint32_t *graph, int64_t N, int32_t d, uint32_t *counts)
{
    if (!graph || !counts || N < 1 || d < 1) return -1;
#pragma omp parallel
    {
        uint8_t *seen = (uint8_t *)calloc((size_t)N, 1);
        uint32_t *list = (uint32_t *)malloc(sizeof(uint32_t) * ((size_t)d + (size_t)d * d));
#pragma omp for schedule(dynamic, 256)
        for (int64_t x = 0; x < N; ++x) {
            size_t n = 0;
            if (!seen || !list) { counts[x] = 0; continue; }
            seen[x] = 1;
            for (int i = 0; i < d; ++i) {
                uint32_t y = graph[(size_t)x * d + i];
                if (!seen[y]) { seen[y] = 1; list[n++] = y; }
                for (int j = 0; j < d; ++j) {
                    uint32_t z = graph[(size_t)y * d + j];
                    if (!seen[z]) { seen[z] = 1; list[n++] = z; }
                }
            }
            counts[x] = (uint32_t)n;
            seen[x] = 0;
            for (size_t t = 0; t < n; ++t) seen[list[t]] = 0;
        }
        free(seen);
        free(list);
    }
    return 0;
}

/* Number of strongly connected components (every node of a component reaches
 * every other one along directed edges): Tarjan's algorithm with an explicit
 * stack.  Returns -1 on bad arguments, -2 when out of memory. */
int64_t oracle_strong_components(const uint32_t *graph, int64_t N, int32_t d)
{
    if (!graph || N < 1 || d < 1) return -1;
    int64_t *index = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);   /* discovery order, -1 = new */
    int64_t *low = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
    uint8_t *on_stack = (uint8_t *)calloc((size_t)N, 1);
    uint32_t *stack = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N);       /* Tarjan's node stack */
    uint32_t *call_node = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N);   /* recursion, unrolled */
    int32_t *call_edge = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    int64_t n_comp = -2;
    if (index && low && on_stack && stack && call_node && call_edge) {
        int64_t next = 0, sp = 0;
        n_comp = 0;
        for (int64_t v = 0; v < N; ++v) index[v] = -1;
        for (int64_t root = 0; root < N; ++root) {
            if (index[root] >= 0) continue;
            int64_t cp = 0;
            call_node[0] = (uint32_t)root; call_edge[0] = 0;
            index[root] = low[root] = next++;
            stack[sp++] = (uint32_t)root; on_stack[root] = 1;
            while (cp >= 0) {
                const uint32_t v = call_node[cp];
                if (call_edge[cp] < d) {
                    const uint32_t w = graph[(size_t)v * d + call_edge[cp]++];
                    if (index[w] < 0) {
                        index[w] = low[w] = next++;
                        stack[sp++] = w; on_stack[w] = 1;
                        ++cp; call_node[cp] = w; call_edge[cp] = 0;
                    } else if (on_stack[w] && index[w] < low[v]) {
                        low[v] = index[w];
                    }
                } else {
                    if (low[v] == index[v]) {            /* v is the root of a component */
                        uint32_t w;
                        do { w = stack[--sp]; on_stack[w] = 0; } while (w != v);
                        ++n_comp;
                    }
                    --cp;
                    if (cp >= 0 && low[v] < low[call_node[cp]]) low[call_node[cp]] = low[v];
                }
            }
        }
    }
    free(index); free(low); free(on_stack); free(stack); free(call_node); free(call_edge);
    return n_comp;
}

/* Number of weakly connected components (edge directions ignored): union-find. */
int64_t oracle_weak_components(const uint32_t *graph, int64_t N, int32_t d)
{
    if (!graph || N < 1 || d < 1) return -1;
    uint32_t *parent = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N);
    if (!parent) return -2;
    for (int64_t v = 0; v < N; ++v) parent[v] = (uint32_t)v;
    for (int64_t v = 0; v < N; ++v)
        for (int i = 0; i < d; ++i) {
            uint32_t a = (uint32_t)v, b = graph[(size_t)v * d + i];
            while (parent[a] != a) { parent[a] = parent[parent[a]]; a = parent[a]; }
            while (parent[b] != b) { parent[b] = parent[parent[b]]; b = parent[b]; }
            if (a != b) parent[a > b ? a : b] = a > b ? b : a;
        }
    int64_t n_comp = 0;
    for (int64_t v = 0; v < N; ++v) n_comp += parent[v] == (uint32_t)v;
    free(parent);
    return n_comp;
}

/* ---- step 0 seed generator --------------------------------------------------- */
/* The paper asks only for "a pseudo-random number generator".  Reading: a
 * stateless counter-based one, the SplitMix64 output function applied twice,
 * first over (seed, query), then over the slot; the top 32 bits are scaled
 * to [0, N) by a multiply-shift. */
uint64_t oracle_splitmix_fin(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint32_t oracle_seed_id(uint64_t seed, uint64_t query, uint64_t slot, uint64_t N)
{
    const uint64_t G = 0x9E3779B97F4A7C15ull;
    uint64_t h = oracle_splitmix_fin(seed + G * (query + 1));
    h = oracle_splitmix_fin(h + G * (slot + 1));
    return (uint32_t)(((h >> 32) * N) >> 32);
}

/* ---- Sec. IV-A: the search ---------------------------------------------------- */

int32_t oracle_auto_max_iterations(int32_t itopk, int32_t search_width)
{
    return 2 * ((itopk + search_width - 1) / search_width) + 32;
}

typedef struct {
    uint8_t *mark;      /* N flags: id has been in a candidate list (Sec. IV-B.3) */
    uint32_t *marked;   /* ids whose flag is set, to undo them */
    size_t n_marked, cap_marked;
} visited_t;

static int visited_test_and_set(visited_t *v, uint32_t id)
{
    if (v->mark[id]) return 1;
    v->mark[id] = 1;
    if (v->n_marked == v->cap_marked) {
        size_t nc = v->cap_marked ? 2 * v->cap_marked : 1024;
        uint32_t *p = (uint32_t *)realloc(v->marked, nc * sizeof(uint32_t));
        if (!p) abort();
        v->marked = p;
        v->cap_marked = nc;
    }
    v->marked[v->n_marked++] = id;
    return 0;
}

static void visited_clear(visited_t *v)
{
    for (size_t t = 0; t < v->n_marked; ++t) v->mark[v->marked[t]] = 0;
    v->n_marked = 0;
}

/* Step 3 for one candidate slot: distance only on first appearance. */
static void fill_candidate(entry_t *e, uint32_t id, visited_t *vis, const float *X,
                           int32_t dim, int32_t metric, const float *q, uint32_t *n_dist)
{
    e->parent = 0;
    if (id == ORACLE_INVALID_ID || visited_test_and_set(vis, id)) {
        e->dist = FLT_MAX;
        e->id = ORACLE_INVALID_ID;
        return;
    }
    e->dist = oracle_dist(q, X + (size_t)id * (size_t)dim, dim, metric);
    e->id = id;
    ++*n_dist;
}

/* One worker's state: buffer = [top-M list | candidate list] (Sec. IV-A). */
typedef struct {
    entry_t *buf;
    int M, n_cand;
    int done;
} worker_t;

/* Step 1: the M smallest of the whole buffer become the top-M list. */
static void update_topm(worker_t *w)
{
    qsort(w->buf, (size_t)(w->M + w->n_cand), sizeof(entry_t), entry_cmp);
}

/*
 * The search of one query with W workers sharing one visited set.  W = 1 is
 * the single-CTA search with p = search_width parents per pass; W > 1 is the
 * multi-CTA search: every worker has p = 1, its own d seeds, its own list of
 * length M_local, and the workers advance in lock step, worker 0 first.
 * reset_interval > 0 simulates the forgettable management: every that many
 * passes the visited set is emptied and the current top-M ids re-registered.
 */
static void search_one(const uint32_t *graph, int64_t N, int32_t d, const float *X, int32_t dim,
                       int32_t metric, const float *q, int64_t qi, int32_t k, int32_t M_local,
                       int32_t p, int32_t W, uint64_t seed, int32_t max_iter,
                       int32_t reset_interval, visited_t *vis, worker_t *wk,
                       uint32_t *ids, float *dists, uint32_t *stats, uint32_t *lists)
{
    uint32_t n_dist = 0, n_parent = 0, n_iter = 0, hit_cap = 0;
    const int n_cand = p * d;
    /* step 0: dummy top-M, random candidates */
    for (int w = 0; w < W; ++w) {
        wk[w].M = M_local;
        wk[w].n_cand = n_cand;
        wk[w].done = 0;
        for (int t = 0; t < M_local; ++t) {
            wk[w].buf[t].dist = FLT_MAX;
            wk[w].buf[t].id = ORACLE_INVALID_ID;
            wk[w].buf[t].parent = 0;
        }
        for (int s = 0; s < n_cand; ++s) {
            uint32_t id = oracle_seed_id(seed, (uint64_t)qi, (uint64_t)w * n_cand + s, (uint64_t)N);
            fill_candidate(&wk[w].buf[M_local + s], id, vis, X, dim, metric, q, &n_dist);
        }
    }
    for (int32_t it = 0;; ++it) {
        int live = 0;
        for (int w = 0; w < W; ++w)
            if (!wk[w].done) update_topm(&wk[w]);                     /* step 1 */
        if (it == max_iter) { hit_cap = 1; break; }
        if (reset_interval > 0 && it > 0 && it % reset_interval == 0) {
            visited_clear(vis);
            for (int w = 0; w < W; ++w)
                for (int t = 0; t < wk[w].M; ++t)
                    if (wk[w].buf[t].id != ORACLE_INVALID_ID)
                        visited_test_and_set(vis, wk[w].buf[t].id);
        }
        for (int w = 0; w < W; ++w) {
            if (wk[w].done) continue;
            entry_t *top = wk[w].buf, *cand = wk[w].buf + wk[w].M;
            int n_par = 0;
            uint32_t par[64];
            for (int t = 0; t < wk[w].M && n_par < p; ++t)            /* step 2 */
                if (top[t].id != ORACLE_INVALID_ID && !top[t].parent) {
                    top[t].parent = 1;
                    par[n_par++] = top[t].id;
                }
            if (n_par == 0) { wk[w].done = 1; wk[w].n_cand = 0; continue; }
            ++live;
            n_parent += (uint32_t)n_par;
            for (int s = 0; s < n_cand; ++s) {                        /* step 3 */
                uint32_t id = (s / d < n_par) ? graph[(size_t)par[s / d] * d + s % d]
                                              : ORACLE_INVALID_ID;
                fill_candidate(&cand[s], id, vis, X, dim, metric, q, &n_dist);
            }
        }
        if (!live) break;
        ++n_iter;
    }
    /* for inspection: every worker's final list, ids only, [W, M_local] */
    if (lists)
        for (int w = 0; w < W; ++w)
            for (int t = 0; t < M_local; ++t) lists[(size_t)w * M_local + t] = wk[w].buf[t].id;
    /* output: the first k under T of the union of the workers' lists */
    if (W == 1) {
        for (int t = 0; t < k; ++t) {
            ids[t] = wk[0].buf[t].id;
            dists[t] = wk[0].buf[t].dist;
        }
    } else {
        entry_t *all = (entry_t *)malloc(sizeof(entry_t) * (size_t)W * M_local);
        if (!all) abort();
        for (int w = 0; w < W; ++w) memcpy(all + (size_t)w * M_local, wk[w].buf, sizeof(entry_t) * M_local);
        qsort(all, (size_t)W * M_local, sizeof(entry_t), entry_cmp);
        for (int t = 0; t < k; ++t) {
            ids[t] = all[t].id;
            dists[t] = all[t].dist;
        }
        free(all);
    }
    if (stats) {
        stats[0] = n_iter;
        stats[1] = n_parent;
        stats[2] = n_dist;
        stats[3] = hit_cap;
    }
    visited_clear(vis);
}

static int search_batch(const uint32_t *graph, int64_t N, int32_t d, const float *X, int32_t dim,
                        int32_t metric, const float *Q, int64_t B, int32_t k, int32_t M_local,
                        int32_t p, int32_t W, uint64_t seed, int32_t max_iter,
                        int32_t reset_interval, int32_t n_threads,
                        uint32_t *ids, float *dists, uint32_t *stats, uint32_t *lists)
{
    if (!graph || !X || !Q || !ids || !dists) return -1;
    if (N < 1 || N >= ((int64_t)1 << 31) || d < 1 || dim < 1 || B < 0) return -1;
    if (k < 1 || p < 1 || p > 64 || W < 1 || M_local < 1 || (int64_t)W * M_local < k) return -1;
    if (max_iter < 0) return -1;
    int err = 0;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
#else
    n_threads = 1;
#endif
#pragma omp parallel num_threads(n_threads)
    {
        visited_t vis = {0};
        vis.mark = (uint8_t *)calloc((size_t)N, 1);
        worker_t *wk = (worker_t *)calloc((size_t)W, sizeof(worker_t));
        int ok = vis.mark && wk;
        for (int w = 0; ok && w < W; ++w) {
            wk[w].buf = (entry_t *)malloc(sizeof(entry_t) * (size_t)(M_local + p * d));
            ok = wk[w].buf != NULL;
        }
        if (!ok) {
#pragma omp atomic write
            err = 1;
        }
#pragma omp for schedule(dynamic, 8)
        for (int64_t b = 0; b < B; ++b) {
            if (!ok) continue;
            search_one(graph, N, d, X, dim, metric, Q + (size_t)b * dim, b, k, M_local, p, W, seed,
                       max_iter, reset_interval, &vis, wk, ids + (size_t)b * k,
                       dists + (size_t)b * k, stats ? stats + (size_t)b * 4 : NULL,
                       lists ? lists + (size_t)b * W * M_local : NULL);
        }
        if (wk) for (int w = 0; w < W; ++w) free(wk[w].buf);
        free(wk);
        free(vis.mark);
        free(vis.marked);
    }
    return err ? -2 : 0;
}

/* Single-CTA search (Sec. IV-A, IV-C.1): M = itopk, p = search_width. */
int oracle_search(const uint32_t *graph, int64_t N, int32_t d, const float *X, int32_t dim,
                  int32_t metric, const float *Q, int64_t B, int32_t k, int32_t itopk,
                  int32_t search_width, uint64_t seed, int32_t max_iter, int32_t reset_interval,
                  int32_t n_threads, uint32_t *ids, float *dists, uint32_t *stats)
{
    if (k > itopk) return -1;
    if (max_iter == 0) max_iter = oracle_auto_max_iterations(itopk, search_width);
    return search_batch(graph, N, d, X, dim, metric, Q, B, k, itopk, search_width, 1, seed,
                        max_iter, reset_interval, n_threads, ids, dists, stats, NULL);
}

/* Multi-CTA search (Sec. IV-C.2): W workers, p = 1 each, local lists of M_local. */
int oracle_search_multi(const uint32_t *graph, int64_t N, int32_t d, const float *X, int32_t dim,
                        int32_t metric, const float *Q, int64_t B, int32_t k, int32_t M_local,
                        int32_t W, uint64_t seed, int32_t max_iter, int32_t n_threads,
                        uint32_t *ids, float *dists, uint32_t *stats)
{
    if (max_iter <= 0) return -1;
    return search_batch(graph, N, d, X, dim, metric, Q, B, k, M_local, 1, W, seed, max_iter, 0,
                        n_threads, ids, dists, stats, NULL);
}

/* The same, also returning every worker's final list (ids, [B, W, M_local]; unused slots
 * ORACLE_INVALID_ID) so that the seed layout, the ownership of nodes and the final merge can
 * be checked from outside. */
int oracle_search_multi_lists(const uint32_t *graph, int64_t N, int32_t d, const float *X, int32_t dim,
                              int32_t metric, const float *Q, int64_t B, int32_t k, int32_t M_local,
                              int32_t W, uint64_t seed, int32_t max_iter, int32_t n_threads,
                              uint32_t *ids, float *dists, uint32_t *stats, uint32_t *lists)
{
    if (max_iter <= 0 || !lists) return -1;
    return search_batch(graph, N, d, X, dim, metric, Q, B, k, M_local, 1, W, seed, max_iter, 0,
                        n_threads, ids, dists, stats, lists);
}

int32_t oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
