/*
 * rnnd_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, single-threaded CPU statement of the graph-construction
 * method of "Relative NN-Descent" (arXiv 2310.20419), in the synchronous-round
 * variant this repository defines.  It exists so that the GPU library can be
 * checked against something written directly from the paper.  Only tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it; the product
 * never does.  It shares no code, header, table or helper with the GPU path.
 *
 * The method is a heuristic iteration, so this file takes the algorithm's
 * steps in the paper's order and notation:
 *
 *   Alg. 6 (RNN-Descent)      -> orc_build_sync / orc_build_blocks / orc_build_paper_order
 *   Alg. 4 (UpdateNeighbors)  -> orc_update_neighbors_sync / _blocks / update_paper_order
 *   Alg. 5 (AddReverseEdges)  -> orc_add_reverse_edges
 *   Alg. 3 (RNGStrategy)      -> orc_rng_strategy
 *   Alg. 1 (Search) + Eq. 4   -> orc_search
 *   Eq. 3  (delta)            -> delta()
 *
 * Readings of points the paper leaves open (each also listed in the design
 * document):
 *   - delta is squared Euclidean distance (every comparison in Alg. 3-5 is
 *     monotone in it).  uint8 data: exact integer.  float data: accumulated in
 *     double in index order, rounded once to float.
 *   - sort order is ascending (delta, id); ties in Alg. 4's test prune (>=).
 *   - the redirected edge of Alg. 4 is (w, v): v enters w's list (Fig. 1(c),
 *     the algorithm box, and the reachability argument of Sec. 4.2).
 *   - a flag belongs to a directed edge entry.
 *   - synchronous round: every vertex is scanned against the same snapshot,
 *     then each list becomes the R first entries, in (delta, id) order, of
 *     kept + redirected edges, without duplicates (an existing entry wins).
 *   - Alg. 5: union, then cap out-lists to R, then cap in-lists to R, each
 *     keeping the shortest by (delta, other endpoint).
 *   - RandomGraph(S): S distinct ids != u from a counter-based generator
 *     (splitmix64 finaliser), so that two implementations agree by
 *     specification.
 *
 * Parity status: exact adjacency on general inputs is pinned by nothing but
 * this file ("parity unpinned" beyond the pins in tests/test_oracle_*.py: the
 * Fig. 1(c) worked example, reduction to Alg. 3 under complete initialisation,
 * the exact relative-neighbourhood graph, the 1-D path-graph fixed point, the
 * RNG inequality Eq. 2, degree bounds, flag-skip equivalence, brute force).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#include <stdio.h>

#define ORC_U8 0
#define ORC_F32 1

typedef struct {
    double dist;   /* delta(owner, id): an exact int for u8, a float value for f32 */
    int32_t id;
    int32_t is_new; /* 1 = "new", 0 = "old" */
} entry_t;

typedef struct {
    entry_t *e;
    int32_t len, cap;
} list_t;

typedef struct {
    const void *X;
    int64_t n;
    int32_t d;
    int dtype;
} data_t;

/* ------------------------------------------------------------------ Eq. 3 */
static double delta_vec(const data_t *D, const void *a, const void *b)
{
    if (D->dtype == ORC_U8) {
        const uint8_t *p = (const uint8_t *)a, *q = (const uint8_t *)b;
        int64_t s = 0;
        for (int32_t k = 0; k < D->d; ++k) {
            int64_t t = (int64_t)p[k] - (int64_t)q[k];
            s += t * t;
        }
        return (double)s;
    } else {
        const float *p = (const float *)a, *q = (const float *)b;
        double s = 0.0;
        for (int32_t k = 0; k < D->d; ++k) {
            double t = (double)p[k] - (double)q[k];
            s += t * t;
        }
        return (double)(float)s;
    }
}

static const void *row_ptr(const data_t *D, const void *base, int64_t i)
{
    size_t es = D->dtype == ORC_U8 ? 1 : 4;
    return (const char *)base + (size_t)i * (size_t)D->d * es;
}

static double delta(const data_t *D, int64_t a, int64_t b)
{
    return delta_vec(D, row_ptr(D, D->X, a), row_ptr(D, D->X, b));
}

/* --------------------------------------------------------------- list ops */
static void list_push(list_t *L, entry_t x)
{
    if (L->len == L->cap) {
        L->cap = L->cap ? 2 * L->cap : 8;
        L->e = (entry_t *)realloc(L->e, (size_t)L->cap * sizeof(entry_t));
    }
    L->e[L->len++] = x;
}

static int list_has(const list_t *L, int32_t id)
{
    for (int32_t i = 0; i < L->len; ++i)
        if (L->e[i].id == id) return 1;
    return 0;
}

/* ascending (delta, id); among equal (delta, id) an "old" entry comes first */
static int entry_cmp(const void *pa, const void *pb)
{
    const entry_t *a = (const entry_t *)pa, *b = (const entry_t *)pb;
    if (a->dist < b->dist) return -1;
    if (a->dist > b->dist) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return a->is_new - b->is_new;
}

static void list_sort(list_t *L)
{
    qsort(L->e, (size_t)L->len, sizeof(entry_t), entry_cmp);
}

/* sort, drop later entries whose id already appeared, keep the first R */
static void list_canonicalise(list_t *L, int32_t R)
{
    list_sort(L);
    int32_t m = 0;
    for (int32_t i = 0; i < L->len && m < R; ++i) {
        int dup = 0;
        for (int32_t j = 0; j < m; ++j)
            if (L->e[j].id == L->e[i].id) { dup = 1; break; }
        if (!dup) L->e[m++] = L->e[i];
    }
    L->len = m;
}

static list_t *graph_alloc(int64_t n)
{
    return (list_t *)calloc((size_t)n, sizeof(list_t));
}

static void graph_free(list_t *G, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) free(G[i].e);
    free(G);
}

/* flat snapshot <-> lists.  Row u of the flat arrays holds deg[u] entries. */
static list_t *graph_from_flat(int64_t n, int32_t W, const int32_t *ids, const double *dist,
                               const uint8_t *flags, const int32_t *deg)
{
    list_t *G = graph_alloc(n);
    for (int64_t u = 0; u < n; ++u)
        for (int32_t k = 0; k < deg[u]; ++k) {
            entry_t x;
            x.id = ids[u * W + k];
            x.dist = dist[u * W + k];
            x.is_new = flags[u * W + k] ? 1 : 0;
            list_push(&G[u], x);
        }
    return G;
}

/* writes at most W entries per row (nearest first); returns the largest list length seen */
static int32_t graph_to_flat(const list_t *G, int64_t n, int32_t W, int32_t *ids, double *dist,
                             uint8_t *flags, int32_t *deg)
{
    int32_t maxlen = 0;
    for (int64_t u = 0; u < n; ++u) {
        int32_t m = G[u].len < W ? G[u].len : W;
        if (G[u].len > maxlen) maxlen = G[u].len;
        deg[u] = m;
        for (int32_t k = 0; k < W; ++k) {
            if (k < m) {
                ids[u * W + k] = G[u].e[k].id;
                if (dist) dist[u * W + k] = G[u].e[k].dist;
                if (flags) flags[u * W + k] = (uint8_t)G[u].e[k].is_new;
            } else {
                ids[u * W + k] = -1;
                if (dist) dist[u * W + k] = 0.0;
                if (flags) flags[u * W + k] = 0;
            }
        }
    }
    return maxlen;
}

/* ------------------------------------- RandomGraph (first step of Alg. 6) */
/* splitmix64 output function (Steele, Lea, Flood 2014; Vigna's reference). */
static uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

#define GOLDEN 0x9E3779B97F4A7C15ULL

uint64_t orc_mix64(uint64_t z) { return mix64(z); }

/* j-th draw of vertex u: a 64-bit word that depends on (seed, u, j) only */
uint64_t orc_draw(uint64_t seed, uint64_t u, uint64_t j)
{
    return mix64(mix64(seed + GOLDEN * (u + 1)) + GOLDEN * (j + 1));
}

/* S distinct neighbours != u.  Draws j = 0,1,.. map to [0,n-1) by the high
 * 32 bits times (n-1) >> 32, then skip over u; a repeated id is ignored.  After
 * 64*S+1024 draws (never reached in practice) the smallest unused ids fill up. */
static void random_row(uint64_t seed, int64_t n, int64_t u, int32_t S, int32_t *out)
{
    int32_t cnt = 0;
    uint64_t jmax = 64ULL * (uint64_t)S + 1024ULL;
    for (uint64_t j = 0; j < jmax && cnt < S; ++j) {
        uint64_t z = orc_draw(seed, (uint64_t)u, j);
        uint64_t c = ((z >> 32) * (uint64_t)(n - 1)) >> 32;
        int32_t id = (int32_t)(c + (c >= (uint64_t)u ? 1 : 0));
        int dup = 0;
        for (int32_t k = 0; k < cnt; ++k)
            if (out[k] == id) { dup = 1; break; }
        if (!dup) out[cnt++] = id;
    }
    for (int64_t id = 0; id < n && cnt < S; ++id) {
        if (id == u) continue;
        int dup = 0;
        for (int32_t k = 0; k < cnt; ++k)
            if (out[k] == (int32_t)id) { dup = 1; break; }
        if (!dup) out[cnt++] = (int32_t)id;
    }
}

static list_t *random_graph(const data_t *D, int32_t S, uint64_t seed)
{
    list_t *G = graph_alloc(D->n);
    int32_t *tmp = (int32_t *)malloc((size_t)S * sizeof(int32_t));
    for (int64_t u = 0; u < D->n; ++u) {
        random_row(seed, D->n, u, S, tmp);
        for (int32_t k = 0; k < S; ++k) {
            entry_t x;
            x.id = tmp[k];
            x.dist = delta(D, u, tmp[k]);
            x.is_new = 1;                       /* Alg. 6: all flags start as new */
            list_push(&G[u], x);
        }
        list_sort(&G[u]);
    }
    free(tmp);
    return G;
}

/* ------------------------------------------- UpdateNeighbors (Alg. 4), scan */
/* One vertex of Alg. 4 against its own list L (sorted on entry).  Kept entries
 * go to `kept` (flags old); each pruned v calls emit(w, v, delta(v,w)). */
typedef struct { int32_t target, id; double dist; } proposal_t;

typedef struct {
    proposal_t *p;
    int64_t len, cap;
} plist_t;

static void plist_push(plist_t *P, proposal_t x)
{
    if (P->len == P->cap) {
        P->cap = P->cap ? 2 * P->cap : 1024;
        P->p = (proposal_t *)realloc(P->p, (size_t)P->cap * sizeof(proposal_t));
    }
    P->p[P->len++] = x;
}

static void scan_vertex(const data_t *D, const list_t *U, int use_flag_skip, list_t *kept,
                        plist_t *props, int64_t *evals)
{
    kept->len = 0;
    for (int32_t i = 0; i < U->len; ++i) {               /* for v in U, ascending */
        entry_t v = U->e[i];
        int f = 1;                                       /* v is kept unless a test fires */
        for (int32_t j = 0; j < kept->len; ++j) {        /* for w in U', in order */
            entry_t w = kept->e[j];
            if (use_flag_skip && !v.is_new && !w.is_new) /* both old: skip */
                continue;
            double dvw = delta(D, v.id, w.id);
            ++*evals;
            if (v.dist >= dvw) {                         /* the prune test: delta(u,v) >= delta(v,w) */
                f = 0;
                proposal_t p;                            /* redirect: E <- E \ (u,v) + (w,v) */
                p.target = w.id; p.id = v.id; p.dist = dvw;
                plist_push(props, p);
                break;                                   /* first failing w only */
            }
        }
        if (f) list_push(kept, v);                       /* v joins U', flag kept as read */
    }
}

/* Synchronous round: all scans read the snapshot G; then every list is rebuilt. */
static void update_neighbors_sync(const data_t *D, list_t *G, int32_t R, int use_flag_skip,
                                  int64_t *evals, int64_t *nprops)
{
    int64_t n = D->n;
    list_t *K = graph_alloc(n);
    plist_t P = {0, 0, 0};
    for (int64_t u = 0; u < n; ++u) {
        scan_vertex(D, &G[u], use_flag_skip, &K[u], &P, evals);
        for (int32_t k = 0; k < K[u].len; ++k) K[u].e[k].is_new = 0;   /* kept: old */
    }
    *nprops += P.len;
    for (int64_t i = 0; i < P.len; ++i) {
        entry_t x;
        x.id = P.p[i].id; x.dist = P.p[i].dist; x.is_new = 1;
        list_push(&K[P.p[i].target], x);
    }
    for (int64_t u = 0; u < n; ++u) {
        list_canonicalise(&K[u], R);
        free(G[u].e);
        G[u] = K[u];
    }
    free(K);
    free(P.p);
}

/* Block-sequential pass (between the synchronous round and the paper's in-place order): the
 * vertices are cut into nblocks runs of consecutive ids, ceil(n / nblocks) each, which take their
 * turn in id order.  Every vertex of a run is scanned against the graph as it stands when the run
 * starts; the run's redirected edges enter their targets' lists (any vertex; lists cut to R as in
 * the synchronous round) before the next run starts, so later runs of the same pass see them, as
 * later vertices do in Alg. 4's own loop.  nblocks = 1 is the synchronous round; nblocks = n is
 * Alg. 4's vertex order. */
static void update_neighbors_blocks(const data_t *D, list_t *G, int32_t R, int64_t nblocks,
                                    int64_t *evals, int64_t *nprops)
{
    int64_t n = D->n, bs = (n + nblocks - 1) / nblocks;
    plist_t P = {0, 0, 0};
    char *dirty = (char *)calloc((size_t)n, 1);
    for (int64_t lo = 0; lo < n; lo += bs) {
        int64_t hi = lo + bs < n ? lo + bs : n;
        list_t *K = graph_alloc(hi - lo);
        P.len = 0;
        for (int64_t u = lo; u < hi; ++u) {
            scan_vertex(D, &G[u], 1, &K[u - lo], &P, evals);
            for (int32_t k = 0; k < K[u - lo].len; ++k) K[u - lo].e[k].is_new = 0;   /* kept: old */
        }
        for (int64_t u = lo; u < hi; ++u) {
            free(G[u].e);
            G[u] = K[u - lo];
        }
        free(K);
        *nprops += P.len;
        for (int64_t i = 0; i < P.len; ++i) {            /* the redirect: v enters w's list, flagged new */
            entry_t x;
            x.id = P.p[i].id; x.dist = P.p[i].dist; x.is_new = 1;
            list_push(&G[P.p[i].target], x);
            dirty[P.p[i].target] = 1;
        }
        for (int64_t i = 0; i < P.len; ++i)
            if (dirty[P.p[i].target]) {
                list_canonicalise(&G[P.p[i].target], R);
                dirty[P.p[i].target] = 0;
            }
    }
    free(dirty);
    free(P.p);
}

/* Paper order: vertices in index order, every redirect applied at once to w's
 * list (no cap on the list length, Sec. 4.4), flags exactly as in Alg. 4. */
static void update_neighbors_paper_order(const data_t *D, list_t *G, int64_t *evals)
{
    list_t kept = {0, 0, 0};
    plist_t P = {0, 0, 0};
    for (int64_t u = 0; u < D->n; ++u) {
        list_sort(&G[u]);                                /* U <- sorted neighbours */
        P.len = 0;
        scan_vertex(D, &G[u], 1, &kept, &P, evals);
        G[u].len = 0;
        for (int32_t k = 0; k < kept.len; ++k) {
            entry_t x = kept.e[k];
            x.is_new = 0;                                /* kept: old */
            list_push(&G[u], x);
        }
        for (int64_t i = 0; i < P.len; ++i) {
            list_t *Lw = &G[P.p[i].target];
            if (!list_has(Lw, P.p[i].id)) {              /* an edge already present is not added again */
                entry_t x;
                x.id = P.p[i].id; x.dist = P.p[i].dist; x.is_new = 1;
                list_push(Lw, x);
            }
        }
    }
    for (int64_t u = 0; u < D->n; ++u) list_sort(&G[u]);
    free(kept.e);
    free(P.p);
}

/* ------------------------------------------------- AddReverseEdges (Alg. 5) */
static void add_reverse_edges(list_t *G, int64_t n, int32_t R)
{
    /* first loop: E <- E + reversed E, added entries flagged new */
    list_t *A = graph_alloc(n);
    for (int64_t u = 0; u < n; ++u)
        for (int32_t k = 0; k < G[u].len; ++k) {
            entry_t x;
            x.id = (int32_t)u; x.dist = G[u].e[k].dist; x.is_new = 1;
            list_push(&A[G[u].e[k].id], x);
        }
    for (int64_t v = 0; v < n; ++v) {
        for (int32_t k = 0; k < A[v].len; ++k)
            if (!list_has(&G[v], A[v].e[k].id)) list_push(&G[v], A[v].e[k]);
        free(A[v].e);
        /* second loop: keep only the R shortest edges leaving v */
        list_canonicalise(&G[v], R);
    }
    free(A);
    /* third loop: keep only the R shortest edges entering v, by (delta, source) */
    list_t *In = graph_alloc(n);
    for (int64_t u = 0; u < n; ++u)
        for (int32_t k = 0; k < G[u].len; ++k) {
            entry_t x;
            x.id = (int32_t)u; x.dist = G[u].e[k].dist; x.is_new = 0;
            list_push(&In[G[u].e[k].id], x);
        }
    for (int64_t v = 0; v < n; ++v) {
        list_sort(&In[v]);
        for (int32_t k = R; k < In[v].len; ++k) {        /* the edges beyond the R shortest */
            list_t *Lu = &G[In[v].e[k].id];
            int32_t m = 0;
            for (int32_t t = 0; t < Lu->len; ++t)
                if (Lu->e[t].id != (int32_t)v) Lu->e[m++] = Lu->e[t];
            Lu->len = m;
        }
        free(In[v].e);
    }
    free(In);
}

/* ============================================================ exported API */

int orc_random_graph(const void *X, int64_t n, int32_t d, int dtype, int32_t S, uint64_t seed,
                     int32_t W, int32_t *ids, double *dist, uint8_t *flags, int32_t *deg)
{
    if (S < 1 || S > W || (int64_t)S > n - 1) return -1;
    data_t D = {X, n, d, dtype};
    list_t *G = random_graph(&D, S, seed);
    graph_to_flat(G, n, W, ids, dist, flags, deg);
    graph_free(G, n);
    return 0;
}

int orc_random_ids(int64_t n, int64_t u, int32_t S, uint64_t seed, int32_t *out)
{
    if (S < 1 || (int64_t)S > n - 1) return -1;
    random_row(seed, n, u, S, out);
    return 0;
}

int orc_update_neighbors_sync(const void *X, int64_t n, int32_t d, int dtype, int32_t R, int32_t W,
                              int32_t *ids, double *dist, uint8_t *flags, int32_t *deg,
                              int use_flag_skip, int64_t *evals, int64_t *nprops)
{
    if (R > W) return -1;
    data_t D = {X, n, d, dtype};
    list_t *G = graph_from_flat(n, W, ids, dist, flags, deg);
    int64_t ev = 0, np = 0;
    update_neighbors_sync(&D, G, R, use_flag_skip, &ev, &np);
    graph_to_flat(G, n, W, ids, dist, flags, deg);
    graph_free(G, n);
    if (evals) *evals = ev;
    if (nprops) *nprops = np;
    return 0;
}

int orc_add_reverse_edges(int64_t n, int32_t R, int32_t W, int32_t *ids, double *dist,
                          uint8_t *flags, int32_t *deg)
{
    if (R > W) return -1;
    list_t *G = graph_from_flat(n, W, ids, dist, flags, deg);
    add_reverse_edges(G, n, R);
    graph_to_flat(G, n, W, ids, dist, flags, deg);
    graph_free(G, n);
    return 0;
}

/* Optional progress lines on stderr, one per finished round (long runs only; no effect on results). */
static int g_progress = 0;
void orc_set_progress(int on) { g_progress = on; }

/* Alg. 6 with synchronous rounds.  round_evals (optional) receives T1*T2
 * counts of the delta(v,w) evaluations Alg. 4 performs; *init_evals = n*S. */
int orc_build_sync(const void *X, int64_t n, int32_t d, int dtype, int32_t S, int32_t R,
                   int32_t T1, int32_t T2, uint64_t seed, int use_flag_skip, int32_t W,
                   int32_t *ids, double *dist, uint8_t *flags, int32_t *deg,
                   int64_t *round_evals, int64_t *round_props, int64_t *init_evals)
{
    if (S < 1 || S > R || R > W || (int64_t)S > n - 1 || T1 < 1 || T2 < 1) return -1;
    data_t D = {X, n, d, dtype};
    list_t *G = random_graph(&D, S, seed);                      /* RandomGraph, flags new */
    if (init_evals) *init_evals = n * (int64_t)S;
    for (int32_t t1 = 0; t1 < T1; ++t1) {                       /* outer loop */
        for (int32_t t2 = 0; t2 < T2; ++t2) {                   /* inner loop */
            int64_t ev = 0, np = 0;
            update_neighbors_sync(&D, G, R, use_flag_skip, &ev, &np);   /* UpdateNeighbors */
            if (round_evals) round_evals[t1 * T2 + t2] = ev;
            if (round_props) round_props[t1 * T2 + t2] = np;
            if (g_progress) {
                fprintf(stderr, "oracle: round %d of %d done, %lld evaluations\n",
                        (int)(t1 * T2 + t2 + 1), (int)(T1 * T2), (long long)ev);
                fflush(stderr);
            }
        }
        if (t1 != T1 - 1) add_reverse_edges(G, n, R);           /* unless last */
    }
    graph_to_flat(G, n, W, ids, dist, flags, deg);
    graph_free(G, n);
    return 0;
}

/* Alg. 6 with synchronous rounds whose merges cut a list to M >= R entries; only AddReverseEdges
 * bounds the degrees by R, as in the paper, where UpdateNeighbors itself never drops an edge for
 * lack of room (Sec. 5.3 reports out-degrees above R at the end).  M = R is orc_build_sync. */
int orc_build_wide(const void *X, int64_t n, int32_t d, int dtype, int32_t S, int32_t R, int32_t M,
                   int32_t T1, int32_t T2, uint64_t seed, int32_t W, int32_t *ids, double *dist,
                   uint8_t *flags, int32_t *deg, int64_t *round_evals, int64_t *round_props)
{
    if (S < 1 || S > R || R > M || M > W || (int64_t)S > n - 1 || T1 < 1 || T2 < 1) return -1;
    data_t D = {X, n, d, dtype};
    list_t *G = random_graph(&D, S, seed);
    for (int32_t t1 = 0; t1 < T1; ++t1) {
        for (int32_t t2 = 0; t2 < T2; ++t2) {
            int64_t ev = 0, np = 0;
            update_neighbors_sync(&D, G, M, 1, &ev, &np);          /* lists cut to M */
            if (round_evals) round_evals[t1 * T2 + t2] = ev;
            if (round_props) round_props[t1 * T2 + t2] = np;
        }
        if (t1 != T1 - 1) add_reverse_edges(G, n, R);               /* degrees cut to R */
    }
    graph_to_flat(G, n, W, ids, dist, flags, deg);
    graph_free(G, n);
    return 0;
}

/* One block-sequential pass on a flat snapshot. */
int orc_update_neighbors_blocks(const void *X, int64_t n, int32_t d, int dtype, int32_t R, int32_t W,
                                int64_t nblocks, int32_t *ids, double *dist, uint8_t *flags,
                                int32_t *deg, int64_t *evals, int64_t *nprops)
{
    if (R > W || nblocks < 1 || nblocks > n) return -1;
    data_t D = {X, n, d, dtype};
    list_t *G = graph_from_flat(n, W, ids, dist, flags, deg);
    int64_t ev = 0, np = 0;
    update_neighbors_blocks(&D, G, R, nblocks, &ev, &np);
    graph_to_flat(G, n, W, ids, dist, flags, deg);
    graph_free(G, n);
    if (evals) *evals = ev;
    if (nprops) *nprops = np;
    return 0;
}

/* Alg. 6 with block-sequential passes. */
int orc_build_blocks(const void *X, int64_t n, int32_t d, int dtype, int32_t S, int32_t R,
                     int32_t T1, int32_t T2, uint64_t seed, int64_t nblocks, int32_t W,
                     int32_t *ids, double *dist, uint8_t *flags, int32_t *deg,
                     int64_t *round_evals, int64_t *round_props)
{
    if (S < 1 || S > R || R > W || (int64_t)S > n - 1 || T1 < 1 || T2 < 1) return -1;
    if (nblocks < 1 || nblocks > n) return -1;
    data_t D = {X, n, d, dtype};
    list_t *G = random_graph(&D, S, seed);                      /* RandomGraph, flags new */
    for (int32_t t1 = 0; t1 < T1; ++t1) {                       /* outer loop */
        for (int32_t t2 = 0; t2 < T2; ++t2) {                   /* inner loop */
            int64_t ev = 0, np = 0;
            update_neighbors_blocks(&D, G, R, nblocks, &ev, &np);       /* UpdateNeighbors */
            if (round_evals) round_evals[t1 * T2 + t2] = ev;
            if (round_props) round_props[t1 * T2 + t2] = np;
            if (g_progress) {
                fprintf(stderr, "oracle: pass %d of %d done, %lld evaluations\n",
                        (int)(t1 * T2 + t2 + 1), (int)(T1 * T2), (long long)ev);
                fflush(stderr);
            }
        }
        if (t1 != T1 - 1) add_reverse_edges(G, n, R);           /* unless last */
    }
    graph_to_flat(G, n, W, ids, dist, flags, deg);
    graph_free(G, n);
    return 0;
}

/* Alg. 6 in the paper's own in-place order (search-quality comparison only).
 * Rows are written nearest-first and cut to W; *max_degree reports the cut-free maximum. */
int orc_build_paper_order(const void *X, int64_t n, int32_t d, int dtype, int32_t S, int32_t R,
                          int32_t T1, int32_t T2, uint64_t seed, int32_t W, int32_t *ids,
                          int32_t *deg, int64_t *total_evals, int32_t *max_degree)
{
    if (S < 1 || (int64_t)S > n - 1 || T1 < 1 || T2 < 1) return -1;
    data_t D = {X, n, d, dtype};
    list_t *G = random_graph(&D, S, seed);
    int64_t ev = 0;
    for (int32_t t1 = 0; t1 < T1; ++t1) {
        for (int32_t t2 = 0; t2 < T2; ++t2) update_neighbors_paper_order(&D, G, &ev);
        if (t1 != T1 - 1) add_reverse_edges(G, n, R);
    }
    int32_t mx = graph_to_flat(G, n, W, ids, NULL, NULL, deg);
    graph_free(G, n);
    if (total_evals) *total_evals = ev;
    if (max_degree) *max_degree = mx;
    return 0;
}

/* Alg. 3 on an explicit candidate set; returns the selected ids in order. */
int orc_rng_strategy(const void *X, int64_t n, int32_t d, int dtype, int64_t u,
                     const int32_t *cand, int32_t nc, int32_t *out, int32_t *nout)
{
    data_t D = {X, n, d, dtype};
    list_t U = {0, 0, 0};
    for (int32_t k = 0; k < nc; ++k) {
        entry_t x;
        x.id = cand[k]; x.dist = delta(&D, u, cand[k]); x.is_new = 1;
        list_push(&U, x);
    }
    list_sort(&U);                                              /* candidates, ascending */
    int32_t m = 0;                                              /* selected set, empty */
    for (int32_t i = 0; i < U.len; ++i) {                       /* for v in order */
        int f = 1;
        for (int32_t j = 0; j < m; ++j)                         /* for selected w */
            if (U.e[i].dist >= delta(&D, U.e[i].id, out[j])) { f = 0; break; }
        if (f) out[m++] = U.e[i].id;
    }
    *nout = m;
    free(U.e);
    return 0;
}

double orc_delta(const void *X, int64_t n, int32_t d, int dtype, int64_t a, int64_t b)
{
    data_t D = {X, n, d, dtype};
    return delta(&D, a, b);
}

/* Exact k nearest database vectors of each query, ties by id. */
int orc_bruteforce_knn(const void *X, int64_t n, int32_t d, int dtype, const void *Q, int64_t nq,
                       int32_t k, int32_t *out_ids)
{
    if ((int64_t)k > n) return -1;
    data_t D = {X, n, d, dtype};
    entry_t *best = (entry_t *)malloc((size_t)(k + 1) * sizeof(entry_t));
    for (int64_t q = 0; q < nq; ++q) {
        int32_t m = 0;
        const void *qv = row_ptr(&D, Q, q);
        for (int64_t i = 0; i < n; ++i) {
            entry_t x;
            x.id = (int32_t)i; x.dist = delta_vec(&D, qv, row_ptr(&D, X, i)); x.is_new = 0;
            int32_t p = m;
            while (p > 0 && entry_cmp(&x, &best[p - 1]) < 0) {
                if (p < k) best[p] = best[p - 1];
                --p;
            }
            if (p < k) { best[p] = x; if (m < k) ++m; }
        }
        for (int32_t t = 0; t < k; ++t) out_ids[q * k + t] = best[t].id;
    }
    free(best);
    return 0;
}

/* Alg. 1 with the out-degree cap K of Eq. 4.  C starts from min(L, n)
 * distinct seeded random vertices (InitializeCandidates is not specified in
 * the paper); the loop ends when C holds no unvisited point, which is when C
 * can no longer change.  Writes the k nearest members of C per query. */
int orc_search(const void *X, int64_t n, int32_t d, int dtype, const int32_t *ids,
               const int32_t *deg, int32_t W, const void *Q, int64_t nq, int32_t L, int32_t K,
               int32_t k, uint64_t seed, int32_t *out_ids, int64_t *dist_evals)
{
    if (k > L || L < 1) return -1;
    data_t D = {X, n, d, dtype};
    int32_t L0 = (int64_t)L < n ? L : (int32_t)n;
    entry_t *C = (entry_t *)malloc((size_t)(L + 1) * sizeof(entry_t)); /* is_new: 1 = unvisited */
    uint8_t *seen = (uint8_t *)malloc((size_t)n);
    int32_t *init = (int32_t *)malloc((size_t)L0 * sizeof(int32_t));
    int64_t ev = 0;
    for (int64_t q = 0; q < nq; ++q) {
        const void *qv = row_ptr(&D, Q, q);
        memset(seen, 0, (size_t)n);
        int32_t m = 0;
        /* InitializeCandidates: seeded random start set; vertex "n" is not a vertex, so nothing is skipped */
        if ((int64_t)L0 == n) for (int32_t t = 0; t < L0; ++t) init[t] = t;
        else random_row(seed, n + 1, n, L0, init) /* ids in [0,n) */;
        for (int32_t t = 0; t < L0; ++t) {
            entry_t x;
            x.id = init[t]; x.dist = delta_vec(&D, qv, row_ptr(&D, X, init[t])); x.is_new = 1;
            ++ev;
            seen[x.id] = 1;
            int32_t p = m++;
            while (p > 0 && entry_cmp(&x, &C[p - 1]) < 0) { C[p] = C[p - 1]; --p; }
            C[p] = x;
        }
        for (;;) {
            int32_t iu = -1;                                    /* nearest unvisited member of C */
            for (int32_t t = 0; t < m; ++t) if (C[t].is_new) { iu = t; break; }
            if (iu < 0) break;                                  /* none left: done */
            C[iu].is_new = 0;
            int64_t u = C[iu].id;
            int32_t du = deg[u] < K ? deg[u] : K;               /* Eq. 4: rows are nearest-first */
            for (int32_t t = 0; t < du; ++t) {                  /* its (capped) neighbours */
                int32_t v = ids[u * W + t];
                if (seen[v]) continue;                          /* evaluated before */
                seen[v] = 1;
                entry_t x;
                x.id = v; x.dist = delta_vec(&D, qv, row_ptr(&D, X, v)); x.is_new = 1;
                ++ev;
                if (m == L && entry_cmp(&x, &C[m - 1]) >= 0) continue;  /* C keeps its L nearest */
                int32_t p = m < L ? m++ : m - 1;
                while (p > 0 && entry_cmp(&x, &C[p - 1]) < 0) { C[p] = C[p - 1]; --p; }
                C[p] = x;
            }
        }
        for (int32_t t = 0; t < k; ++t) out_ids[q * k + t] = t < m ? C[t].id : -1;
        seed += GOLDEN;
    }
    free(C); free(seen); free(init);
    if (dist_evals) *dist_evals = ev;
    return 0;
}
