/*
 * GREM over a stream of edge chunks, two partitions -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, single-threaded CPU statement of Alg. 1 "GREM Bipartite Graph Partitioning" with the
 * helpers of Alg. 2 (Armada paper, Sec. 4.1) in the stream model the paper itself uses: the input
 * is an edge list in random order, a chunk is `c_size` consecutive edges, the chunk's nodes are
 * the distinct endpoints of its edges, and each of them is (re)evaluated from the chunk's edges
 * only.  It is used to check the GPU library and as a timed CPU baseline; it shares no code,
 * header, table or helper with the GPU path, and the GPU path never calls it.
 *
 * What follows the paper directly:
 *   - cnt_nbrs (Alg. 2): for a node, every chunk edge that touches it adds one to the count of the
 *     partition of the edge's other end (the node itself for a loop); unassigned ends add nothing.
 *   - first chunk (Alg. 1): its nodes take the labels of `seed_algo`, here handed in as data;
 *     sizes are the label counts; the stored estimates are cnt_nbrs under those labels.
 *   - blend (Alg. 1): a node that already has a label replaces the fresh counts by the mean of
 *     the stored estimate and the fresh counts; the result is stored whether or not the node moves.
 *   - assign, fix_sizes (Alg. 2).
 *   - fixed-greedy mode (Sec. 4.1, the algorithm "as described so far"): a node is decided once,
 *     when first seen, and never looked at again.
 *
 * Readings where the paper is silent or sequential (listed in the repository's design notes):
 *   - the chunk's nodes are taken in ascending id;
 *   - chunk-synchronous: every decision of a chunk reads labels and sizes as they were when the
 *     chunk started; moves are admitted in ascending id while fewer than P - sizes[t] earlier
 *     nodes of the chunk asked for t; a rejected node that had a label keeps it; rejected new
 *     nodes are then placed one by one, ascending id, in the currently smaller partition (0 on a
 *     tie) -- the same reading as the row-chunk oracle in this directory;
 *   - a re-evaluated node is taken out of its partition's size before `assign` looks at the sizes;
 *   - arg_min ties go to partition 0;
 *   - estimates are IEEE doubles; the mean is (old + fresh) * 0.5, one rounding of the sum at most
 *     (the halving is exact short of underflow); the GPU path does the same two operations;
 *   - nodes that never occur in an edge stay unassigned (-1); P is the caller's (Alg. 1 input),
 *     2P >= n is required so that a new node always finds room.
 *
 * Pins (tests/, CPU only): a literal node-at-a-time transcription of Alg. 1/2 with exact rationals
 * on instances where it detects no dependence inside any chunk; counts against dense incidence
 * algebra; the closed-form chunk weights of Sec. 4.1; a hand-worked example; invariants; seeded
 * planted-partition recovery and the refined-below-fixed cut ordering of Sec. 4.2.
 * Labels on graphs outside those pins (e.g. power-law streams with many chunks) are "parity
 * unpinned" beyond the invariants.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GREM_EDGE_OK 0
#define GREM_EDGE_ERR_ARG (-1)
#define GREM_EDGE_ERR_NOMEM (-2)
#define GREM_EDGE_ERR_SEED (-4)
#define GREM_EDGE_ERR_INTERNAL (-5)

#define GREM_EDGE_REFINE 0
#define GREM_EDGE_FIXED 1

typedef struct grem_edge_oracle_state {
    const int32_t *src, *dst;
    int64_t m, n, c_size, P;
    const int32_t *seed_parts;
    int32_t mode;
    int64_t next_chunk, nchunks;
    int32_t *parts;        /* n, -1 = unassigned */
    int64_t sizes[2];
    double *nbr_counts;    /* n x 2 */
    /* per-chunk temporaries, kept so that tests can look at the last chunk */
    int32_t *c_nodes;      /* distinct endpoints of the chunk, ascending */
    int64_t c_count;
    int64_t *fresh;        /* c_count x 2: cnt_nbrs of the last chunk */
    int32_t *prop;         /* c_count proposals, -2 = node not evaluated (fixed-greedy mode) */
    uint8_t *mark;         /* n */
    int64_t *first;        /* n+1: start of a node's list of incident chunk edges */
    int64_t *incident;     /* 2*c_size edge indices grouped by node */
    int64_t *overflow;
} grem_edge_oracle_state;

void grem_edge_oracle_destroy(grem_edge_oracle_state *st)
{
    if (!st) return;
    free(st->parts); free(st->nbr_counts); free(st->c_nodes); free(st->fresh); free(st->prop);
    free(st->mark); free(st->first); free(st->incident); free(st->overflow);
    free(st);
}

grem_edge_oracle_state *grem_edge_oracle_create(const int32_t *src, const int32_t *dst, int64_t m,
                                                int64_t n, int64_t c_size, int64_t P,
                                                const int32_t *seed_parts, int32_t mode, int *status)
{
    int dummy;
    if (!status) status = &dummy;
    *status = GREM_EDGE_ERR_ARG;
    if (!src || !dst || !seed_parts || m < 1 || n < 1 || n > INT32_MAX || c_size < 1 || P < 1 ||
        2 * P < n || (mode != GREM_EDGE_REFINE && mode != GREM_EDGE_FIXED))
        return NULL;
    for (int64_t e = 0; e < m; ++e)
        if (src[e] < 0 || src[e] >= n || dst[e] < 0 || dst[e] >= n) return NULL;
    grem_edge_oracle_state *st = (grem_edge_oracle_state *)calloc(1, sizeof(*st));
    if (!st) { *status = GREM_EDGE_ERR_NOMEM; return NULL; }
    st->src = src; st->dst = dst; st->m = m; st->n = n; st->c_size = c_size; st->P = P;
    st->seed_parts = seed_parts; st->mode = mode;
    st->nchunks = (m + c_size - 1) / c_size;
    int64_t ce = c_size < m ? c_size : m;
    int64_t cn = 2 * ce < n ? 2 * ce : n;
    st->parts = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    st->nbr_counts = (double *)calloc((size_t)n * 2, sizeof(double));
    st->c_nodes = (int32_t *)malloc(sizeof(int32_t) * (size_t)cn);
    st->fresh = (int64_t *)malloc(sizeof(int64_t) * (size_t)cn * 2);
    st->prop = (int32_t *)malloc(sizeof(int32_t) * (size_t)cn);
    st->mark = (uint8_t *)calloc((size_t)n, 1);
    st->first = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
    st->incident = (int64_t *)malloc(sizeof(int64_t) * (size_t)ce * 2);
    st->overflow = (int64_t *)malloc(sizeof(int64_t) * (size_t)cn);
    if (!st->parts || !st->nbr_counts || !st->c_nodes || !st->fresh || !st->prop || !st->mark ||
        !st->first || !st->incident || !st->overflow) {
        grem_edge_oracle_destroy(st);
        *status = GREM_EDGE_ERR_NOMEM;
        return NULL;
    }
    for (int64_t v = 0; v < n; ++v) st->parts[v] = -1;
    *status = GREM_EDGE_OK;
    return st;
}

/* assign of Alg. 2 on sizes from which the node itself has already been taken out. */
static int32_t assign(double nbrs0, double nbrs1, const int64_t sizes[2], int64_t P)
{
    if (nbrs0 < nbrs1 && sizes[1] < P) return 1;
    if (nbrs1 < nbrs0 && sizes[0] < P) return 0;
    return sizes[1] < sizes[0] ? 1 : 0;
}

/* One chunk of Alg. 1's loop.  Returns 1 if a chunk was processed, 0 when the stream is used up,
 * <0 on a bad seed or a broken guarantee. */
int grem_edge_oracle_step(grem_edge_oracle_state *st)
{
    if (!st) return GREM_EDGE_ERR_ARG;
    if (st->next_chunk >= st->nchunks) return 0;
    const int64_t lo = st->next_chunk * st->c_size;
    const int64_t hi = lo + st->c_size < st->m ? lo + st->c_size : st->m;
    const int64_t P = st->P;
    int32_t *parts = st->parts;

    /* c_nodes: the distinct endpoints, ascending (a sweep over the mark array keeps the order). */
    int64_t lowest = st->n, highest = -1;
    for (int64_t e = lo; e < hi; ++e) {
        int32_t a = st->src[e], b = st->dst[e];
        st->mark[a] = 1; st->mark[b] = 1;
        if (a < lowest) lowest = a;
        if (b < lowest) lowest = b;
        if (a > highest) highest = a;
        if (b > highest) highest = b;
    }
    int64_t cc = 0;
    for (int64_t v = lowest; v <= highest; ++v)
        if (st->mark[v]) { st->c_nodes[cc++] = (int32_t)v; st->mark[v] = 0; }
    st->c_count = cc;

    /* The chunk's edges grouped by the node they touch, in stream order (a loop is listed once). */
    for (int64_t i = 0; i < cc; ++i) st->first[st->c_nodes[i]] = 0;
    for (int64_t e = lo; e < hi; ++e) {
        st->first[st->src[e]] += 1;
        if (st->dst[e] != st->src[e]) st->first[st->dst[e]] += 1;
    }
    {
        int64_t run = 0;
        for (int64_t i = 0; i < cc; ++i) {
            int32_t v = st->c_nodes[i];
            int64_t d = st->first[v];
            st->first[v] = run;        /* becomes the write cursor, restored below */
            run += d;
        }
        for (int64_t e = lo; e < hi; ++e) {
            st->incident[st->first[st->src[e]]++] = e;
            if (st->dst[e] != st->src[e]) st->incident[st->first[st->dst[e]]++] = e;
        }
        /* first[v] now is the END of v's list; starts are the previous node's end */
    }

    const int is_first = (st->next_chunk == 0);
    if (is_first) {
        /* seed_algo's labels for the first chunk's nodes, and their sizes */
        for (int64_t i = 0; i < cc; ++i) {
            int32_t v = st->c_nodes[i];
            int32_t s = st->seed_parts[v];
            if (s != 0 && s != 1) return GREM_EDGE_ERR_SEED;
            parts[v] = s;
            st->sizes[s] += 1;
        }
        if (st->sizes[0] > P || st->sizes[1] > P) return GREM_EDGE_ERR_SEED;
    }

    /* Phase 1 (reads parts and sizes only): cnt_nbrs, blend, assign. */
    const int64_t snap[2] = { st->sizes[0], st->sizes[1] };
    int64_t begin = 0;
    for (int64_t i = 0; i < cc; ++i) {
        const int32_t n_ = st->c_nodes[i];
        const int64_t end = st->first[n_];
        int64_t cnt[2] = { 0, 0 };
        for (int64_t q = begin; q < end; ++q) {
            const int64_t e = st->incident[q];
            const int32_t nbr = (st->dst[e] == n_) ? st->src[e] : st->dst[e];
            if (parts[nbr] != -1) cnt[parts[nbr]] += 1;
        }
        begin = end;
        st->fresh[2 * i] = cnt[0]; st->fresh[2 * i + 1] = cnt[1];
        const int32_t old_part = parts[n_];
        double nbrs0 = (double)cnt[0], nbrs1 = (double)cnt[1];
        if (is_first) {
            st->nbr_counts[2 * (size_t)n_] = nbrs0; st->nbr_counts[2 * (size_t)n_ + 1] = nbrs1;
            st->prop[i] = -2;
            continue;
        }
        if (old_part != -1) {
            if (st->mode == GREM_EDGE_FIXED) { st->prop[i] = -2; continue; }
            nbrs0 = (st->nbr_counts[2 * (size_t)n_] + nbrs0) * 0.5;
            nbrs1 = (st->nbr_counts[2 * (size_t)n_ + 1] + nbrs1) * 0.5;
        }
        int64_t without[2] = { snap[0] - (old_part == 0), snap[1] - (old_part == 1) };
        st->prop[i] = assign(nbrs0, nbrs1, without, P);
        st->nbr_counts[2 * (size_t)n_] = nbrs0; st->nbr_counts[2 * (size_t)n_ + 1] = nbrs1;
    }

    /* Phase 2: admission in ascending id (fix_sizes for the admitted). */
    int64_t asked[2] = { 0, 0 }, nover = 0;
    for (int64_t i = 0; i < cc; ++i) {
        const int32_t t = st->prop[i];
        if (t == -2) continue;
        const int32_t n_ = st->c_nodes[i];
        const int32_t old_part = parts[n_];
        if (t == old_part) continue;
        if (asked[t] < P - snap[t]) {
            parts[n_] = t;
            st->sizes[t] += 1;
            if (old_part != -1) st->sizes[old_part] -= 1;
        } else if (old_part == -1) {
            st->overflow[nover++] = n_;
        }
        asked[t] += 1;
    }

    /* Phase 3: rejected new nodes, one by one, to the smaller partition. */
    for (int64_t i = 0; i < nover; ++i) {
        const int32_t t = st->sizes[1] < st->sizes[0] ? 1 : 0;
        if (!(st->sizes[t] < P)) return GREM_EDGE_ERR_INTERNAL;
        parts[st->overflow[i]] = t;
        st->sizes[t] += 1;
    }

    if (st->sizes[0] > P || st->sizes[1] > P || st->sizes[0] < 0 || st->sizes[1] < 0)
        return GREM_EDGE_ERR_INTERNAL;
    for (int64_t i = 0; i < cc; ++i)
        if (parts[st->c_nodes[i]] != 0 && parts[st->c_nodes[i]] != 1) return GREM_EDGE_ERR_INTERNAL;
    st->next_chunk += 1;
    return 1;
}

const int32_t *grem_edge_oracle_parts(const grem_edge_oracle_state *st) { return st->parts; }
const int64_t *grem_edge_oracle_sizes(const grem_edge_oracle_state *st) { return st->sizes; }
const double *grem_edge_oracle_nbr_counts(const grem_edge_oracle_state *st) { return st->nbr_counts; }
int64_t grem_edge_oracle_next_chunk(const grem_edge_oracle_state *st) { return st->next_chunk; }
int64_t grem_edge_oracle_chunk_count(const grem_edge_oracle_state *st) { return st->nchunks; }
/* The last processed chunk: its nodes, their fresh counts (cnt_nbrs) and proposals. */
int64_t grem_edge_oracle_last_nodes(const grem_edge_oracle_state *st, const int32_t **nodes,
                                    const int64_t **fresh, const int32_t **prop)
{
    if (nodes) *nodes = st->c_nodes;
    if (fresh) *fresh = st->fresh;
    if (prop) *prop = st->prop;
    return st->c_count;
}

/* Whole run.  parts_out: n, sizes_out: 2 (may be NULL), nbr_counts_out: 2n (may be NULL). */
int grem_edge_oracle_run(const int32_t *src, const int32_t *dst, int64_t m, int64_t n,
                         int64_t c_size, int64_t P, const int32_t *seed_parts, int32_t mode,
                         int32_t *parts_out, int64_t *sizes_out, double *nbr_counts_out)
{
    int status;
    grem_edge_oracle_state *st = grem_edge_oracle_create(src, dst, m, n, c_size, P, seed_parts, mode, &status);
    if (!st) return status;
    int rc;
    while ((rc = grem_edge_oracle_step(st)) == 1) { }
    if (rc == 0) {
        memcpy(parts_out, st->parts, sizeof(int32_t) * (size_t)n);
        if (sizes_out) { sizes_out[0] = st->sizes[0]; sizes_out[1] = st->sizes[1]; }
        if (nbr_counts_out) memcpy(nbr_counts_out, st->nbr_counts, sizeof(double) * (size_t)n * 2);
    }
    grem_edge_oracle_destroy(st);
    return rc;
}

/* Number of listed edges whose two ends carry different labels (Sec. 1). */
int64_t grem_edge_oracle_cut(const int32_t *src, const int32_t *dst, int64_t m, const int32_t *parts)
{
    int64_t cut = 0;
    for (int64_t e = 0; e < m; ++e)
        if (parts[src[e]] != parts[dst[e]]) cut += 1;
    return cut;
}
