/*
 * GREM reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, single-threaded, deliberately slow CPU statement of the chunk-synchronous k-way
 * GREM rule (Armada paper, Sec. 4.1 "GREM: Min-Edge-Cut Partitioning", Alg. 1 and Alg. 2),
 * used only to check the GPU library and as the timed CPU baseline.  It shares no code, header,
 * table or helper with the GPU path, and the GPU path never calls it.
 *
 * What follows the paper directly:
 *   - cnt_nbrs (Alg. 2): per node, count neighbours per partition, skipping unassigned ones.
 *   - the blend of Alg. 1 (a previously assigned node averages its stored estimate with the
 *     fresh count).  est_r = (est_{r-1} + h_r)/2 is kept exactly as the integer
 *     E_r = 2^r * est_r = E_{r-1} + 2^(r-1) * h_r  (E_0 = h_0): a common positive factor per node
 *     does not change any comparison between partitions, and no rounding ever happens.
 *   - assign (Alg. 2): go where most (estimated) neighbours are unless that partition is full,
 *     otherwise the smallest partition; ties to the lowest index.
 *   - fix_sizes (Alg. 2): +1 on the new partition, -1 on the old one.
 *   - the seed (Alg. 1, first chunk): nodes that arrive with a label keep it at their first
 *     visit and only record their estimate.
 *
 * Readings where the paper is silent or where the streaming model is restated (all listed in
 * the design notes of this repository):
 *   - the stream is a CSR: a chunk is `chunk` consecutive vertex rows, the row owner is the node
 *     that is (re)evaluated, from its full row; a node is visited once per pass and passes
 *     1..R are the "reappearances" of Sec. 4.1;
 *   - chunk-synchronous: every decision of a chunk reads the labels and sizes as they were when
 *     the chunk started; moves are then admitted in ascending vertex id while the target has
 *     room, rejected refined nodes stay, rejected new nodes go one by one to the currently
 *     smallest partition (the paper's own "partition is full" fallback);
 *   - k-way directly: candidates are the partitions with room, ordered by (estimate desc,
 *     size asc, id asc); at k=2 this is exactly `assign`;
 *   - a node being re-assigned is first taken out of its partition's size (fix_sizes' decrement
 *     evaluated before assign), so a node is never evicted merely because it fills its own part.
 *
 * Pins (tests/, CPU only): brute-force cut and balance on tiny graphs; equality with an
 * independent sequential k=2 procedure at chunk=1; closed forms (chunk >= n, edgeless graphs,
 * blend weights); invariants after every chunk; seeded planted-partition recovery; refinement
 * not increasing the cut on the test graphs; permutation and padding symmetries.
 * Labels on graphs outside those pins (e.g. R-MAT at large k) are "parity unpinned" beyond the
 * invariants.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define GREM_ORACLE_OK 0
#define GREM_ORACLE_ERR_ARG (-1)
#define GREM_ORACLE_ERR_NOMEM (-2)
#define GREM_ORACLE_ERR_RANGE (-3)
#define GREM_ORACLE_ERR_SEED (-4)
#define GREM_ORACLE_ERR_INTERNAL (-5)

typedef struct grem_oracle_state {
    const int64_t *rowptr;
    const int32_t *colidx;
    int64_t n;
    int32_t k;
    int64_t P;
    int64_t chunk;
    int32_t R;
    int32_t pass;      /* pass of the next chunk step */
    int64_t next_chunk; /* chunk index of the next chunk step */
    int64_t nchunks;
    int32_t *L;   /* n labels, -1 = unassigned */
    int64_t *S;   /* k sizes */
    uint32_t *E;  /* n*k scaled estimates */
    /* per-chunk temporaries */
    int32_t *prop;     /* chunk proposals */
    int64_t *Sh;       /* k snapshot sizes */
    int64_t *seen;     /* k */
    int64_t *h;        /* k */
    int64_t *overflow; /* chunk */
    int internal_error;
} grem_oracle_state;

/* Capacity P of one partition (Sec. 4.1: balanced parts of ceil(V/p) nodes, Alg. 1 input P),
 * widened by the caller's slack. */
int64_t grem_oracle_capacity(int64_t n, int32_t k, double balance_slack)
{
    if (n < 1 || k < 1) return -1;
    int64_t base = (n + k - 1) / k;
    double prod = (double)n * balance_slack;
    double quot = prod / (double)k;
    int64_t slack_cap = (int64_t)ceil(quot);
    return base > slack_cap ? base : slack_cap;
}

void grem_oracle_destroy(grem_oracle_state *st)
{
    if (!st) return;
    free(st->L); free(st->S); free(st->E); free(st->prop); free(st->Sh);
    free(st->seen); free(st->h); free(st->overflow);
    free(st);
}

/* Creates the state of Alg. 1 before the first chunk: parts = seed or -1, sizes = counts of the
 * seed, nbr_counts = 0.  The CSR arrays are borrowed and must outlive the state. */
grem_oracle_state *grem_oracle_create(const int64_t *rowptr, const int32_t *colidx, int64_t n,
                                      int32_t k, double balance_slack, int64_t chunk,
                                      int32_t refine_passes, const int32_t *seed_labels,
                                      int *status)
{
    int dummy;
    if (!status) status = &dummy;
    *status = GREM_ORACLE_ERR_ARG;
    if (!rowptr || !colidx || n < 1 || n > INT32_MAX || k < 1 || chunk < 1 || refine_passes < 0 ||
        !(balance_slack >= 1.0))
        return NULL;
    /* E must hold deg * 2^R */
    int64_t maxdeg = 0;
    for (int64_t v = 0; v < n; ++v) {
        int64_t d = rowptr[v + 1] - rowptr[v];
        if (d < 0) return NULL;
        if (d > maxdeg) maxdeg = d;
    }
    if (refine_passes >= 32 || (maxdeg << refine_passes) >= ((int64_t)1 << 32)) {
        *status = GREM_ORACLE_ERR_RANGE;
        return NULL;
    }
    grem_oracle_state *st = (grem_oracle_state *)calloc(1, sizeof(*st));
    if (!st) { *status = GREM_ORACLE_ERR_NOMEM; return NULL; }
    st->rowptr = rowptr; st->colidx = colidx; st->n = n; st->k = k;
    st->P = grem_oracle_capacity(n, k, balance_slack);
    /* a chunk at least as long as the graph is the whole graph (and n + chunk cannot overflow) */
    int64_t cl = chunk < n ? chunk : n;
    st->chunk = cl; st->R = refine_passes;
    st->nchunks = (n + cl - 1) / cl;
    st->L = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    st->S = (int64_t *)calloc((size_t)k, sizeof(int64_t));
    st->E = (uint32_t *)calloc((size_t)n * (size_t)k, sizeof(uint32_t));
    st->prop = (int32_t *)malloc(sizeof(int32_t) * (size_t)cl);
    st->Sh = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    st->seen = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    st->h = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    st->overflow = (int64_t *)malloc(sizeof(int64_t) * (size_t)cl);
    if (!st->L || !st->S || !st->E || !st->prop || !st->Sh || !st->seen || !st->h || !st->overflow) {
        grem_oracle_destroy(st);
        *status = GREM_ORACLE_ERR_NOMEM;
        return NULL;
    }
    for (int64_t v = 0; v < n; ++v) {
        int32_t s = seed_labels ? seed_labels[v] : -1;
        if (s < -1 || s >= k) { grem_oracle_destroy(st); *status = GREM_ORACLE_ERR_SEED; return NULL; }
        st->L[v] = s;
        if (s >= 0) st->S[s] += 1;
    }
    for (int32_t j = 0; j < k; ++j)
        if (st->S[j] > st->P) { grem_oracle_destroy(st); *status = GREM_ORACLE_ERR_SEED; return NULL; }
    *status = GREM_ORACLE_OK;
    return st;
}

/* One chunk of Alg. 1's loop, chunk-synchronous.  Returns 1 if a chunk was processed, 0 if the
 * run is complete, <0 on a broken guarantee. */
int grem_oracle_step(grem_oracle_state *st)
{
    if (!st) return GREM_ORACLE_ERR_ARG;
    if (st->pass > st->R) return 0;
    const int64_t n = st->n, P = st->P;
    const int32_t k = st->k, r = st->pass;
    const int64_t lo = st->next_chunk * st->chunk;
    const int64_t hi = (lo + st->chunk < n) ? lo + st->chunk : n;
    int32_t *L = st->L; int64_t *S = st->S;

    /* Snapshot.  Labels of the chunk's own vertices are only overwritten in phase 2, and phase 1
     * reads labels only; so reading L during phase 1 IS reading the snapshot.  Sizes are copied. */
    for (int32_t j = 0; j < k; ++j) st->Sh[j] = S[j];

    /* Phase 1: count (cnt_nbrs), blend (Alg. 1), propose (assign). */
    for (int64_t v = lo; v < hi; ++v) {
        for (int32_t j = 0; j < k; ++j) st->h[j] = 0;
        for (int64_t e = st->rowptr[v]; e < st->rowptr[v + 1]; ++e) {
            int32_t u = st->colidx[e];
            int32_t lu = L[u];
            if (lu != -1) st->h[lu] += 1;
        }
        uint32_t *Ev = st->E + (size_t)v * (size_t)k;
        for (int32_t j = 0; j < k; ++j) {
            if (r == 0) Ev[j] = (uint32_t)st->h[j];
            else Ev[j] = Ev[j] + (uint32_t)(st->h[j] << (r - 1));
        }
        int32_t old = L[v];
        if (r == 0 && old >= 0) {         /* seeded vertex: keep the seed, estimate recorded */
            st->prop[v - lo] = old;
            continue;
        }
        int32_t best = -1; uint32_t bestE = 0; int64_t bestS = 0;
        for (int32_t j = 0; j < k; ++j) {
            int64_t Sj = st->Sh[j] - (j == old ? 1 : 0);   /* v taken out of its own part */
            if (!(Sj < P)) continue;                        /* full */
            if (best < 0 || Ev[j] > bestE || (Ev[j] == bestE && Sj < bestS)) {
                best = j; bestE = Ev[j]; bestS = Sj;
            }
        }
        if (best < 0) { st->internal_error = 1; return GREM_ORACLE_ERR_INTERNAL; }
        st->prop[v - lo] = best;
    }

    /* Phase 2: admission in ascending id (fix_sizes for the admitted). */
    int64_t nover = 0;
    for (int32_t j = 0; j < k; ++j) st->seen[j] = 0;
    for (int64_t v = lo; v < hi; ++v) {
        int32_t t = st->prop[v - lo];
        int32_t old = L[v];                     /* still the snapshot value for v itself */
        if (t == old) continue;
        if (st->seen[t] < P - st->Sh[t]) {
            L[v] = t; S[t] += 1;
            if (old >= 0) S[old] -= 1;
        } else if (old < 0) {
            st->overflow[nover++] = v;
        }
        st->seen[t] += 1;
    }

    /* Phase 3: rejected new vertices, one by one, to the smallest partition (lowest id). */
    for (int64_t i = 0; i < nover; ++i) {
        int32_t best = 0;
        for (int32_t j = 1; j < k; ++j) if (S[j] < S[best]) best = j;
        if (!(S[best] < P)) { st->internal_error = 1; return GREM_ORACLE_ERR_INTERNAL; }
        L[st->overflow[i]] = best; S[best] += 1;
    }

    /* Guarantees of the rule. */
    for (int32_t j = 0; j < k; ++j)
        if (S[j] > P || S[j] < 0) { st->internal_error = 1; return GREM_ORACLE_ERR_INTERNAL; }
    for (int64_t v = lo; v < hi; ++v)
        if (L[v] < 0 || L[v] >= k) { st->internal_error = 1; return GREM_ORACLE_ERR_INTERNAL; }

    st->next_chunk += 1;
    if (st->next_chunk == st->nchunks) { st->next_chunk = 0; st->pass += 1; }
    return 1;
}

int64_t grem_oracle_get_capacity(const grem_oracle_state *st) { return st->P; }
int32_t grem_oracle_get_pass(const grem_oracle_state *st) { return st->pass; }
int64_t grem_oracle_get_next_chunk(const grem_oracle_state *st) { return st->next_chunk; }
const int32_t *grem_oracle_labels(const grem_oracle_state *st) { return st->L; }
const int64_t *grem_oracle_sizes(const grem_oracle_state *st) { return st->S; }
const uint32_t *grem_oracle_estimates(const grem_oracle_state *st) { return st->E; }

/* Whole run: pass 0 plus `refine_passes` refinement passes.  sizes_out (k) and estimates_out
 * (n*k) may be NULL. */
int grem_oracle_partition_seeded(const int64_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                                 double balance_slack, int64_t chunk, int32_t refine_passes,
                                 const int32_t *seed_labels, int32_t *labels_out,
                                 int64_t *sizes_out, uint32_t *estimates_out)
{
    if (!labels_out) return GREM_ORACLE_ERR_ARG;
    int status;
    grem_oracle_state *st = grem_oracle_create(rowptr, colidx, n, k, balance_slack, chunk,
                                               refine_passes, seed_labels, &status);
    if (!st) return status;
    int rc;
    while ((rc = grem_oracle_step(st)) == 1) { }
    if (rc < 0) { grem_oracle_destroy(st); return rc; }
    /* S must equal the label counts */
    int64_t *cnt = (int64_t *)calloc((size_t)k, sizeof(int64_t));
    if (!cnt) { grem_oracle_destroy(st); return GREM_ORACLE_ERR_NOMEM; }
    for (int64_t v = 0; v < n; ++v) cnt[st->L[v]] += 1;
    for (int32_t j = 0; j < k; ++j)
        if (cnt[j] != st->S[j]) { free(cnt); grem_oracle_destroy(st); return GREM_ORACLE_ERR_INTERNAL; }
    free(cnt);
    memcpy(labels_out, st->L, sizeof(int32_t) * (size_t)n);
    if (sizes_out) memcpy(sizes_out, st->S, sizeof(int64_t) * (size_t)k);
    if (estimates_out) memcpy(estimates_out, st->E, sizeof(uint32_t) * (size_t)n * (size_t)k);
    grem_oracle_destroy(st);
    return GREM_ORACLE_OK;
}

int grem_oracle_partition(const int64_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                          double balance_slack, int64_t chunk, int32_t refine_passes,
                          int32_t *labels_out)
{
    return grem_oracle_partition_seeded(rowptr, colidx, n, k, balance_slack, chunk, refine_passes,
                                        NULL, labels_out, NULL, NULL);
}

/* Number of CSR entries (v,u) whose endpoints carry different labels (Sec. 1: cut edges are
 * those with endpoints in different partitions).  For a symmetric loop-free CSR the undirected
 * cut is half of it. */
int64_t grem_oracle_edge_cut(const int64_t *rowptr, const int32_t *colidx, int64_t n,
                             const int32_t *labels)
{
    if (!rowptr || !colidx || !labels || n < 0) return -1;
    int64_t cut = 0;
    for (int64_t v = 0; v < n; ++v)
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e)
            if (labels[colidx[e]] != labels[v]) cut += 1;
    return cut;
}
