/*
 * grem.h -- C ABI of the MI355X (gfx950) GREM partitioner.
 *
 * GREM is the streaming greedy min-edge-cut partitioner with continuous refinement of the Armada
 * paper (Sec. 4.1, Alg. 1 "GREM Bipartite Graph Partitioning" and Alg. 2 "GREM Helper
 * Functions").  This library computes its chunk-synchronous, direct k-way form on one GPU:
 *
 *   P  = max(ceil(n/k), ceil(n*balance_slack/k))          capacity of a partition (Alg. 1 input P)
 *   L[v] = seed or -1,  S[j] = #{v: L[v]=j},  E[v][j] = 0
 *   for pass r = 0 .. refine_passes, for each chunk C of `chunk` consecutive vertex rows:
 *     (all reads below see L and S as they were when the chunk started)
 *     h[v][j]  = #{entries u of row v with L[u] = j}       (cnt_nbrs, Alg. 2; unassigned skipped)
 *     E[v][j]  = h                       in pass 0
 *              = E[v][j] + h * 2^(r-1)   in pass r >= 1    (the running average of Alg. 1 kept as
 *                                                           the exact integer 2^r * average)
 *     proposal = v's seed if r = 0 and v is seeded, else the partition with room
 *                (S'[j] < P, S' = S without v itself) that maximises (E[v][j], -S'[j], -j)
 *                                                          (assign, Alg. 2)
 *     admission in ascending v: a vertex whose proposal t differs from its label moves if fewer
 *     than P - S[t] earlier vertices of the chunk proposed t; a rejected refined vertex keeps its
 *     label; rejected new vertices are then placed one by one, in ascending v, in the currently
 *     smallest partition (lowest id on ties)            (fix_sizes and the arg_min fallback, Alg. 2)
 *
 * The result is a pure function of the arguments: the same bytes on every run.
 *
 * Conventions for every entry point
 *   - All array pointers are DEVICE pointers owned by the caller.  The library neither frees nor
 *     keeps them once the work it enqueued has completed.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Argument checks and
 *     one small validation read-back happen before the call returns; the passes themselves are
 *     only enqueued on `stream` -- synchronise the stream before reading the outputs.
 *   - Return value: GREM_OK or a negative GREM_ERR_* code; nothing throws or aborts.  On error the
 *     outputs are unspecified.
 *   - The CSR must be well formed (rowptr non-decreasing, rowptr[0] = 0, 0 <= colidx < n); this is
 *     the caller's contract and is not checked.  Entries are counted exactly as stored (loops and
 *     duplicates included); nothing requires symmetry.
 *   - Concurrency: entry points may be called from several host threads and on several streams at
 *     once; a call keeps its state in memory of its own (allocated stream-ordered on `stream` and
 *     released when its work is done).  The one exception is the optional caller-owned workspace
 *     (grem_set_workspace): calls that use it share it and must not overlap in time.
 *   - Host synchronisation: a call reads a few counters back before it enqueues its passes (the
 *     graph's largest degree and number of entries, the sizes of the re-laid-out copy, the seed's
 *     validity): one read-back on the plain route, two or three on the two-phase route;
 *     grem_partition_planned without a seed reads nothing back.
 */
#ifndef GREM_H
#define GREM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GREM_OK 0
#define GREM_ERR_ARG (-1)    /* null pointer, n < 1, n > 2^31-1, k < 1, k > GREM_MAX_K, chunk < 1,
                                refine_passes < 0, balance_slack < 1 or NaN */
#define GREM_ERR_NOMEM (-2)  /* workspace allocation failed or the given workspace is too small */
#define GREM_ERR_HIP (-3)    /* a HIP runtime call failed */
#define GREM_ERR_RANGE (-4)  /* max_degree * 2^refine_passes >= 2^32 (E would overflow), or a tile
                                of rows holds 2^32 or more entries */
#define GREM_ERR_SEED (-5)   /* a seed label outside {-1} u [0,k), or a seeded partition above P */
#define GREM_ERR_LIMIT (-6)  /* the input is larger than a fixed-size buffer of the entry point allows */

#define GREM_MAX_K 4096

/* Histogram placement for the per-vertex partition counts (Alg. 2, cnt_nbrs): the route a
 * partition call takes.  All routes give the same result, bit for bit. */
#define GREM_HIST_AUTO 0     /* LDS when a tile of rows fits the LDS budget (k <= 1024), else global */
#define GREM_HIST_LDS 1      /* force LDS (error GREM_ERR_ARG if k > 1024) */
#define GREM_HIST_GLOBAL 2   /* force accumulation straight into E's rows in global memory */
#define GREM_HIST_SWEEP 3    /* force the two-phase path: a re-laid-out copy of the entries; after a
                                chunk is relabelled its labels are looked up, from LDS, for every
                                entry that refers to them, and the rows' workgroups later count
                                the stored results into LDS histograms (GREM_ERR_ARG unless
                                k <= 32 and the plan fits its limits).  AUTO takes it for k <= 32
                                when the label table is larger than L2 and chunks are large. */

/* Sec. 4.1 (Alg. 1 with all nodes unassigned at the start).  rowptr: n+1 entries; colidx:
 * rowptr[n] entries; labels_out: n entries, each in [0,k) on completion. */
int grem_partition(const int64_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                   double balance_slack, int64_t chunk, int32_t refine_passes,
                   int32_t *labels_out, void *stream);

/* Same, with the output of Alg. 1's `seed_algo` supplied as data: seed_labels has n entries, -1 =
 * unassigned; a seeded vertex keeps its label at its pass-0 visit and only records its estimate
 * (first-chunk treatment in Alg. 1).  seed_labels may be NULL (= grem_partition) and may alias
 * labels_out. */
int grem_partition_seeded(const int64_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                          double balance_slack, int64_t chunk, int32_t refine_passes,
                          const int32_t *seed_labels, int32_t *labels_out, void *stream);

/* The same two calls for a CSR whose rowptr is int32 (fewer than 2^31 entries). */
int grem_partition_r32(const int32_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                       double balance_slack, int64_t chunk, int32_t refine_passes,
                       int32_t *labels_out, void *stream);
int grem_partition_seeded_r32(const int32_t *rowptr, const int32_t *colidx, int64_t n, int32_t k,
                              double balance_slack, int64_t chunk, int32_t refine_passes,
                              const int32_t *seed_labels, int32_t *labels_out, void *stream);

/* The same run, also returning the rest of Alg. 1's state.  rowptr_bits is 32 or 64.
 * sizes_out: k int64 partition sizes (Alg. 1 `sizes`), may be NULL.  estimates_out: n*k uint32,
 * row-major, the scaled running estimates E (Alg. 1 `nbr_counts` times 2^refine_passes), may be
 * NULL; when given it is used as E's storage and the workspace shrinks by n*k*4 bytes. */
int grem_partition_state(const void *rowptr, int32_t rowptr_bits, const int32_t *colidx, int64_t n,
                         int32_t k, double balance_slack, int64_t chunk, int32_t refine_passes,
                         const int32_t *seed_labels, int32_t *labels_out, int64_t *sizes_out,
                         uint32_t *estimates_out, void *stream);

/* Per-call options: how the run is carried out, never what it computes.  All zero (or a NULL
 * pointer where one is taken) = the defaults. */
typedef struct grem_options {
    int32_t histogram_mode;   /* GREM_HIST_*; AUTO picks by k, graph size and chunk size */
    int32_t col_bits;         /* two-phase route: log2 of the vertices per column block; 0 = automatic
                                 (17, i.e. 64 KB of LDS with two labels per byte, or less when chunks are
                                 shorter), else 4..18.  Small values only make sense on small graphs */
    int32_t hub_degree;       /* two-phase route: rows of at least this many entries are "hubs", whose
                                 entries are spread evenly over the chunk's workgroups; 0 = default
                                 (8192), else 1..65535.  The other rows' estimates are kept in 16 bits
                                 while (hub_degree - 1) * 2^refine_passes < 65536 (the default: up to 3
                                 refinement passes), else in 32 */
    int32_t long_row_degree;  /* plain route: a tile of rows is scored by one workgroup; rows of at least
                                 this many entries are taken out of their tile and spread over a grid of
                                 their own; 0 = default (16384) */
    int32_t plan_max_k;       /* grem_plan_create: the largest k the plan is to serve, 0 = 16, at most 32.
                                 Above 16 the plan is laid out with narrower column blocks (2^16 vertices)
                                 and more hub shares; it still serves every smaller k */
    int32_t reserved[3];      /* must be zero */
} grem_options;

/* grem_partition_state with options.  GREM_ERR_ARG also for an unknown histogram mode, an option out
 * of range, GREM_HIST_LDS with k > 1024, GREM_HIST_SWEEP with k > 32 or a geometry the two-phase
 * route cannot take. */
int grem_partition_opt(const void *rowptr, int32_t rowptr_bits, const int32_t *colidx, int64_t n,
                       int32_t k, double balance_slack, int64_t chunk, int32_t refine_passes,
                       const int32_t *seed_labels, int32_t *labels_out, int64_t *sizes_out,
                       uint32_t *estimates_out, const grem_options *options, void *stream);

/* ---- Several runs on one graph -----------------------------------------------------------------
 * The two-phase route (k <= 32) works on a re-laid-out copy of the CSR entries that depends only on
 * the graph, `chunk` and the two-phase options -- not on k, the slack, the seed or the number of
 * passes.  A plan holds that copy, so that further runs on the same graph (other seeds, slacks, k,
 * pass counts; the levels of a recursive driver) skip the re-layout, which otherwise is about half
 * of a call.
 *
 * grem_plan_create re-lays the entries out (synchronous: it returns when the plan is complete) into
 * device memory the plan owns (hipMalloc; 5 bytes per entry and per pad slot plus the offset tables, 5.8 per
 * entry in all on a 3.2e9-entry power-law graph; an intermediate
 * copy of 4 bytes per entry is allocated stream-ordered and released before the call returns).
 * rowptr must stay valid and unchanged while the plan lives; colidx is not read after the call
 * returns.  Errors: GREM_ERR_ARG (bad arguments or options, or a geometry the two-phase route cannot
 * take: more than 4096 column blocks, ...), GREM_ERR_NOMEM, GREM_ERR_HIP, GREM_ERR_RANGE.
 * grem_plan_destroy synchronises the device and frees the plan (NULL is allowed).
 *
 * grem_partition_planned: the run of grem_partition_opt for the plan's graph and chunk size, k <= grem_plan_max_k,
 * same result bit for bit.  Per-call state (labels, estimates, the looked-up labels: about 0.5
 * bytes per entry -- 1 byte when k > 16 -- plus n*(2k+1) bytes) comes from the workspace or a stream-ordered allocation.
 * Several runs may use one plan at the same time (it is read-only).  Without a seed the call reads
 * nothing back and returns as soon as its work is enqueued. */
typedef struct grem_plan grem_plan;
int grem_plan_create(const void *rowptr, int32_t rowptr_bits, const int32_t *colidx, int64_t n,
                     int64_t chunk, const grem_options *options, void *stream, grem_plan **plan_out);
int grem_plan_destroy(grem_plan *plan);
size_t grem_plan_device_bytes(const grem_plan *plan);
/* Largest k the plan serves: options.plan_max_k (16 by default), or less for a graph so full of hubs that the hub counters of a
 * workgroup would not fit its LDS at that k (GREM_ERR_ARG beyond it). */
int32_t grem_plan_max_k(const grem_plan *plan);
/* Bytes of workspace (grem_set_workspace) with which such a grem_partition_planned call allocates
 * nothing: the run's labels, estimates and looked-up labels.  seeded / with_estimates_out: whether
 * seed_labels / estimates_out will be passed.  0 on bad arguments.  (Without a workspace every call
 * allocates this much stream-ordered and gives it back when its work is done; for large graphs
 * that alone can take longer than the run.) */
size_t grem_plan_call_bytes(const grem_plan *plan, int32_t k, int32_t refine_passes, int32_t seeded,
                            int32_t with_estimates_out);
int grem_partition_planned(const grem_plan *plan, int32_t k, double balance_slack,
                           int32_t refine_passes, const int32_t *seed_labels, int32_t *labels_out,
                           int64_t *sizes_out, uint32_t *estimates_out, void *stream);

/* ---- Evaluating a labelling on a plan -----------------------------------------------------------
 * cnt_nbrs (Alg. 2) of every vertex at once under a labelling that stays as it is:
 *   counts_out[v*k + j] = number of CSR entries of row v whose column has label j
 * (columns without a label are in no count).  The plan's copy of the entries serves every label
 * look-up from LDS, where a walk over the CSR arrays pays a cache miss per entry: on a graph whose
 * label table exceeds the L2 this is several times faster than grem_edge_cut / grem_expected_cut.
 * labels: n device int32, each -1 (no label) or in [0, k); k <= grem_plan_max_k.  counts_out: n*k device uint32,
 * 16-byte aligned.  State comes from the workspace or a stream-ordered allocation:
 * grem_plan_call_bytes(plan, k, 0, 1, 1) bytes (grem_plan_edge_cut: n*k*4 more).  One read-back (the
 * labels' validity) happens inside the call.
 * Errors: GREM_ERR_ARG, GREM_ERR_SEED (a label outside -1 .. k-1), GREM_ERR_NOMEM, GREM_ERR_HIP.
 *
 * grem_plan_edge_cut: the result of grem_edge_cut for the plan's graph (a vertex without a label differs
 * from every labelled neighbour), from those counts.
 * grem_plan_expected_cut (declared with grem_expected_cut below): Eq. (1) from those counts.
 * grem_plan_n: the plan's number of vertices (0 for NULL). */
int64_t grem_plan_n(const grem_plan *plan);
int grem_plan_neighbour_counts(const grem_plan *plan, int32_t k, const int32_t *labels,
                               uint32_t *counts_out, void *stream);
int grem_plan_edge_cut(const grem_plan *plan, int32_t k, const int32_t *labels,
                       int64_t *cut_entries_out, void *stream);

/* Number of CSR entries (v,u) with labels[v] != labels[u] (Sec. 1: cut edges have their endpoints
 * in different partitions), written to the single device int64 *cut_entries_out.  For a symmetric
 * loop-free CSR the undirected cut is half of it and the cut fraction is cut_entries / nnz.
 * labels: n int32 values, any values. */
int grem_edge_cut(const int64_t *rowptr, const int32_t *colidx, int64_t n, const int32_t *labels,
                  int64_t *cut_entries_out, void *stream);
int grem_edge_cut_r32(const int32_t *rowptr, const int32_t *colidx, int64_t n,
                      const int32_t *labels, int64_t *cut_entries_out, void *stream);

/* Host helpers.  grem_capacity returns P (or -1 on bad arguments). */
int64_t grem_capacity(int64_t n, int32_t k, double balance_slack);

/* Bytes of device workspace with which any partition call on such a graph runs on the plain route
 * without allocating: E (n*k*4; subtract it when estimates_out is passed), the compact labels, the
 * chunk's proposals and the admission tables.  0 on bad arguments. */
size_t grem_workspace_bytes(int64_t n, int32_t k, int64_t chunk);

/* Bytes with which a call can also take the two-phase route (k <= 32) without allocating: an upper
 * bound for any graph of n rows and nnz entries under the given options (NULL = defaults): the
 * re-laid-out copy and its tables, and, sharing one region, the intermediate copy of the re-layout
 * (4 bytes per entry) and the per-call state.  Never less than grem_workspace_bytes.  A workspace
 * between the two sizes makes GREM_HIST_AUTO keep the plain route.  0 on bad arguments. */
size_t grem_workspace_bytes_two_phase(int64_t n, int64_t nnz, int32_t k, int64_t chunk,
                                      const grem_options *options);

/* Optional caller-owned workspace (device memory, 256-byte aligned) used by later partition
 * calls (not by plans) instead of per-call stream-ordered allocations; (NULL, 0) removes it.  The
 * library never frees it.  Process-wide; calls that use it must not overlap in time. */
int grem_set_workspace(void *dev_ptr, size_t bytes);

/* ---- Measurement aids (process-wide; not meant for concurrent runs) ------------------------------
 * Timing with HIP events on the caller's stream.  Level 0: off.  Level 1: one event at the start
 * of a partition call, one before its first pass and one after every pass and after the final
 * expansion of the outputs (grem_profile_read_marks).  Level 2: also two events around every kernel
 * launch (grem_profile_read; the brackets slow a call down by a few per cent).
 * grem_profile_read synchronises on the recorded events, adds up the launches of one kernel class
 * since the last grem_profile_reset, and returns total milliseconds and the launch count.
 * grem_profile_read_marks writes the milliseconds between consecutive marks since the last reset:
 * [0] everything before the first pass (validation, plan, re-layout), [1 .. refine_passes + 1] the
 * passes, then the expansion of the outputs; returns the number of intervals written (at most
 * `capacity`) or a negative error code.  Classes: */
#define GREM_KERNEL_PREPASS 0
#define GREM_KERNEL_SCORE 1      /* row stream + label gather + histogram + blend + argmax; on the
                                    two-phase path: histogram of stored look-ups + blend + argmax */
#define GREM_KERNEL_COUNT 2
#define GREM_KERNEL_SCAN 3
#define GREM_KERNEL_APPLY 4      /* admission; two-phase path with few hubs per chunk: with the hubs' blend and proposal */
#define GREM_KERNEL_SPILL_SCAN 5
#define GREM_KERNEL_SPILL_FILL 6 /* two-phase path, chunks of at most 1024 tiles: the whole spill in one launch */
#define GREM_KERNEL_EXPAND 7
#define GREM_KERNEL_RELAYOUT 8   /* one-time planning and re-layout of the entries (two-phase path) */
#define GREM_KERNEL_LOOKUP 9     /* two-phase path: label look-ups for the entries that refer to a chunk */
#define GREM_KERNEL_HUBS 10      /* blend and proposal of the high-degree rows of the two-phase path */
#define GREM_KERNEL_CLASSES 11
int grem_profile_enable(int32_t level);
int grem_profile_reset(void);
int grem_profile_read(int32_t kernel_class, double *total_ms, int64_t *launches);
int grem_profile_read_marks(double *ms_out, int32_t capacity);

/* ---- Alg. 1 in the stream model the paper states it in (Sec. 4.1): chunks of an edge list, two
 * partitions ----------------------------------------------------------------------------------
 *
 * Input: m edges (src[e], dst[e]), 0 <= ids < n, in the caller's (random) order; loops and repeated
 * edges are allowed and count as listed.  Chunk i is edges [i*c_size, (i+1)*c_size); its nodes are
 * the distinct endpoints of its edges, taken in ascending id.
 *   first chunk:  its nodes take seed_parts[v] (the output of Alg. 1's `seed_algo`, handed in as
 *                 data; must be 0 or 1), sizes = label counts, nbr_counts[v] = cnt_nbrs of the chunk
 *   later chunks, all reads seeing parts and sizes as they were when the chunk started:
 *     fresh[v][j] = chunk edges at v whose other end (v itself for a loop) is in partition j
 *     nbr_counts[v] = fresh if v has no label, else (nbr_counts[v] + fresh) * 0.5 in IEEE double
 *     request = assign(nbr_counts[v], sizes without v, P) of Alg. 2, arg_min ties -> 0
 *     admission in ascending v: a node whose request t differs from its label moves if fewer than
 *     P - sizes[t] earlier nodes of the chunk asked for t; a rejected node that has a label keeps
 *     it; rejected new nodes are then placed one by one, ascending v, in the currently smaller
 *     partition (0 on a tie)
 *   mode GREM_EDGE_FIXED: a node that has a label is never looked at again (Sec. 4.1, "fixed
 *   assignments"; the ablation of Sec. 4.2 and Fig. 7).
 * Nodes in no edge end with -1 and zero counts.  P is Alg. 1's input (e.g. grem_capacity(n, 2, s));
 * 2P >= n is required.
 *
 * src, dst: m int32 each; seed_parts: n int32, read only at the first chunk's nodes; parts_out: n
 * int32; sizes_out: 2 int64 or NULL; nbr_counts_out: n*2 doubles, row-major, or NULL (when given it
 * is the working storage).  All device pointers.  Scratch memory is allocated on `stream` for the
 * call (about 9n bytes, plus 16n when nbr_counts_out is NULL).  The call checks the endpoints' range
 * and the seed (two small read-backs) before it enqueues the remaining chunks.
 * Errors: GREM_ERR_ARG (null pointer, m < 1, n < 1, n > 2^31-1, c_size < 1, P < 1, 2P < n, unknown
 * mode, an endpoint outside [0,n)), GREM_ERR_SEED (a first-chunk node whose seed is not 0 or 1, or
 * a seeded partition above P), GREM_ERR_NOMEM, GREM_ERR_HIP. */
#define GREM_EDGE_REFINE 0
#define GREM_EDGE_FIXED 1
int grem_edge_stream_bipartition(const int32_t *src, const int32_t *dst, int64_t m, int64_t n,
                                 int64_t c_size, int64_t P, const int32_t *seed_parts, int32_t mode,
                                 int32_t *parts_out, int64_t *sizes_out, double *nbr_counts_out,
                                 void *stream);

/* More than two partitions the paper's way (Sec. 4.1: partition into two, then re-partition each
 * part in two; Sec. 6.2: GREM partitions recursively for p > 2): 2^levels partitions.
 * Every node starts in group 0.  At level l = 0..levels-1 every group g (ascending) is split by
 * grem_edge_stream_bipartition run on the group's own subgraph: its nodes renumbered 0..nv-1 in
 * ascending id; the listed edges with both ends in the group, in stream order, in chunks of
 * ceil(m_g / chunks) edges; P = grem_capacity(nv, 2, balance_slack); first chunk seeded with
 * seed_bits[l*n + v] (the seed algorithm's answer at that level, handed in as data; 0 or 1).  Nodes of
 * the group that no such edge touches are then placed one by one, ascending id, in the currently
 * smaller half (0 on a tie).  A node of group g in half b moves to group 2g + b.
 * seed_bits: levels*n int32; labels_out: n int32, each in [0, 2^levels).  Device pointers.  Scratch
 * (about 25 bytes per edge and 30 per node) is allocated on `stream`; the call reads back a few
 * counters per group.  Errors as for grem_edge_stream_bipartition, plus GREM_ERR_ARG for levels
 * outside 1..20, chunks < 1, balance_slack < 1. */
int grem_recursive_bisection(const int32_t *src, const int32_t *dst, int64_t m, int64_t n,
                             int32_t levels, int64_t chunks, double balance_slack,
                             const int32_t *seed_bits, int32_t mode, int32_t *labels_out, void *stream);

/* The storage layer's edge buckets (Sec. 3: bucket (i, j) holds all edges from nodes of partition i
 * to nodes of partition j, each bucket stored sequentially): the m listed edges are written to
 * out_src / out_dst grouped by (labels[src], labels[dst]) in the order of i*k + j; inside a bucket
 * the edges keep their stream order (a reading: the paper fixes none; it makes the result unique).
 * bucket_offsets: k*k+1 int64, bucket (i, j) is out[bucket_offsets[i*k+j] .. bucket_offsets[i*k+j+1]).
 * labels: n int32, every endpoint's label must lie in [0, k).  All device pointers; out_* must not
 * alias the inputs.  Scratch (n + 2m bytes plus at most 512 MB of tile histograms) is allocated on
 * `stream`; one flag read-back happens inside the call.
 * Errors: GREM_ERR_ARG (null pointer, m < 1, m >= 2^32, n < 1, n > 2^31-1, k < 1, k > 128, an endpoint
 * outside [0,n), an endpoint's label outside [0,k)), GREM_ERR_NOMEM, GREM_ERR_HIP. */
int grem_edge_buckets(const int32_t *src, const int32_t *dst, int64_t m, int64_t n,
                      const int32_t *labels, int32_t k, int32_t *out_src, int32_t *out_dst,
                      int64_t *bucket_offsets, void *stream);

/* Eq. (1) of Sec. 4.2: the expected number of cut edges when every node is assigned greedily from a
 * fraction x of the edges while all other nodes hold the given two-way labelling.  For node i with
 * k_i labelled neighbours (labels 0 or 1; others are skipped), k0_i of them in the partition holding
 * more, and d_i = min(k_i, floor(k_i*x + 0.5)) draws (the paper's k*x, made an integer):
 *   out[0] = sum_i (k_i - k0_i)(1 - q_i) + k0_i q_i,  q_i = Pr(K < d_i/2), K ~ Hypergeometric(k_i, k0_i, d_i)
 *   out[1] = sum_i (k_i - k0_i)                        (the value at x = 1)
 * Every edge of a symmetric CSR is seen from both ends.  The expected cuts with refinement over two
 * chunks are the same expression at 2x.  rowptr (rowptr_bits 32 or 64), colidx, labels (n int32), out
 * (2 doubles): device pointers.  Floating point: the tail is summed in double (in the log domain when a node has more than 256 draws);
 * agreement with an exact evaluation to about 1e-9 relative.  Errors: GREM_ERR_ARG (null pointer,
 * n < 1, bad rowptr_bits, x outside (0, 1]), GREM_ERR_NOMEM, GREM_ERR_HIP. */
int grem_expected_cut(const void *rowptr, int32_t rowptr_bits, const int32_t *colidx, int64_t n,
                      const int32_t *labels, double x, double *out, void *stream);

/* Eq. (1) for the graph of a plan: the same two sums as grem_expected_cut (up to the order of the
 * additions: about 1e-13 relative), with the neighbour counts taken from grem_plan_neighbour_counts.
 * labels: n device int32, each -1, 0 or 1 (GREM_ERR_SEED otherwise).  Allocates n*8 bytes and the
 * per-workgroup sums stream-ordered, beside what grem_plan_neighbour_counts takes.
 * Errors: GREM_ERR_ARG (null pointer, x outside (0, 1]), GREM_ERR_SEED, GREM_ERR_NOMEM, GREM_ERR_HIP. */
int grem_plan_expected_cut(const grem_plan *plan, const int32_t *labels, double x, double *out,
                           void *stream);

/* grem_expected_cut for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * result, bit for bit, as grem_expected_cut, but the per-workgroup partial sums go to a fixed 4 MiB
 * buffer that is part of the library's device image (one copy per GPU, held until the process
 * ends) instead of a stream-ordered allocation; the call allocates and frees nothing.
 *   - n may be at most grem_expected_cut_noalloc_max_n() (4,194,304 rows: one workgroup per 16
 *     rows, two doubles per workgroup); a larger n returns GREM_ERR_LIMIT and launches nothing.
 *   - The device that owns the arrays and `stream` must be the current device.  The first call on
 *     a device looks up that device's copy of the buffer (hipGetSymbolAddress; no allocation, but
 *     make that first call outside graph capture).
 *   - All calls on one GPU share the buffer: calls that overlap in time on one GPU (different
 *     streams, different threads) race and must be serialised by the caller.  Nothing in the
 *     buffer has to survive or be cleared between calls: every slot a call reads it has written.
 * Errors: GREM_ERR_ARG as for grem_expected_cut, GREM_ERR_LIMIT, GREM_ERR_HIP. */
int grem_expected_cut_noalloc(const void *rowptr, int32_t rowptr_bits, const int32_t *colidx, int64_t n,
                              const int32_t *labels, double x, double *out, void *stream);
int64_t grem_expected_cut_noalloc_max_n(void);

/* Number of listed edges whose ends carry different labels (Sec. 1), written to the single device
 * int64 *cut_out.  parts: int32 labels covering every listed id, any values. */
int grem_edge_list_cut(const int32_t *src, const int32_t *dst, int64_t m, const int32_t *parts,
                       int64_t *cut_out, void *stream);

/* Timing of the edge kernel (cnt_nbrs over a chunk's edges) with HIP events on the caller's stream,
 * for measurement: while enabled each launch is bracketed by two events; the read synchronises on
 * them, returns their total in milliseconds, the launch count and the number of edges those
 * launches processed (each may be NULL), and forgets them.  Calls made by
 * grem_recursive_bisection are included. */
int grem_edge_stream_profile_enable(int32_t on);
int grem_edge_stream_profile_read(double *count_ms, int64_t *launches, int64_t *edges);

const char *grem_status_string(int code);
const char *grem_kernel_name(int32_t kernel_class);

#ifdef __cplusplus
}
#endif
#endif /* GREM_H */
