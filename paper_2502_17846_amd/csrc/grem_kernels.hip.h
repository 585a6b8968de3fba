// Device kernels of the GREM partitioner for gfx950 (wave64).  Included once, by grem.hip.
//
// One chunk of rows is processed by a short sequence of launches on the caller's stream:
//   score  : stream the chunk's CSR rows, gather neighbour labels, histogram them per vertex,
//            blend into E, and pick each vertex's proposal               (Alg. 2 cnt_nbrs, assign;
//                                                                          Alg. 1 blend)
//   count  : per tile of vertices, how many movers propose each partition
//   scan   : exclusive prefix of those counts over the tiles (id order), room = P - S
//   apply  : admit movers by rank, relabel, update sizes                 (Alg. 2 fix_sizes)
//   spill  : (first pass only) place rejected new vertices one by one in the smallest partition
//            -- done in closed form by levels                            (Alg. 2 arg_min fallback)
// Every quantity is an integer and every cross-thread combination is an integer sum or a rank in
// vertex-id order, so the result does not depend on scheduling.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace grem {

constexpr int kScoreThreads = 256;
constexpr int kAdmitThreads = 256;
constexpr int kAdmitTile = 1024;       // vertices per tile in count/apply/spill
constexpr int kScanThreads = 1024;
constexpr int kGlobalTile = 64;        // vertices per tile when histograms live in E's rows
constexpr int GREM_MAX_K_DEVICE = 4096;

template <typename LabelT> struct LabelTraits;
template <> struct LabelTraits<uint8_t> { static constexpr uint32_t kUnassigned = 0xFFu; };
template <> struct LabelTraits<uint16_t> { static constexpr uint32_t kUnassigned = 0xFFFFu; };

__device__ __forceinline__ int lane_id() { return (int)__lane_id(); }
__device__ __forceinline__ unsigned long long lanes_below(int lane) {
    return (lane == 0) ? 0ull : (~0ull >> (64 - lane));
}

// Largest r in [0, tv) with rowrel[r] <= i; tv is a power of two.  Picks the row that owns entry
// i and skips empty rows (equal offsets resolve to the last, the non-empty one).
__device__ __forceinline__ int owning_row(const uint32_t *rowrel, uint32_t i, int tv) {
    int r = 0;
    for (int step = tv >> 1; step >= 1; step >>= 1)
        if (rowrel[r + step] <= i) r += step;
    return r;
}

// ------------------------------------------------------------------------------------------------
// prepass: compact labels from the seed, seed sizes, seed validity, and (when rowptr is given)
// the maximum degree
// misc[0] = max degree, misc[1] = number of invalid seed labels, misc[3] = number of entries,
// misc[5] = number of vertices the seed leaves without a label
// ------------------------------------------------------------------------------------------------
constexpr int kPrepassLdsK = 1024;      // up to this k the seed sizes are counted in LDS first
template <typename RowT, typename LabelT>
__global__ __launch_bounds__(256) void k_prepass(const RowT *__restrict__ rowptr,
                                                 const int32_t *__restrict__ seed, int64_t n, int k,
                                                 LabelT *__restrict__ Lc,
                                                 unsigned long long *__restrict__ S,
                                                 unsigned long long *__restrict__ misc) {
    __shared__ unsigned long long s_maxdeg;
    __shared__ unsigned int s_bad, s_none;
    // (a workgroup's vertices: at most n / gridDim.x + 256 < 2^32)
    __shared__ unsigned int s_size[kPrepassLdsK];
    const bool in_lds = seed && k <= kPrepassLdsK;
    if (threadIdx.x == 0) { s_maxdeg = 0; s_bad = 0; s_none = 0; }
    if (in_lds)
        for (int j = threadIdx.x; j < k; j += 256) s_size[j] = 0;
    __syncthreads();
    unsigned long long mymax = 0;
    unsigned int bad = 0, none = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) {
        if (rowptr) {
            unsigned long long d = (unsigned long long)(rowptr[v + 1] - rowptr[v]);
            if (d > mymax) mymax = d;
        }
        uint32_t lab = LabelTraits<LabelT>::kUnassigned;
        if (seed) {
            int32_t s = seed[v];
            if (s >= 0 && s < k) {
                lab = (uint32_t)s;
                // (a labelling that covers every vertex would otherwise queue n atomics at k addresses)
                if (in_lds) atomicAdd(&s_size[s], 1u);
                else atomicAdd(&S[s], 1ull);
            } else if (s != -1) {
                bad += 1;
            } else {
                none += 1;
            }
        }
        Lc[v] = (LabelT)lab;
    }
    if (mymax) atomicMax(&s_maxdeg, mymax);
    if (bad) atomicAdd(&s_bad, bad);
    if (none) atomicAdd(&s_none, none);
    __syncthreads();
    if (in_lds)
        for (int j = threadIdx.x; j < k; j += 256)
            if (s_size[j]) atomicAdd(&S[j], (unsigned long long)s_size[j]);
    if (threadIdx.x == 0) {
        if (s_maxdeg) atomicMax(&misc[0], s_maxdeg);
        if (s_bad) atomicAdd(&misc[1], (unsigned long long)s_bad);
        if (s_none) atomicAdd(&misc[5], (unsigned long long)s_none);
        if (blockIdx.x == 0 && rowptr) misc[3] = (unsigned long long)rowptr[n];
    }
}

// misc[2] = number of seeded partitions above capacity
__global__ void k_check_seed_sizes(const long long *__restrict__ S, int k, long long P,
                                   unsigned long long *__restrict__ misc) {
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < k && S[j] > P) atomicAdd(&misc[2], 1ull);
}

// ------------------------------------------------------------------------------------------------
// Long rows of the plain score kernels.  A tile's workgroup leaves out rows of `degree` entries or
// more (it would walk them alone) and appends them to the chunk's list; k_long_rows then spreads
// the entries of the listed rows over a whole grid, `part` entries per workgroup and turn, and
// k_long_propose picks their proposals.  degree = 0xFFFFFFFF: nothing is ever left out.
// ------------------------------------------------------------------------------------------------
struct LongRows {
    uint32_t degree;
    uint32_t part;
    uint32_t *count;        // rows in the list (zero before the chunk's score kernel)
    uint32_t *list;         // their vertex ids, in no particular order
};

// Every thread of the tile's workgroup calls this after rowrel is complete and *flag is 0; true
// if the tile has a long row.
__device__ __forceinline__ bool note_long_rows(const uint32_t *rowrel, int nv, int64_t v0, const LongRows &lr,
                                               int *flag) {
    if (lr.degree == 0xFFFFFFFFu) return false;
    for (int i = threadIdx.x; i < nv; i += blockDim.x) {
        if (rowrel[i + 1] - rowrel[i] >= lr.degree) {
            *flag = 1;
            lr.list[atomicAdd(lr.count, 1u)] = (uint32_t)(v0 + i);
        }
    }
    __syncthreads();
    return *flag != 0;
}

// Adds the neighbour-label counts of the listed rows, times 2^(pass-1) (1 in the first pass), to
// their rows of E with integer atomics; the counts of one part are collected in LDS first (k
// words).  The parts of all listed rows, numbered in list order, are dealt out round-robin over
// the workgroups; the list is taken kScoreThreads rows at a time (a thread per row works out its
// number of parts, a prefix sum tells every workgroup which parts of the batch are its own).
template <typename RowT, typename LabelT>
__global__ __launch_bounds__(kScoreThreads) void k_long_rows(
    const RowT *__restrict__ rowptr, const int32_t *__restrict__ colidx, const LabelT *__restrict__ Lc,
    uint32_t *__restrict__ E, int k, int pass, int64_t gather_limit, LongRows lr) {
    extern __shared__ uint32_t smem[];
    uint32_t *hist = smem;                  // k
    __shared__ uint32_t s_pre[kScoreThreads + 1];
    __shared__ uint32_t s_wtot[kScoreThreads / 64];
    constexpr uint32_t UN = LabelTraits<LabelT>::kUnassigned;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const uint32_t nlong = *lr.count;
    const uint32_t inc = pass == 0 ? 1u : (1u << (pass - 1));
    constexpr int U = 4;
    unsigned long long dealt = 0;           // parts of the batches before this one
    for (uint32_t i0 = 0; i0 < nlong; i0 += kScoreThreads) {
        uint32_t mine = 0;
        if (i0 + tid < nlong) {
            const int64_t v = (int64_t)lr.list[i0 + tid];
            const uint32_t deg = (uint32_t)((int64_t)rowptr[v + 1] - (int64_t)rowptr[v]);
            mine = (deg + lr.part - 1) / lr.part;
        }
        uint32_t run = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = __shfl_up(run, off);
            if (lane >= off) run += o;
        }
        if (lane == 63) s_wtot[wave] = run;
        __syncthreads();
        for (int w = 0; w < wave; ++w) run += s_wtot[w];
        s_pre[tid] = run - mine;
        if (tid == kScoreThreads - 1) s_pre[kScoreThreads] = run;
        __syncthreads();
        const uint32_t batch_parts = s_pre[kScoreThreads];
        // first part of this batch that falls to this workgroup
        uint32_t x = (uint32_t)((blockIdx.x + gridDim.x - (uint32_t)(dealt % gridDim.x)) % gridDim.x);
        for (; x < batch_parts; x += gridDim.x) {
            int r = 0;                      // largest r with s_pre[r] <= x
            for (int step = kScoreThreads >> 1; step >= 1; step >>= 1)
                if (s_pre[r + step] <= x) r += step;
            const uint32_t q = x - s_pre[r];
            const int64_t v = (int64_t)lr.list[i0 + r];
            const int64_t e0 = (int64_t)rowptr[v];
            const uint32_t deg = (uint32_t)((int64_t)rowptr[v + 1] - e0);
            const int32_t *cbase = colidx + e0;
            for (int j = tid; j < k; j += kScoreThreads) hist[j] = 0;
            __syncthreads();
            const uint32_t from = q * lr.part;
            const uint32_t to = (deg - from < lr.part) ? deg : from + lr.part;
            for (uint32_t base = from + tid; base < to; base += kScoreThreads * U) {
                int32_t col[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t e = base + u * kScoreThreads;
                    col[u] = (e < to) ? __builtin_nontemporal_load(cbase + e) : -1;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (col[u] >= 0 && (int64_t)col[u] < gather_limit) {
                        const uint32_t lab = (uint32_t)Lc[col[u]];
                        if (lab != UN) atomicAdd(&hist[lab], 1u);
                    }
                }
            }
            __syncthreads();
            uint32_t *erow = E + (size_t)v * (size_t)k;
            for (int j = tid; j < k; j += kScoreThreads)
                if (hist[j]) atomicAdd(&erow[j], hist[j] * inc);
            __syncthreads();
        }
        dealt += batch_parts;
        __syncthreads();                    // s_pre is rewritten by the next batch
    }
}

// One wavefront per listed row: the proposal from its (now complete) row of E, by the rule of the
// score kernels.
template <typename LabelT>
__global__ __launch_bounds__(64) void k_long_propose(const LabelT *__restrict__ Lc, const long long *__restrict__ S,
                                                     const uint32_t *__restrict__ E, LabelT *__restrict__ prop,
                                                     int64_t chunk_lo, int k, int pass, long long P, LongRows lr) {
    constexpr uint32_t UN = LabelTraits<LabelT>::kUnassigned;
    const int lane = lane_id();
    const uint32_t nlong = *lr.count;
    for (uint32_t i = blockIdx.x; i < nlong; i += gridDim.x) {
        const int64_t v = (int64_t)lr.list[i];
        const uint32_t old = (uint32_t)Lc[v];
        uint32_t best = old;
        if (!(pass == 0 && old != UN)) {
            unsigned long long bestkey = 0;
            int bestj = 0x7fffffff;
            const uint32_t *erow = E + (size_t)v * (size_t)k;
            for (int j = lane; j < k; j += 64) {
                const uint32_t rm = (uint32_t)(P - S[j]) + ((uint32_t)j == old ? 1u : 0u);
                const unsigned long long key = rm ? (((unsigned long long)erow[j] << 32) | rm) : 0ull;
                if (key > bestkey) { bestkey = key; bestj = j; }   // j ascends: first maximum kept
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const unsigned long long okey = __shfl_xor(bestkey, off);
                const int oj = __shfl_xor(bestj, off);
                if (okey > bestkey || (okey == bestkey && oj < bestj)) { bestkey = okey; bestj = oj; }
            }
            best = (uint32_t)bestj;
        }
        if (lane == 0) prop[v - chunk_lo] = (LabelT)best;
    }
}

// ------------------------------------------------------------------------------------------------
// score, histograms in LDS.  One workgroup owns `tv` consecutive rows (tv a power of two) and
// walks their entries edge-parallel: consecutive lanes read consecutive colidx entries (coalesced),
// gather the neighbour's label, find the owning row in the tile's row offsets (LDS) and add 1 to
// that row's counter of the label (LDS atomic).  Then the tile's slice of E, which is contiguous,
// is blended in one coalesced sweep, and one thread per vertex picks the proposal.
//   gather_limit: neighbours with id >= gather_limit are known to be unassigned (first pass of an
//   unseeded run: everything from the chunk's first row on), so their label is not fetched.
// ------------------------------------------------------------------------------------------------
template <typename RowT, typename LabelT>
__global__ __launch_bounds__(kScoreThreads) void k_score_lds(
    const RowT *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const LabelT *__restrict__ Lc, const long long *__restrict__ S, uint32_t *__restrict__ E,
    LabelT *__restrict__ prop, int64_t chunk_lo, int64_t chunk_hi, int k, int tv, int pass,
    long long P, int64_t gather_limit, LongRows lr) {
    extern __shared__ uint32_t smem[];
    __shared__ int s_long;
    uint32_t *hist = smem;                  // tv * k
    uint32_t *rowrel = hist + (size_t)tv * k;   // tv + 1
    uint32_t *room = rowrel + tv + 1;       // k
    constexpr uint32_t UN = LabelTraits<LabelT>::kUnassigned;
    const int tid = threadIdx.x;
    const int64_t v0 = chunk_lo + (int64_t)blockIdx.x * tv;
    const int64_t left = chunk_hi - v0;
    const int nv = left < tv ? (int)left : tv;
    const int64_t e0 = (int64_t)rowptr[v0];

    for (int i = tid; i <= tv; i += kScoreThreads) {
        int ii = i < nv ? i : nv;
        rowrel[i] = (uint32_t)((int64_t)rowptr[v0 + ii] - e0);
    }
    for (int i = tid; i < tv * k; i += kScoreThreads) hist[i] = 0;
    for (int j = tid; j < k; j += kScoreThreads) room[j] = (uint32_t)(P - S[j]);
    if (tid == 0) s_long = 0;
    __syncthreads();
    const bool any_long = note_long_rows(rowrel, nv, v0, lr, &s_long);

    const uint32_t ne = rowrel[tv];
    const int32_t *cbase = colidx + e0;
    constexpr int U = 4;
    auto count_entries = [&](uint32_t from, uint32_t to) {
        for (uint32_t base = from + tid; base < to; base += kScoreThreads * U) {
            int32_t col[U];
            uint32_t lab[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t i = base + u * kScoreThreads;
                col[u] = (i < to) ? __builtin_nontemporal_load(cbase + i) : -1;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                lab[u] = UN;
                if (col[u] >= 0 && (int64_t)col[u] < gather_limit) lab[u] = (uint32_t)Lc[col[u]];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (lab[u] != UN) {
                    int r = owning_row(rowrel, base + u * kScoreThreads, tv);
                    atomicAdd(&hist[r * k + (int)lab[u]], 1u);
                }
            }
        }
    };
    if (!any_long) {
        count_entries(0, ne);
    } else {                                    // the stretches between the long rows
        uint32_t from = 0;
        for (int r = 0; r < nv; ++r) {
            const uint32_t a = rowrel[r], b = rowrel[r + 1];
            if (b - a >= lr.degree) { count_entries(from, a); from = b; }
        }
        count_entries(from, ne);
    }
    __syncthreads();

    // blend: E = h (first pass) or E += h * 2^(pass-1); the blended row stays in LDS.  A long row's
    // estimates are only cleared here (first pass): k_long_rows adds its counts to them.
    {
        uint32_t *Etile = E + (size_t)v0 * (size_t)k;
        const int total = nv * k;
        if (any_long) {
            const int sh = pass - 1;
            for (int i = tid; i < total; i += kScoreThreads) {
                const int r = i / k;
                if (rowrel[r + 1] - rowrel[r] >= lr.degree) {
                    if (pass == 0) Etile[i] = 0u;
                } else {
                    const uint32_t e = pass == 0 ? hist[i] : Etile[i] + (hist[i] << sh);
                    hist[i] = e;
                    Etile[i] = e;
                }
            }
        } else if (pass == 0) {
            for (int i = tid; i < total; i += kScoreThreads)
                __builtin_nontemporal_store(hist[i], Etile + i);
        } else {
            const int sh = pass - 1;
            for (int i = tid; i < total; i += kScoreThreads) {
                uint32_t e = __builtin_nontemporal_load(Etile + i) + (hist[i] << sh);
                hist[i] = e;
                __builtin_nontemporal_store(e, Etile + i);
            }
        }
    }
    __syncthreads();

    // proposal: best partition with room by (E desc, room desc, id asc); a thread per vertex, or, when
    // there are many partitions, a wavefront per vertex
    if (k >= 64) {
        const int lane = lane_id();
        for (int t = tid >> 6; t < nv; t += kScoreThreads / 64) {
            if (any_long && rowrel[t + 1] - rowrel[t] >= lr.degree) continue;     // k_long_propose's
            const int64_t v = v0 + t;
            const uint32_t old = (uint32_t)Lc[v];
            uint32_t best = old;
            if (!(pass == 0 && old != UN)) {
                unsigned long long bestkey = 0;
                int bestj = 0x7fffffff;
                const uint32_t *hrow = hist + t * k;
                for (int j = lane; j < k; j += 64) {
                    const uint32_t rm = room[j] + ((uint32_t)j == old ? 1u : 0u);
                    const unsigned long long key = rm ? (((unsigned long long)hrow[j] << 32) | rm) : 0ull;
                    if (key > bestkey) { bestkey = key; bestj = j; }   // j ascends: first maximum kept
                }
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) {
                    const unsigned long long okey = __shfl_xor(bestkey, off);
                    const int oj = __shfl_xor(bestj, off);
                    if (okey > bestkey || (okey == bestkey && oj < bestj)) { bestkey = okey; bestj = oj; }
                }
                best = (uint32_t)bestj;
            }
            if (lane == 0) prop[v - chunk_lo] = (LabelT)best;
        }
        return;
    }
    for (int t = tid; t < nv; t += kScoreThreads) {
        if (any_long && rowrel[t + 1] - rowrel[t] >= lr.degree) continue;     // k_long_propose's
        const int64_t v = v0 + t;
        const uint32_t old = (uint32_t)Lc[v];
        uint32_t best = old;
        if (!(pass == 0 && old != UN)) {
            unsigned long long bestkey = 0;
            int bestj = 0x7fffffff;
            int jj = t % k;
            const uint32_t *hrow = hist + t * k;
            for (int j = 0; j < k; ++j) {
                uint32_t rm = room[jj] + ((uint32_t)jj == old ? 1u : 0u);
                unsigned long long key = rm ? (((unsigned long long)hrow[jj] << 32) | rm) : 0ull;
                if (key > bestkey || (key == bestkey && key != 0 && jj < bestj)) {
                    bestkey = key;
                    bestj = jj;
                }
                jj += 1;
                if (jj == k) jj = 0;
            }
            best = (uint32_t)bestj;
        }
        prop[v - chunk_lo] = (LabelT)best;
    }
}

// ------------------------------------------------------------------------------------------------
// score, histograms in global memory (large k): counts are added straight into E's rows with
// integer atomics of 2^(pass-1) (1 in the first pass, after zeroing the rows); proposals are
// picked by one wavefront per vertex with a shuffle arg-max.
// ------------------------------------------------------------------------------------------------
template <typename RowT, typename LabelT>
__global__ __launch_bounds__(kScoreThreads) void k_score_global(
    const RowT *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const LabelT *__restrict__ Lc, const long long *__restrict__ S, uint32_t *__restrict__ E,
    LabelT *__restrict__ prop, int64_t chunk_lo, int64_t chunk_hi, int k, int pass, long long P,
    int64_t gather_limit, LongRows lr) {
    extern __shared__ uint32_t smem[];
    __shared__ int s_long;
    constexpr int tv = kGlobalTile;
    uint32_t *rowrel = smem;            // tv + 1
    uint32_t *room = rowrel + tv + 1;   // k
    constexpr uint32_t UN = LabelTraits<LabelT>::kUnassigned;
    const int tid = threadIdx.x;
    const int64_t v0 = chunk_lo + (int64_t)blockIdx.x * tv;
    const int64_t left = chunk_hi - v0;
    const int nv = left < tv ? (int)left : tv;
    const int64_t e0 = (int64_t)rowptr[v0];
    uint32_t *Etile = E + (size_t)v0 * (size_t)k;

    for (int i = tid; i <= tv; i += kScoreThreads) {
        int ii = i < nv ? i : nv;
        rowrel[i] = (uint32_t)((int64_t)rowptr[v0 + ii] - e0);
    }
    for (int j = tid; j < k; j += kScoreThreads) room[j] = (uint32_t)(P - S[j]);
    if (pass == 0) {
        const int total = nv * k;
        for (int i = tid; i < total; i += kScoreThreads) Etile[i] = 0u;
        __threadfence();
    }
    if (tid == 0) s_long = 0;
    __syncthreads();
    const bool any_long = note_long_rows(rowrel, nv, v0, lr, &s_long);

    const uint32_t ne = rowrel[tv];
    const int32_t *cbase = colidx + e0;
    const uint32_t inc = pass == 0 ? 1u : (1u << (pass - 1));
    constexpr int U = 4;
    auto count_entries = [&](uint32_t from, uint32_t to) {
        for (uint32_t base = from + tid; base < to; base += kScoreThreads * U) {
            int32_t col[U];
            uint32_t lab[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t i = base + u * kScoreThreads;
                col[u] = (i < to) ? __builtin_nontemporal_load(cbase + i) : -1;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                lab[u] = UN;
                if (col[u] >= 0 && (int64_t)col[u] < gather_limit) lab[u] = (uint32_t)Lc[col[u]];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (lab[u] != UN) {
                    int r = owning_row(rowrel, base + u * kScoreThreads, tv);
                    atomicAdd(&Etile[(size_t)r * k + lab[u]], inc);
                }
            }
        }
    };
    if (!any_long) {
        count_entries(0, ne);
    } else {                                    // the stretches between the long rows
        uint32_t from = 0;
        for (int r = 0; r < nv; ++r) {
            const uint32_t a = rowrel[r], b = rowrel[r + 1];
            if (b - a >= lr.degree) { count_entries(from, a); from = b; }
        }
        count_entries(from, ne);
    }
    __threadfence();
    __syncthreads();

    const int lane = lane_id();
    const int wave = tid >> 6;
    constexpr int nwaves = kScoreThreads / 64;
    for (int t = wave; t < nv; t += nwaves) {
        if (any_long && rowrel[t + 1] - rowrel[t] >= lr.degree) continue;     // k_long_propose's
        const int64_t v = v0 + t;
        const uint32_t old = (uint32_t)Lc[v];
        uint32_t best = old;
        if (!(pass == 0 && old != UN)) {
            unsigned long long bestkey = 0;
            int bestj = 0x7fffffff;
            const uint32_t *erow = Etile + (size_t)t * k;
            for (int j = lane; j < k; j += 64) {
                uint32_t e = __hip_atomic_load(erow + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                uint32_t rm = room[j] + ((uint32_t)j == old ? 1u : 0u);
                unsigned long long key = rm ? (((unsigned long long)e << 32) | rm) : 0ull;
                if (key > bestkey) { bestkey = key; bestj = j; }   // j ascends: first maximum kept
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                unsigned long long okey = __shfl_xor(bestkey, off);
                int oj = __shfl_xor(bestj, off);
                if (okey > bestkey || (okey == bestkey && oj < bestj)) { bestkey = okey; bestj = oj; }
            }
            best = (uint32_t)bestj;
        }
        if (lane == 0) prop[v - chunk_lo] = (LabelT)best;
    }
}

// ------------------------------------------------------------------------------------------------
// count: cnt[tile][t] = movers of the tile proposing t
// ------------------------------------------------------------------------------------------------
template <typename LabelT>
__global__ __launch_bounds__(kAdmitThreads) void k_count(const LabelT *__restrict__ Lc,
                                                         const LabelT *__restrict__ prop,
                                                         int64_t chunk_lo, int64_t chunk_hi, int k,
                                                         uint32_t *__restrict__ cnt) {
    extern __shared__ uint32_t smem[];
    uint32_t *c = smem;   // k
    const int tid = threadIdx.x;
    for (int j = tid; j < k; j += kAdmitThreads) c[j] = 0;
    __syncthreads();
    const int64_t lo = chunk_lo + (int64_t)blockIdx.x * kAdmitTile;
    for (int i = tid; i < kAdmitTile; i += kAdmitThreads) {
        int64_t v = lo + i;
        if (v < chunk_hi) {
            uint32_t t = prop[v - chunk_lo];
            if (t != (uint32_t)Lc[v]) atomicAdd(&c[t], 1u);
        }
    }
    __syncthreads();
    uint32_t *out = cnt + (size_t)blockIdx.x * k;
    for (int j = tid; j < k; j += kAdmitThreads) out[j] = c[j];
}

// ------------------------------------------------------------------------------------------------
// scan: per partition, exclusive prefix of cnt over the tiles (in place); room[j] = P - S[j]
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kScanThreads) void k_scan(uint32_t *__restrict__ cnt, int ntiles, int k,
                                                       const long long *__restrict__ S, long long P,
                                                       long long *__restrict__ room) {
    __shared__ uint32_t part[kScanThreads];
    const int tid = threadIdx.x;
    for (int j = tid; j < k; j += kScanThreads) room[j] = P - S[j];
    for (int c0 = 0; c0 < k; c0 += kScanThreads) {
        const int kc = (k - c0) < kScanThreads ? (k - c0) : kScanThreads;
        const int nseg = kScanThreads / kc;
        const int col = tid % kc, seg = tid / kc;
        const bool active = seg < nseg;
        const int tps = (ntiles + nseg - 1) / nseg;
        const int tlo = seg * tps;
        const int thi = (tlo + tps < ntiles) ? tlo + tps : ntiles;
        uint32_t sum = 0;
        if (active)
            for (int t = tlo; t < thi; ++t) sum += cnt[(size_t)t * k + c0 + col];
        part[tid] = active ? sum : 0u;
        __syncthreads();
        if (active) {
            uint32_t base = 0;
            for (int s = 0; s < seg; ++s) base += part[s * kc + col];
            for (int t = tlo; t < thi; ++t) {
                size_t idx = (size_t)t * k + c0 + col;
                uint32_t c = cnt[idx];
                cnt[idx] = base;
                base += c;
            }
        }
        __syncthreads();
    }
}

// Rank of each lane among the lanes of its wavefront that are `active` and hold the same `t`,
// in lane order; *same_total = how many such lanes; *leader = is the first of them.
__device__ __forceinline__ int rank_among_equal(bool active, uint32_t t, int lane, int *same_total,
                                                bool *leader) {
    int rank = 0;
    *same_total = 0;
    *leader = false;
    unsigned long long remaining = __ballot(active);
    while (remaining) {
        int first = __ffsll((long long)remaining) - 1;
        uint32_t lt = (uint32_t)__shfl((int)t, first);
        unsigned long long m = __ballot(active && t == lt);
        if (active && t == lt) {
            rank = __popcll(m & lanes_below(lane));
            *same_total = __popcll(m);
            *leader = (lane == first);
        }
        remaining &= ~m;
    }
    return rank;
}

// ------------------------------------------------------------------------------------------------
// apply: admit movers whose rank among the chunk's earlier movers to the same partition is below
// the room; relabel; size deltas; in the first pass count the vertices left unassigned per tile.
//   SELF_PREFIX = false: base[tile][t] = movers to t in earlier tiles (k_scan's output)
//   SELF_PREFIX = true : base[tile][t] = movers to t in that tile; the workgroup adds up the rows of
//                        the earlier tiles itself (no k_scan launch; pays when tiles * k is small)
// room[t] = P - S[t] as of the chunk's start.
// LDS: run[k], wcnt[nwaves * k], dS[k], tbl[k] (SELF_PREFIX)
// ------------------------------------------------------------------------------------------------
template <typename LabelT, bool SELF_PREFIX>
__global__ __launch_bounds__(kAdmitThreads) void k_apply(
    LabelT *__restrict__ Lc, const LabelT *__restrict__ prop, int64_t chunk_lo, int64_t chunk_hi,
    int k, const uint32_t *__restrict__ base, const long long *__restrict__ room,
    unsigned long long *__restrict__ S, uint32_t *__restrict__ ocnt, int pass) {
    extern __shared__ uint32_t smem[];
    constexpr int nwaves = kAdmitThreads / 64;
    constexpr int rounds = kAdmitTile / kAdmitThreads;
    uint32_t *run = smem;                 // k       movers seen so far in this tile
    uint32_t *wcnt = run + k;             // nwaves*k movers of this round per wave
    int32_t *dS = (int32_t *)(wcnt + nwaves * k);   // k size deltas
    uint32_t *tbl = (uint32_t *)(dS + k); // k       movers in earlier tiles (SELF_PREFIX)
    __shared__ uint32_t s_unassigned;
    constexpr uint32_t UN = LabelTraits<LabelT>::kUnassigned;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int64_t lo = chunk_lo + (int64_t)blockIdx.x * kAdmitTile;

    // this thread's vertices, one per round
    uint32_t tv[rounds], oldv[rounds];
#pragma unroll
    for (int r = 0; r < rounds; ++r) {
        const int64_t v = lo + r * kAdmitThreads + tid;
        tv[r] = 0;
        oldv[r] = 0;
        if (v < chunk_hi) { tv[r] = prop[v - chunk_lo]; oldv[r] = (uint32_t)Lc[v]; }
    }

    for (int j = tid; j < k; j += kAdmitThreads) { run[j] = 0; dS[j] = 0; if (SELF_PREFIX) tbl[j] = 0; }
    for (int j = tid; j < nwaves * k; j += kAdmitThreads) wcnt[j] = 0;
    if (tid == 0) s_unassigned = 0;
    __syncthreads();
    const uint32_t *tbase = base + (size_t)blockIdx.x * k;
    if (SELF_PREFIX) {
        for (int c0 = 0; c0 < k; c0 += kAdmitThreads) {
            const int kc = (k - c0) < kAdmitThreads ? (k - c0) : kAdmitThreads;
            const int nseg = kAdmitThreads / kc;
            const int col = tid % kc, seg = tid / kc;
            if (seg < nseg) {
                uint32_t sum = 0;
                for (int t = seg; t < (int)blockIdx.x; t += nseg) sum += base[(size_t)t * k + c0 + col];
                if (sum) atomicAdd(&tbl[c0 + col], sum);
            }
        }
        __syncthreads();
        tbase = tbl;
    }
    uint32_t my_unassigned = 0;
#pragma unroll
    for (int round = 0; round < rounds; ++round) {
        const int64_t v = lo + round * kAdmitThreads + tid;
        const bool inside = v < chunk_hi;
        const uint32_t t = tv[round], old = oldv[round];
        const bool mover = inside && t != old;
        int same_total; bool leader;
        const int wrank = rank_among_equal(mover, t, lane, &same_total, &leader);
        if (leader) wcnt[wave * k + t] = (uint32_t)same_total;
        __syncthreads();
        bool admitted = false;
        if (mover) {
            long long rank = (long long)tbase[t] + run[t] + wrank;
            for (int w = 0; w < wave; ++w) rank += wcnt[w * k + t];
            admitted = rank < room[t];
        }
        __syncthreads();
        if (leader) { atomicAdd(&run[t], (uint32_t)same_total); wcnt[wave * k + t] = 0; }
        if (admitted) {
            Lc[v] = (LabelT)t;
            atomicAdd(&dS[t], 1);
            if (old != UN) atomicAdd(&dS[old], -1);
        } else if (inside && old == UN) {
            my_unassigned += 1;    // rejected new vertex (a new vertex is always a mover)
        }
        __syncthreads();
    }
    if (pass == 0) {
        if (my_unassigned) atomicAdd(&s_unassigned, my_unassigned);
    }
    __syncthreads();
    for (int j = tid; j < k; j += kAdmitThreads) {
        int32_t d = dS[j];
        if (d != 0) atomicAdd(&S[j], (unsigned long long)(long long)d);
    }
    if (pass == 0 && tid == 0) ocnt[blockIdx.x] = s_unassigned;
}

// The waves' mover counts wcnt[tile][wave][t] of a workgroup's tiles -> the number of movers to t before
// that wave: in its tile's earlier waves and in the workgroup's earlier tiles (own[tile][t] movers each).
// One entry per thread and turn, the 16 waves of a (tile, t) pair in 16 neighbouring lanes.
template <int KP, int TPW>
__device__ __forceinline__ void wave_counts_to_prefix(uint32_t (*wcnt)[kAdmitTile / 64][KP], const uint32_t (*own)[KP]) {
    constexpr int nwaves = kAdmitTile / 64;
    static_assert(nwaves == 16, "a (tile, partition) pair's waves fill a row of 16 lanes");
    for (int e = threadIdx.x; e < TPW * nwaves * KP; e += kAdmitTile) {
        const int w = e & (nwaves - 1), col = (e / nwaves) % KP, h = e / (nwaves * KP);
        const uint32_t c = wcnt[h][w][col];
        uint32_t inc = c;
#pragma unroll
        for (int off = 1; off < nwaves; off <<= 1) {
            const uint32_t o = __shfl_up(inc, off, nwaves);
            if (w >= off) inc += o;
        }
        uint32_t base = 0;
        for (int g = 0; g < h; ++g) base += own[g][col];
        wcnt[h][w][col] = base + inc - c;
    }
}

// ------------------------------------------------------------------------------------------------
// apply for k <= KP (16 or 32): the same admission, one vertex of each of kSmallApplyTiles neighbouring
// tiles per thread, a workgroup of kAdmitTile threads per such group of tiles.  cnt[tile][t] = movers
// to t in that tile, tot[t] >= movers to t in the whole chunk, room[t] = P - S[t] as of the chunk's
// start.  A partition with no room admits nobody, one with room for all its movers admits everybody;
// only for the others (room for some) are ranks needed: the workgroup adds up their columns of the
// earlier tiles' counts and takes one ballot per such partition and tile.
// ------------------------------------------------------------------------------------------------
constexpr int kSmallApplyTiles = 4;     // neighbouring tiles per workgroup of k_apply_small

template <int KP>
__global__ __launch_bounds__(kAdmitTile) void k_apply_small(uint8_t *__restrict__ Lc, const uint8_t *__restrict__ prop,
                                                            int64_t chunk_lo, int64_t chunk_hi, int k,
                                                            const uint32_t *__restrict__ cnt,
                                                            const long long *__restrict__ room,
                                                            const uint32_t *__restrict__ tot,
                                                            unsigned long long *__restrict__ S,
                                                            uint32_t *__restrict__ ocnt, int pass,
                                                            uint8_t *__restrict__ Lc4) {
    static_assert(KP == 16 || KP == 32, "partitions per workgroup table");
    constexpr int nwaves = kAdmitTile / 64;
    constexpr int TPW = kSmallApplyTiles;
    constexpr int SEGS = kAdmitTile / KP;           // threads per column when the earlier tiles are added up
    __shared__ uint32_t tbl[KP];                    // movers in the tiles before the workgroup's
    __shared__ uint32_t wcnt[TPW][nwaves][KP];      // movers per tile and wave, then their exclusive prefix
    __shared__ uint32_t s_own[TPW][KP];             // movers of the workgroup's tiles
    __shared__ int32_t dS[KP];
    __shared__ long long s_room[KP];
    __shared__ uint32_t s_ranked;                   // bit t: partition t has room for some of its movers only
    __shared__ uint32_t s_unassigned[TPW];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int tile0 = TPW * (int)blockIdx.x;
    int64_t v[TPW];
    bool inside[TPW];
    uint32_t t[TPW], old[TPW];
#pragma unroll
    for (int h = 0; h < TPW; ++h) {
        v[h] = chunk_lo + (int64_t)(tile0 + h) * kAdmitTile + tid;
        inside[h] = v[h] < chunk_hi;
        t[h] = 0;
        old[h] = 0;
        if (inside[h]) { t[h] = prop[v[h] - chunk_lo]; old[h] = (uint32_t)Lc[v[h]]; }
    }
    // the earlier tiles' counts, column `col` by SEGS threads: asked for now, together with the labels, when
    // the tiles are few (needed only if the partition turns out to be one with room for some: then the
    // loads' latency is already behind us), else after that is known
    const int col = tid & (KP - 1), seg = tid / KP;
    const bool early = tile0 <= 16 * SEGS;
    uint32_t before = 0;
    if (early && col < k) {
        uint32_t x[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int r = seg + SEGS * u;
            x[u] = r < tile0 ? cnt[(size_t)r * k + col] : 0u;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) before += x[u];
    }
    uint32_t own[TPW];
#pragma unroll
    for (int h = 0; h < TPW; ++h)
        own[h] = (tid < k && chunk_lo + (int64_t)(tile0 + h) * kAdmitTile < chunk_hi) ? cnt[(size_t)(tile0 + h) * k + tid] : 0u;
    if (tid < 64) {
        long long rm = 0;
        bool some = false;
        if (tid < k) {
            rm = room[tid];
            some = rm > 0 && (long long)tot[tid] > rm;
        }
        const unsigned long long m = __ballot(some);
        if (tid < KP) { tbl[tid] = 0; dS[tid] = 0; s_room[tid] = rm; }
        if (tid < TPW) s_unassigned[tid] = 0;
        if (tid == 0) s_ranked = (uint32_t)m;
    }
    __syncthreads();
    const uint32_t ranked = s_ranked;
    bool mover[TPW];
    uint32_t wrank[TPW];
#pragma unroll
    for (int h = 0; h < TPW; ++h) { mover[h] = inside[h] && t[h] != old[h]; wrank[h] = 0; }
    if (ranked) {
        if ((ranked >> col) & 1u) {   // earlier tiles: thread (seg, col) adds up rows seg, seg + SEGS, ...
            uint32_t sum = before;
            if (!early)
                for (int r = seg; r < tile0; r += SEGS) sum += cnt[(size_t)r * k + col];
            if (sum) atomicAdd(&tbl[col], sum);
        }
#pragma unroll
        for (int h = 0; h < TPW; ++h) {
            uint32_t mine = 0;
            for (uint32_t left = ranked; left; left &= left - 1) {
                const uint32_t j = (uint32_t)__ffs(left) - 1u;
                const unsigned long long m = __ballot(mover[h] && t[h] == j);
                if (mover[h] && t[h] == j) wrank[h] = (uint32_t)__popcll(m & lanes_below(lane));
                if ((uint32_t)lane == j) mine = (uint32_t)__popcll(m);
            }
            if (lane < KP) wcnt[h][wave][lane] = mine;
        }
        if (tid < KP)
#pragma unroll
            for (int h = 0; h < TPW; ++h) s_own[h][tid] = own[h];
        __syncthreads();
        wave_counts_to_prefix<KP, TPW>(wcnt, s_own);
        __syncthreads();
    }
#pragma unroll
    for (int h = 0; h < TPW; ++h) {
        bool admitted = false;
        if (mover[h]) {
            const long long rm = s_room[t[h]];
            if ((ranked >> t[h]) & 1u) {
                const long long rank = (long long)tbl[t[h]] + wcnt[h][wave][t[h]] + wrank[h];
                admitted = rank < rm;
            } else {
                admitted = rm > 0;          // room for all of the partition's movers, or for none
            }
        }
        if (admitted) {
            Lc[v[h]] = (uint8_t)t[h];
            atomicAdd(&dS[t[h]], 1);
            if (old[h] != 0xFFu) atomicAdd(&dS[old[h]], -1);
        } else if (pass == 0 && inside[h] && old[h] == 0xFFu) {
            atomicAdd(&s_unassigned[h], 1u);    // rejected new vertex (a new vertex is always a mover)
        }
        if (Lc4) {
            // the tile's labels as they now stand, two per byte (chunk_lo is even: the lanes 2i, 2i + 1
            // hold the vertices 2j, 2j + 1); only meaningful once every vertex has a label
            const uint32_t now = admitted ? t[h] : old[h];
            const uint32_t next = (uint32_t)__shfl_xor((int)now, 1);
            if (!(tid & 1) && inside[h]) Lc4[v[h] >> 1] = (uint8_t)((now & 15u) | (next << 4));
        }
    }
    __syncthreads();
    if (tid < k) {
        const int32_t d = dS[tid];
        if (d != 0) atomicAdd(&S[tid], (unsigned long long)(long long)d);
    }
    if (pass == 0 && tid < TPW && chunk_lo + (int64_t)(tile0 + tid) * kAdmitTile < chunk_hi)
        ocnt[tile0 + tid] = s_unassigned[tid];
}

// Exclusive prefix of `mine` over the threads of a workgroup (every thread calls it): shuffles
// inside the wavefront, then the totals of the earlier wavefronts from `wave_total` (LDS, one slot
// per wavefront, free for reuse after the next barrier).
__device__ __forceinline__ long long block_exclusive_sum(long long mine, long long *wave_total) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    long long inc = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const long long o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    if (lane == 63) wave_total[wave] = inc;
    __syncthreads();
    long long before = inc - mine;
    for (int w = 0; w < wave; ++w) before += wave_total[w];
    return before;
}

// ------------------------------------------------------------------------------------------------
// spill scan (first pass): exclusive prefix of the per-tile unassigned counts, and the level
// tables of "add one to the smallest partition, lowest id on ties, repeatedly":
//   order the partitions by (S, id): s[0] <= s[1] <= ...;  C[a] = sum_{q<a} (s[a] - s[q]) is the
//   number of placements made before the a+1 smallest partitions are level; while the a smallest
//   are level, placements cycle through them in ascending id.
// misc[4] = total to place.  fillRank[j] = position of j in that order, fillC[a] for a = 0..k
// (C[0] = 0, C[k] = infinity).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kScanThreads) void k_spill_scan(uint32_t *__restrict__ ocnt, int ntiles,
                                                             int k, const long long *__restrict__ S,
                                                             int32_t *__restrict__ fillRank,
                                                             long long *__restrict__ fillSorted,
                                                             long long *__restrict__ fillC,
                                                             unsigned long long *__restrict__ misc) {
    __shared__ long long part[kScanThreads / 64];
    __shared__ long long Sl[GREM_MAX_K_DEVICE];
    __shared__ long long s_total;
    const int tid = threadIdx.x;
    {   // prefix over tiles
        const int tps = (ntiles + kScanThreads - 1) / kScanThreads;
        const int tlo = tid * tps;
        const int thi = (tlo + tps < ntiles) ? tlo + tps : ntiles;
        long long sum = 0;
        for (int t = tlo; t < thi; ++t) sum += ocnt[t];
        long long b = block_exclusive_sum(sum, part);
        if (tid == kScanThreads - 1) s_total = b + sum;
        for (int t = tlo; t < thi; ++t) {
            uint32_t c = ocnt[t];
            ocnt[t] = (uint32_t)b;
            b += c;
        }
        __syncthreads();
    }
    const long long total = s_total;
    if (tid == 0) misc[4] = (unsigned long long)total;
    if (total == 0) return;
    for (int j = tid; j < k; j += kScanThreads) Sl[j] = S[j];
    __syncthreads();
    for (int j = tid; j < k; j += kScanThreads) {
        const long long sj = Sl[j];
        int rank = 0;
        for (int i = 0; i < k; ++i) {
            long long si = Sl[i];
            rank += (si < sj || (si == sj && i < j)) ? 1 : 0;
        }
        fillRank[j] = rank;
        fillSorted[rank] = sj;
    }
    __threadfence();
    __syncthreads();
    {   // prefix sums of the sorted sizes -> C
        const int per = (k + kScanThreads - 1) / kScanThreads;
        const int qlo = tid * per;
        const int qhi = (qlo + per < k) ? qlo + per : k;
        long long sum = 0;
        for (int q = qlo; q < qhi; ++q)
            sum += __hip_atomic_load(fillSorted + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        long long ps = block_exclusive_sum(sum, part);
        for (int q = qlo; q < qhi; ++q) {
            long long sq = __hip_atomic_load(fillSorted + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            fillC[q] = (long long)q * sq - ps;     // sum_{p<q} (s[q] - s[p])
            ps += sq;
        }
        if (tid == 0) fillC[k] = 0x7fffffffffffffffLL;
    }
}

// ------------------------------------------------------------------------------------------------
// spill fill (first pass): the i-th unassigned vertex of the chunk (ascending id) takes the i-th
// placement of the level sequence.
// ------------------------------------------------------------------------------------------------
template <typename LabelT>
__global__ __launch_bounds__(kAdmitThreads) void k_spill_fill(
    LabelT *__restrict__ Lc, int64_t chunk_lo, int64_t chunk_hi, int k,
    const uint32_t *__restrict__ obase, const int32_t *__restrict__ fillRank,
    const long long *__restrict__ fillC, unsigned long long *__restrict__ S,
    const unsigned long long *__restrict__ misc) {
    if (misc[4] == 0) return;
    extern __shared__ uint32_t smem[];
    constexpr int nwaves = kAdmitThreads / 64;
    int32_t *dS = (int32_t *)smem;        // k
    __shared__ uint32_t wsum[nwaves];
    __shared__ uint32_t s_run;
    constexpr uint32_t UN = LabelTraits<LabelT>::kUnassigned;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    for (int j = tid; j < k; j += kAdmitThreads) dS[j] = 0;
    if (tid == 0) s_run = 0;
    __syncthreads();
    const int64_t lo = chunk_lo + (int64_t)blockIdx.x * kAdmitTile;
    const long long tile_base = obase[blockIdx.x];
    for (int round = 0; round < kAdmitTile / kAdmitThreads; ++round) {
        const int64_t v = lo + round * kAdmitThreads + tid;
        const bool un = (v < chunk_hi) && ((uint32_t)Lc[v] == UN);
        const unsigned long long m = __ballot(un);
        if (lane == 0) wsum[wave] = (uint32_t)__popcll(m);
        __syncthreads();
        if (un) {
            long long i = tile_base + s_run + __popcll(m & lanes_below(lane));
            for (int w = 0; w < wave; ++w) i += wsum[w];
            // smallest a in [1,k] with i < C[a]
            int lo_a = 1, hi_a = k;
            while (lo_a < hi_a) {
                int mid = (lo_a + hi_a) >> 1;
                if (i < fillC[mid]) hi_a = mid; else lo_a = mid + 1;
            }
            const int a = lo_a;
            const long long off = i - fillC[a - 1];
            int idx = (int)(off % a);
            int j = idx;
            if (a < k) {          // idx-th smallest id among the a smallest partitions
                for (j = 0; j < k - 1; ++j) {
                    if (fillRank[j] < a) { if (idx == 0) break; idx -= 1; }
                }
            }
            Lc[v] = (LabelT)j;
            atomicAdd(&dS[j], 1);
        }
        __syncthreads();
        if (tid == 0) { uint32_t s = 0; for (int w = 0; w < nwaves; ++w) s += wsum[w]; s_run += s; }
        __syncthreads();
    }
    for (int j = tid; j < k; j += kAdmitThreads) {
        int32_t d = dS[j];
        if (d != 0) atomicAdd(&S[j], (unsigned long long)(long long)d);
    }
}

// ------------------------------------------------------------------------------------------------
// The spill of a chunk of few tiles into k <= KP partitions in one launch (k_spill_scan and
// k_spill_fill in one): every workgroup (kSmallApplyTiles tiles, a thread per vertex and tile) adds up the
// tiles' counts of rejected new vertices and builds the level tables for itself.  With nothing to
// place it ends there.  The sizes are read from Sin (as the admission left them) and written, by
// workgroup 0 and in closed form, to another array Sout: partition j, at position pos among the a
// smallest partitions by id, takes len / a + (pos < len % a) of the len placements made while a
// partitions are level.  (The callers alternate between two arrays from chunk to chunk; Sout is
// written in full in every launch.)
// ------------------------------------------------------------------------------------------------
constexpr int kSpillPer = 4;                                   // tiles per thread in the prefix
constexpr int kSpillSmallTiles = kSpillPer * kAdmitTile;       // most tiles of a chunk

template <int KP>
__global__ __launch_bounds__(kAdmitTile) void k_spill_small(uint8_t *__restrict__ Lc, int64_t chunk_lo, int64_t chunk_hi,
                                                            int k, const uint32_t *__restrict__ ocnt, int ntiles,
                                                            const long long *__restrict__ Sin,
                                                            long long *__restrict__ Sout) {
    constexpr int nwaves = kAdmitTile / 64;
    constexpr int TPW = kSmallApplyTiles;
    __shared__ uint32_t wtot[nwaves];
    __shared__ uint32_t s_base[TPW + 1];            // rejected vertices before each of the workgroup's tiles
    __shared__ uint32_t s_total;
    __shared__ long long Sl[KP], sorted[KP], C[KP + 1];
    __shared__ int rnk[KP];
    __shared__ uint32_t wun[TPW][nwaves];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int tile0 = TPW * (int)blockIdx.x;
    // exclusive prefix of the tiles' counts (at most kSpillSmallTiles tiles: thread tid takes the tiles
    // kSpillPer * tid .. kSpillPer * tid + kSpillPer - 1)
    uint32_t part[kSpillPer], mine = 0;
#pragma unroll
    for (int x = 0; x < kSpillPer; ++x) {
        const int tile = kSpillPer * tid + x;
        part[x] = tile < ntiles ? ocnt[tile] : 0u;
        mine += part[x];
    }
    long long sj = 0;
    if (tid < k) sj = Sin[tid];
    uint32_t inc = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    if (lane == 63) wtot[wave] = inc;
    if (tid < k) Sl[tid] = sj;
    __syncthreads();
    uint32_t before = inc - mine;
    for (int w = 0; w < wave; ++w) before += wtot[w];
    {
        uint32_t run = before;
#pragma unroll
        for (int x = 0; x < kSpillPer; ++x) {
            const int tile = kSpillPer * tid + x;
            if (tile >= tile0 && tile < tile0 + TPW) s_base[tile - tile0] = run;
            run += part[x];
        }
    }
    if (tid == kAdmitTile - 1) s_total = before + mine;
    __syncthreads();
    const uint32_t total = s_total;
    if (total == 0) {
        if (blockIdx.x == 0 && tid < k) Sout[tid] = sj;
        return;
    }
    // level tables: order the partitions by (size, id); C[a] = placements made before a + 1 partitions are level
    if (tid < k) {
        int r = 0;
        for (int i = 0; i < k; ++i) r += (Sl[i] < sj || (Sl[i] == sj && i < tid)) ? 1 : 0;
        rnk[tid] = r;
        sorted[r] = sj;
    }
    __syncthreads();
    if (tid <= k) {
        long long ps = 0;
        for (int q = 0; q < tid && q < k; ++q) ps += sorted[q];
        C[tid] = tid < k ? (long long)tid * sorted[tid] - ps : 0x7fffffffffffffffLL;
    }
    __syncthreads();
    // the rejected new vertices of the workgroup's tiles, in ascending id
    bool un[TPW];
    int64_t v[TPW];
#pragma unroll
    for (int h = 0; h < TPW; ++h) {
        v[h] = chunk_lo + (int64_t)(tile0 + h) * kAdmitTile + tid;
        un[h] = v[h] < chunk_hi && Lc[v[h]] == 0xFFu;
    }
    uint32_t within[TPW];
#pragma unroll
    for (int h = 0; h < TPW; ++h) {
        const unsigned long long m = __ballot(un[h]);
        within[h] = (uint32_t)__popcll(m & lanes_below(lane));
        if (lane == 0) wun[h][wave] = (uint32_t)__popcll(m);
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < TPW; ++h) {
        if (!un[h]) continue;
        long long i = (long long)s_base[h] + within[h];
        for (int w = 0; w < wave; ++w) i += wun[h][w];
        int a = 1;
        while (a < k && i >= C[a]) ++a;                 // smallest a in [1, k] with i < C[a]
        int idx = (int)((unsigned long long)(i - C[a - 1]) % (unsigned)a);
        int j = idx;
        if (a < k) {            // the idx-th smallest id among the a smallest partitions
            for (j = 0; j < k - 1; ++j)
                if (rnk[j] < a) { if (idx == 0) break; idx -= 1; }
        }
        Lc[v[h]] = (uint8_t)j;
    }
    if (blockIdx.x == 0 && tid < k) {
        long long add = 0;
        for (int a = 1; a <= k; ++a) {
            const long long hi = C[a] < (long long)total ? C[a] : (long long)total;
            if (C[a - 1] >= (long long)total) break;
            const long long len = hi - C[a - 1];
            if (len <= 0) continue;
            if (rnk[tid] < a) {
                int pos = 0;
                for (int q = 0; q < tid; ++q) pos += rnk[q] < a ? 1 : 0;
                add += len / a + (pos < (int)(len % a) ? 1 : 0);
            }
        }
        Sout[tid] = sj + add;
    }
}

// ------------------------------------------------------------------------------------------------
// expand: compact labels -> int32 output
// ------------------------------------------------------------------------------------------------
template <typename LabelT>
__global__ __launch_bounds__(256) void k_expand(const LabelT *__restrict__ Lc, int64_t n,
                                                int32_t *__restrict__ out) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) {
        uint32_t l = Lc[v];
        out[v] = (l == LabelTraits<LabelT>::kUnassigned) ? -1 : (int32_t)l;
    }
}

// ------------------------------------------------------------------------------------------------
// edge cut: entries whose endpoints carry different labels, one integer sum
// ------------------------------------------------------------------------------------------------
template <typename RowT>
__global__ __launch_bounds__(256) void k_edge_cut(const RowT *__restrict__ rowptr,
                                                  const int32_t *__restrict__ colidx, int64_t n,
                                                  const int32_t *__restrict__ labels,
                                                  unsigned long long *__restrict__ out) {
    constexpr int tv = 256;
    __shared__ unsigned long long rowrel[tv + 1];   // 64-bit: a tile may hold any number of entries
    __shared__ int32_t lab[tv];
    __shared__ unsigned long long s_sum;
    const int tid = threadIdx.x;
    const int64_t v0 = (int64_t)blockIdx.x * tv;
    const int64_t left = n - v0;
    const int nv = left < tv ? (int)left : tv;
    const int64_t e0 = (int64_t)rowptr[v0];
    for (int i = tid; i <= tv; i += 256) {
        int ii = i < nv ? i : nv;
        rowrel[i] = (unsigned long long)((int64_t)rowptr[v0 + ii] - e0);
    }
    if (tid < nv) lab[tid] = labels[v0 + tid];
    if (tid == 0) s_sum = 0;
    __syncthreads();
    const unsigned long long ne = rowrel[tv];
    unsigned long long mine = 0;
    for (unsigned long long i = tid; i < ne; i += 256) {
        int32_t c = __builtin_nontemporal_load(colidx + e0 + i);
        int32_t lu = labels[c];
        int r = 0;
        for (int step = tv >> 1; step >= 1; step >>= 1)
            if (rowrel[r + step] <= i) r += step;
        mine += (lu != lab[r]) ? 1ull : 0ull;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mine += __shfl_xor(mine, off);
    if (lane_id() == 0 && mine) atomicAdd(&s_sum, mine);
    __syncthreads();
    if (tid == 0 && s_sum) atomicAdd(out, s_sum);
}

// The same sum from the vertices' neighbour counts under the labelling (counts[v * k + j] = entries of
// row v whose column has label j; columns without a label are in no count): a labelled vertex differs
// from every neighbour outside its own count, an unlabelled one from every labelled neighbour.
template <typename RowT>
__global__ __launch_bounds__(256) void k_cut_from_counts(const RowT *__restrict__ rowptr,
                                                         const int32_t *__restrict__ labels,
                                                         const uint32_t *__restrict__ counts, int64_t n, int k,
                                                         unsigned long long *__restrict__ out) {
    __shared__ unsigned long long s_sum;
    if (threadIdx.x == 0) s_sum = 0;
    __syncthreads();
    unsigned long long mine = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) {
        const int32_t l = labels[v];
        const uint32_t *row = counts + (size_t)v * (size_t)k;
        if (l >= 0 && l < k) {
            mine += (unsigned long long)(rowptr[v + 1] - rowptr[v]) - (unsigned long long)row[l];
        } else {
            for (int j = 0; j < k; ++j) mine += row[j];
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mine += __shfl_xor(mine, off);
    if (lane_id() == 0 && mine) atomicAdd(&s_sum, mine);
    __syncthreads();
    if (threadIdx.x == 0 && s_sum) atomicAdd(out, s_sum);
}

__global__ void k_zero_u64(unsigned long long *p, int count) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0ull;
}

__global__ void k_copy_sizes(const long long *__restrict__ S, int k, int64_t *__restrict__ out) {
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < k) out[j] = S[j];
}

}  // namespace grem
