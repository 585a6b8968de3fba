// Two-phase score path (k <= 32): the same counts as k_score_lds (Alg. 2 cnt_nbrs, Alg. 1 blend,
// Alg. 2 assign), organised so that every neighbour-label look-up is served from LDS and every
// byte that crosses HBM is part of a long sequential stream.
//
// Why: a look-up into a label table larger than L2 costs one 64-byte fabric request whatever the
// table's size (57 G look-ups/s on MI355X), and even an L2-resident table serves only 267 G/s,
// while LDS serves several thousand G/s.  A label changes only when its vertex's chunk is
// processed, so all look-ups of the labels of one chunk's vertices can be done right after that
// chunk, by workgroups that hold those labels in LDS -- for every row that refers to them, in this
// pass (rows of later chunks) or the next (rows of earlier chunks and of the chunk itself).
//
// How: once per graph the CSR entries are re-laid-out into tuples (row in slice, column in block):
//   * a column block is 2^cb consecutive vertices counted from the start of their chunk;
//   * a row slice is 2048 consecutive rows counted from the start of their chunk;
//   * rows of degree >= hub_degree ("hubs") are taken out of their slice: the chunk's hub entries,
//     concatenated in row order, are cut in equal shares (k_plan_chunks picks how many);
//   * a "row" r of chunk c is slice r (r < nsl) or share r - nsl; there are nr = nsl + (the largest
//     number of shares of any chunk) rows per chunk;
//   * sub-segment (c, r, jb) holds the tuples of row r of chunk c whose column lies in block jb,
//     padded to a multiple of 8 tuples.
// A tuple lives in three streams, each with as few bytes as its reader needs:
//   T  : its column in the block, 20 bits, and per group of eight tuples the place of their labels in
//        Lx (24 bytes per group); sub-segments ordered (jb, c, r): all tuples that refer to one
//        column block are contiguous                                   -- read by k_tp_lookup
//   Lx : the label of that column, 4 bits (8 when k > 16); sub-segments ordered (c, r, jb): all tuples of one row
//        slice are contiguous                    -- written by k_tp_lookup, read by k_tp_score
//   R  : its row in the slice << 5, 16 bits (bit 0 = padding), ordered like Lx; written once by the
//        re-layout, read by k_tp_score (row << 5 is the byte offset of the row's 16-bit counters)
// After chunk c has been relabelled, k_tp_lookup streams the columns of c's column blocks
// (contiguous in T), looks the labels up in an LDS copy of the block's labels (two per byte) and
// writes them to Lx, sub-segment by sub-segment (each a contiguous piece of some 40 bytes).  Before
// chunk c is relabelled, k_tp_score has one workgroup per row slice stream that slice's tuples -- one
// contiguous piece of R and of Lx -- into 16-bit LDS counters, then blends E and proposes.  (Seeded
// runs: in their first pass a neighbour may be unassigned; the score kernel then reads the row
// fields from a copy of R in which bit 0 marks such tuples.)
//
// Balance: every workgroup of k_tp_score also counts an equal part of one hub share's stream (32-bit
// counters per hub the share touches) and adds its partial counts to a per-chunk table in global
// memory with integer atomics; k_hub_finalize then blends and proposes for the hubs.  The order of
// entries inside a sub-segment and the order of the atomic adds are arbitrary; all of it is integer
// sums, so the result is not.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "grem_kernels.hip.h"

namespace grem {

constexpr int kSliceRowBits = 11;
constexpr int kSliceRows = 1 << kSliceRowBits;     // rows per slice (row index << 5 fits the 16 bits of R)
constexpr int kPlanThreads = 256;
constexpr int kPlanParts = kSliceRows / kPlanThreads;     // finest cut of a slice the re-layout uses
constexpr int kTpThreads = 1024;                   // k_tp_lookup and k_tp_score
constexpr int kMaxBlocks = 4096;                   // column blocks (LDS tables in the re-layout kernels)
constexpr int kMaxShareHubs = 2048;                // hubs one share may touch (index fits the row field)
constexpr int kMaxColBits = 18;                    // 2^18 labels, two per byte: 128 KB of LDS

typedef unsigned long long u64;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x3a __attribute__((ext_vector_type(3), aligned(4)));     // 12 bytes at any 4-byte boundary

struct SweepPlan {
    // per slice (global slice index gs = chunk * nsl + i)
    uint32_t *sl_reg_cnt;     // regular (non-hub) entries
    u64 *sl_reg_start;        // their start, relative to the chunk's first entry
    uint32_t *sl_nh;          // hubs in the slice
    uint32_t *sl_hub_start;   // index of the slice's first hub in the chunk's hub list
    u64 *sl_hent;             // hub entries in the slice
    u64 *sl_hent_start;       // their start in the chunk's hub entry stream
    uint32_t *sl_part_reg0;   // [kPlanParts per slice] regular entries of the slice's rows before row 256 * p
    uint32_t *share_h0;       // first hub touched by share gs
    uint32_t *share_nhs;      // hubs touched by share gs
    // per chunk
    u64 *ch_regtot;           // regular entries
    uint32_t *ch_nh;          // hubs
    u64 *ch_H;                // hub entries
    uint32_t *ch_nvs;         // hub shares of the chunk (0 without hubs, else 1 .. its number of slices)
    u64 *ch_hbase;            // start of the chunk's hub entry stream in the stream of all chunks (+1: total)
    u64 *ch_reg0;             // regular entries of the chunks before it (+1: total)
    u64 *ch_hub0;             // hubs of the chunks before it (+1: total)
    // hub lists: chunk c's hubs at hub_row[ch_hub0[c] + i]; prefix of their degrees at
    // hub_off[ch_hub0[c] + c + i], i = 0..nh (one more slot per chunk)
    int32_t *hub_row;
    u64 *hub_off;
};

// Geometry and offset tables of the re-laid-out entries.  A sub-segment's length is its tuple count
// rounded up to a multiple of kSubPad.
constexpr uint32_t kSubPad = 8;

struct TpTables {
    uint32_t *cnt;    // [nch][nr][nblk]: tuples of sub-segment (c, r, jb) (re-layout only)
    uint32_t *ta;     // [nblk][nch][nr + 1]: start of sub-segment (c, r, jb) inside segment (jb, c) of T;
                      // entry nr: the segment's length
    uint32_t *dd;     // [nblk][nch][nr]: start of sub-segment (c, r, jb) inside row stream (c, r) of Lx / R
    u64 *tstart;      // [nblk][nch] (+1): first slot of segment (jb, c) in T
    u64 *sstart;      // [nch][nr] (+1): first slot of row stream (c, r) in Lx and R
    uint32_t *lo;     // [nch * nsl * npr][ngroups + 1]: start of block group g's run inside the unit's range of U
    uint32_t *loh;    // [nch * nsl * nps][ngroups + 1]: the same for the parts of the hub shares
    u64 *ustart;      // [nch * nsl * npr]: first tuple of a slice part's range of U (regular entries, compacted)
    u64 *ustart_h;    // [nch * nsl * nps]: the same for the parts of the hub shares (after all regular entries)
    int npr;          // parts per slice (a power of two: equal row ranges)
    int nps;          // parts per hub share (equal ranges of its entries)
    int gb;           // log2 of the column blocks per group of the intermediate copy U
    int ngroups;      // ceil(nblk / 2^gb)
    uint32_t chunk;   // rows per chunk (already clamped to n)
    int chunk_shift;  // log2(chunk) when it is a power of two, else -1
    uint32_t chunk_magic, chunk_magic_shift;   // u / chunk = mulhi(u, magic) >> shift for every u < 2^31
    int nch;          // chunks
    int nsl;          // row slices per chunk
    int nr;           // rows (slices, then hub shares) per chunk
    int nbc;          // column blocks per chunk
    int nblk;         // nch * nbc
    int cb;           // log2 of the vertices per column block
    int flat;         // chunk is a power of two and at least a block: block of vertex u = u >> cb
};

__device__ __forceinline__ uint32_t tp_block_of(uint32_t u, const TpTables &g, uint32_t *col_low) {
    if (g.flat) {                       // chunks are whole numbers of blocks: the blocks tile the vertex ids
        *col_low = u & ((1u << g.cb) - 1u);
        return u >> g.cb;
    }
    const uint32_t cu = g.chunk_shift >= 0 ? (u >> g.chunk_shift) : (__umulhi(u, g.chunk_magic) >> g.chunk_magic_shift);
    const uint32_t rel = u - cu * g.chunk;
    *col_low = rel & ((1u << g.cb) - 1u);
    return cu * (uint32_t)g.nbc + (rel >> g.cb);
}

// exclusive prefix over the workgroup (256 threads) of (a, b); totals returned through ta, tb
__device__ __forceinline__ void block_scan2(uint32_t a, u64 b, uint32_t *ea, u64 *eb, uint32_t *ta,
                                            u64 *tb, uint32_t *s_a, u64 *s_b) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    uint32_t ia = a;
    u64 ib = b;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t oa = __shfl_up(ia, off);
        u64 ob = __shfl_up(ib, off);
        if (lane >= off) { ia += oa; ib += ob; }
    }
    __syncthreads();                      // s_a / s_b free for reuse
    if (lane == 63) { s_a[wave] = ia; s_b[wave] = ib; }
    __syncthreads();
    uint32_t ba = 0, tta = 0;
    u64 bb = 0, ttb = 0;
    for (int w = 0; w < kPlanThreads / 64; ++w) {
        if (w < wave) { ba += s_a[w]; bb += s_b[w]; }
        tta += s_a[w];
        ttb += s_b[w];
    }
    *ea = ba + ia - a;
    *eb = bb + ib - b;
    *ta = tta;
    *tb = ttb;
}

// ------------------------------------------------------------------------------------------------
// plan 1: per slice, regular entries, hubs, hub entries; misc[0] = the graph's largest degree,
// misc[3] = its number of entries
// ------------------------------------------------------------------------------------------------
template <typename RowT>
__global__ __launch_bounds__(256) void k_plan_slices(const RowT *__restrict__ rowptr, int64_t n,
                                                     int64_t chunk, int nsl, uint32_t hub_degree,
                                                     SweepPlan pl, u64 *__restrict__ misc) {
    __shared__ u64 s_reg, s_hent, s_maxdeg;
    __shared__ uint32_t s_nh, s_part[kPlanParts];
    const int tid = threadIdx.x;
    const int64_t c = blockIdx.x / nsl;
    const int i = blockIdx.x % nsl;
    const int64_t chunk_lo = c * chunk;
    const int64_t chunk_hi = (chunk_lo + chunk < n) ? chunk_lo + chunk : n;
    const int64_t v0 = chunk_lo + (int64_t)i * kSliceRows;
    if (tid == 0) { s_reg = 0; s_hent = 0; s_nh = 0; s_maxdeg = 0; }
    if (tid < kPlanParts) s_part[tid] = 0;
    __syncthreads();
    u64 reg = 0, hent = 0, maxdeg = 0;
    uint32_t nh = 0;
#pragma unroll
    for (int p = 0; p < kPlanParts; ++p) {          // rows 256 p .. 256 p + 255: one per thread
        const int64_t v = v0 + p * kPlanThreads + tid;
        uint32_t regp = 0;
        if (v < chunk_hi) {
            const u64 d = (u64)(rowptr[v + 1] - rowptr[v]);
            if (d >= hub_degree) { nh += 1; hent += d; } else { reg += d; regp = (uint32_t)d; }
            maxdeg = d > maxdeg ? d : maxdeg;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) regp += __shfl_xor(regp, off);
        if (lane_id() == 0 && regp) atomicAdd(&s_part[p], regp);
    }
    if (reg) atomicAdd(&s_reg, reg);
    if (nh) { atomicAdd(&s_hent, hent); atomicAdd(&s_nh, nh); }
    // (wavefront maximum first: one LDS atomic per wavefront)
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { const u64 o = __shfl_xor(maxdeg, off); maxdeg = o > maxdeg ? o : maxdeg; }
    if (lane_id() == 0 && maxdeg) atomicMax(&s_maxdeg, maxdeg);
    __syncthreads();
    if (tid == 0) {
        pl.sl_reg_cnt[blockIdx.x] = (uint32_t)s_reg;
        pl.sl_nh[blockIdx.x] = s_nh;
        pl.sl_hent[blockIdx.x] = s_hent;
        uint32_t run = 0;
        for (int p = 0; p < kPlanParts; ++p) { pl.sl_part_reg0[(size_t)blockIdx.x * kPlanParts + p] = run; run += s_part[p]; }
        // (few workgroups raise the maximum: the plain read spares the others the atomic)
        if (s_maxdeg > __hip_atomic_load(&misc[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(&misc[0], s_maxdeg);
        if (blockIdx.x == 0) misc[3] = (u64)rowptr[n];
    }
}

// ------------------------------------------------------------------------------------------------
// plan 2: per chunk, exclusive prefixes over its slices, and the number of hub shares: enough
// shares that one touches at most about hubs_per_share hubs, few enough that a share's sub-segment of a
// column block still holds some 64 entries, at most one per slice.  misc[6] = most hubs in a
// chunk, misc[7] = most entries in a chunk, misc[9] = most regular entries in a slice (set here
// from the slices' counts), misc[10] = most entries in a hub share, misc[11] = most hub shares in a
// chunk, misc[8] = hub entries of all chunks, misc[12] = hubs of all chunks.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_plan_chunks(int64_t n, int64_t chunk, int nsl, int nblk,
                                                     uint32_t hubs_per_share, SweepPlan pl, u64 *__restrict__ misc) {
    __shared__ u64 p_reg[256], p_hent[256];
    __shared__ uint32_t p_nh[256];
    const int tid = threadIdx.x;
    const int64_t c = blockIdx.x;
    const int64_t chunk_lo = c * chunk;
    const size_t g0 = (size_t)c * nsl;
    const int per = (nsl + 255) / 256;
    const int q0 = tid * per;
    const int q1 = (q0 + per < nsl) ? q0 + per : nsl;
    u64 reg = 0, hent = 0;
    uint32_t nh = 0;
    u64 maxreg = 0;
    for (int q = q0; q < q1; ++q) {
        const u64 rq = pl.sl_reg_cnt[g0 + q];
        reg += rq;
        maxreg = rq > maxreg ? rq : maxreg;
        nh += pl.sl_nh[g0 + q];
        hent += pl.sl_hent[g0 + q];
    }
    if (maxreg) atomicMax(&misc[9], maxreg);
    p_reg[tid] = reg; p_nh[tid] = nh; p_hent[tid] = hent;
    __syncthreads();
    u64 breg = 0, bhent = 0;
    uint32_t bnh = 0;
    for (int s = 0; s < tid; ++s) { breg += p_reg[s]; bnh += p_nh[s]; bhent += p_hent[s]; }
    for (int q = q0; q < q1; ++q) {
        pl.sl_reg_start[g0 + q] = breg;
        pl.sl_hub_start[g0 + q] = bnh;
        pl.sl_hent_start[g0 + q] = bhent;
        breg += pl.sl_reg_cnt[g0 + q];
        bnh += pl.sl_nh[g0 + q];
        bhent += pl.sl_hent[g0 + q];
    }
    if (tid == 255) {        // the last thread's running totals are the chunk's totals
        pl.ch_regtot[c] = breg;
        pl.ch_nh[c] = bnh;
        pl.ch_H[c] = bhent;
        pl.ch_hbase[c] = bhent;             // these three: scanned over the chunks by k_tp_scan
        pl.ch_reg0[c] = breg;
        pl.ch_hub0[c] = (u64)bnh;
        const int64_t chunk_hi = (chunk_lo + chunk < n) ? chunk_lo + chunk : n;
        const u64 nsl_c = (u64)((chunk_hi - chunk_lo + kSliceRows - 1) / kSliceRows);
        u64 nvs = 0;
        if (bnh != 0) {
            nvs = bhent / (64ull * (u64)nblk);
            const u64 by_hubs = ((u64)bnh + hubs_per_share - 1ull) / (u64)hubs_per_share;
            if (nvs < by_hubs) nvs = by_hubs;
            if (nvs < 1) nvs = 1;
            if (nvs > nsl_c) nvs = nsl_c;
        }
        pl.ch_nvs[c] = (uint32_t)nvs;
        atomicMax(&misc[6], (u64)bnh);
        atomicMax(&misc[7], breg + bhent);
        if (nvs) atomicMax(&misc[10], bhent / nvs + 1);
        if (nvs) atomicMax(&misc[11], nvs);
        atomicAdd(&misc[8], bhent);
        atomicAdd(&misc[12], (u64)bnh);
    }
}

// ------------------------------------------------------------------------------------------------
// plan 3: per slice, its hubs in row order into the chunk's hub list, with the prefix of degrees
// ------------------------------------------------------------------------------------------------
template <typename RowT>
__global__ __launch_bounds__(256) void k_plan_hubs(const RowT *__restrict__ rowptr, int64_t n,
                                                   int64_t chunk, int nsl, uint32_t hub_degree,
                                                   SweepPlan pl) {
    __shared__ uint32_t s_a[4];
    __shared__ u64 s_b[4];
    const int tid = threadIdx.x;
    const int64_t c = blockIdx.x / nsl;
    const int i = blockIdx.x % nsl;
    const u64 hub0 = pl.ch_hub0[c];
    if (i == 0 && tid == 0) pl.hub_off[hub0 + (u64)c + pl.ch_nh[c]] = pl.ch_H[c];     // the list's closing offset
    if (pl.sl_nh[blockIdx.x] == 0) return;
    const int64_t chunk_lo = c * chunk;
    const int64_t chunk_hi = (chunk_lo + chunk < n) ? chunk_lo + chunk : n;
    const int64_t v0 = chunk_lo + (int64_t)i * kSliceRows;
    uint32_t run_nh = pl.sl_hub_start[blockIdx.x];
    u64 run_ent = pl.sl_hent_start[blockIdx.x];
    for (int base = 0; base < kSliceRows; base += 256) {      // same trip count for every thread
        const int64_t v = v0 + base + tid;
        u64 d = 0;
        if (v < chunk_hi) d = (u64)(rowptr[v + 1] - rowptr[v]);
        const bool hub = v < chunk_hi && d >= hub_degree;
        uint32_t ea, ta;
        u64 eb, tb;
        block_scan2(hub ? 1u : 0u, hub ? d : 0ull, &ea, &eb, &ta, &tb, s_a, s_b);
        if (hub) {
            pl.hub_row[hub0 + run_nh + ea] = (int32_t)v;
            pl.hub_off[hub0 + (u64)c + run_nh + ea] = run_ent + eb;
        }
        run_nh += ta;
        run_ent += tb;
    }
}

// ------------------------------------------------------------------------------------------------
// plan 4: per share, the hubs it touches.  Share i of a chunk with NS shares and H hub entries is
// [H*i/NS, H*(i+1)/NS) of the chunk's hub entry stream.  misc[5] = most hubs touched by one share.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_plan_shares(int64_t n, int64_t chunk, int nsl, int total_slices,
                                                     SweepPlan pl, u64 *__restrict__ misc) {
    const int gs = blockIdx.x * blockDim.x + threadIdx.x;
    if (gs >= total_slices) return;
    const int64_t c = gs / nsl;
    const int i = gs % nsl;
    const int64_t chunk_lo = c * chunk;
    const int64_t chunk_hi = (chunk_lo + chunk < n) ? chunk_lo + chunk : n;
    uint32_t h0 = 0, nhs = 0;
    const u64 NS = (u64)pl.ch_nvs[c];
    if ((u64)i < NS && chunk_lo < chunk_hi) {
        const u64 H = pl.ch_H[c];
        const u64 a = H * (u64)i / NS, b = H * (u64)(i + 1) / NS;
        if (a != b) {
            const uint32_t nh = pl.ch_nh[c];
            const u64 *goff = pl.hub_off + pl.ch_hub0[c] + (u64)c;        // nh + 1 entries, goff[nh] = H
            uint32_t lo = 0, hi = nh;                           // largest idx with goff[idx] <= a
            while (hi - lo > 1) { uint32_t mid = (lo + hi) >> 1; if (goff[mid] <= a) lo = mid; else hi = mid; }
            h0 = lo;
            hi = nh;                                            // largest idx with goff[idx] < b
            while (hi - lo > 1) { uint32_t mid = (lo + hi) >> 1; if (goff[mid] < b) lo = mid; else hi = mid; }
            nhs = lo - h0 + 1;
            atomicMax(&misc[5], (u64)nhs);
        }
    }
    pl.share_h0[gs] = h0;
    pl.share_nhs[gs] = nhs;
}

// The re-layout works on UNITS: part q of the `npr` equal row ranges of a slice (SHARE = false), or
// part q of the `nps` equal ranges of a hub share's piece of the chunk's hub entry stream
// (SHARE = true).  A unit's entries are contiguous in the CSR (or in the stream), and few enough
// that its tuples fit in LDS.  tp_load_round hands them to the workgroup's threads: (row field,
// column) for each, the row field being the row's index in the slice, or the hub's index among
// the hubs the share touches.
//   regular: rowrel[rp + 1] in LDS (rp rows per part, a power of two), entries colidx[e0 ..);
//            rows of degree >= hub_degree are skipped
//   share  : stream positions [a, a + len); hoff[nhs + 1] / hrow[nhs] in LDS
struct TpEntrySource {
    const int32_t *colidx;
    // regular
    const uint32_t *rowrel;
    int64_t e0;
    uint32_t ne, hub_degree, row0;
    int rp;
    bool has_hubs;
    // share
    const u64 *hoff, *hrow;
    u64 a;
    uint32_t len, nhs;
};

constexpr int kTpBatch = 8;      // entries per thread and round

// The workgroup visits the unit's entries in rounds of kTpThreads * kTpBatch; tp_load_round gives a
// thread its kTpBatch entries of a round (row field, column, on[u] = false: no entry), all loads and
// searches side by side so that their latencies overlap.
template <bool SHARE>
__device__ __forceinline__ uint32_t tp_rounds(const TpEntrySource &src) {
    const uint32_t ne = SHARE ? src.len : src.ne;
    return (ne + kTpThreads * kTpBatch - 1) / (kTpThreads * kTpBatch);
}

template <bool SHARE>
__device__ __forceinline__ void tp_load_round(const TpEntrySource &src, uint32_t round, uint32_t (&row)[kTpBatch],
                                              uint32_t (&col)[kTpBatch], bool (&on)[kTpBatch]) {
    constexpr int U = kTpBatch;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    constexpr int NW = kTpThreads / 64;
    if (!SHARE) {
        // a wavefront takes 64 * U consecutive entries: their rows span a short range, found once (two
        // searches side by side), inside which every lane then looks for its own (U searches side by
        // side, the same number of steps for all)
        const int32_t *cbase = src.colidx + src.e0;
        const uint32_t blk = (round * NW + (uint32_t)wave) * 64u * U;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t p = blk + u * 64 + lane;
            on[u] = p < src.ne;
            col[u] = on[u] ? (uint32_t)__builtin_nontemporal_load(cbase + p) : 0u;
            row[u] = 0;
        }
        if (blk >= src.ne) return;
        // The row of an entry p is the largest r with rowrel[r] <= p (empty rows resolve to the last of equal
        // offsets, the one that holds p).  Lane u < U finds it for the first entry of the wavefront's u-th
        // run of 64 entries (a binary search each, side by side); every lane then walks on from there: 64
        // consecutive entries seldom span more than two or three rows.
        uint32_t first_row = 0;
        {
            const uint32_t target = blk + 64u * (uint32_t)(lane < U ? lane : 0);
            const uint32_t tc = target < src.ne ? target : src.ne - 1u;
            for (int step = src.rp >> 1; step >= 1; step >>= 1)
                if (src.rowrel[first_row + step] <= tc) first_row += step;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            row[u] = (uint32_t)__builtin_amdgcn_readlane((int)first_row, u);
            if (on[u]) {
                const uint32_t p = blk + u * 64 + lane;
                while (src.rowrel[row[u] + 1] <= p) ++row[u];
            }
        }
        if (src.has_hubs) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (src.rowrel[row[u] + 1] - src.rowrel[row[u]] >= src.hub_degree) on[u] = false;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) row[u] += src.row0;
    } else {
        // a wavefront takes 64 * U consecutive positions of the hub entry stream: the hub of the first is
        // found once, the others' hubs lie a step or two further on (hubs are long rows)
        const uint32_t blk = (round * NW + (uint32_t)wave) * 64u * U;
#pragma unroll
        for (int u = 0; u < U; ++u) { on[u] = false; col[u] = 0; row[u] = 0; }
        if (blk >= src.len) return;
        uint32_t first = 0, hi = src.nhs;
        {
            const u64 e = src.a + blk;
            while (hi - first > 1) { const uint32_t mid = (first + hi) >> 1; if (src.hoff[mid] <= e) first = mid; else hi = mid; }
        }
        const u64 next = src.hoff[first + 1];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t p = blk + u * 64 + lane;
            on[u] = p < src.len;
            if (on[u]) {
                const u64 e = src.a + p;                     // position in the chunk's hub entry stream
                uint32_t h = first;
                if (e >= next) {
                    h = first + 1;
                    while (src.hoff[h + 1] <= e) ++h;        // hoff[nhs] is beyond the share's last entry
                }
                row[u] = h;
                col[u] = (uint32_t)__builtin_nontemporal_load(src.colidx + (int64_t)(src.hrow[h] + (e - src.hoff[h])));
            }
        }
    }
}

// Sets up the entry source of part q (of np) of slice or share (c, i) in LDS (`lds` must hold
// kSliceRows / np + 1 u32 for a slice, or 2 * share_hubs + 1 u64 for a share); false if the unit
// has no rows / does not exist.  Ends with a barrier when it returns true.
template <typename RowT, bool SHARE>
__device__ __forceinline__ bool tp_entry_source(const RowT *__restrict__ rowptr,
                                                const int32_t *__restrict__ colidx, int64_t n,
                                                uint32_t hub_degree, const SweepPlan &pl, const TpTables &tb,
                                                int64_t c, int i, int q, int np, int share_hubs, void *lds,
                                                TpEntrySource *src) {
    const int tid = threadIdx.x;
    const int64_t chunk_lo = c * (int64_t)tb.chunk;
    const int64_t chunk_hi = (chunk_lo + tb.chunk < n) ? chunk_lo + tb.chunk : n;
    const size_t gs = (size_t)c * tb.nsl + i;
    src->colidx = colidx;
    if (!SHARE) {
        const int rp = kSliceRows / np;
        const int64_t v0 = chunk_lo + (int64_t)i * kSliceRows + (int64_t)q * rp;
        if (v0 >= chunk_hi) return false;                       // part beyond the (ragged) chunk
        uint32_t *rowrel = reinterpret_cast<uint32_t *>(lds);
        const int64_t left = chunk_hi - v0;
        const int nv = left < rp ? (int)left : rp;
        const int64_t e0 = (int64_t)rowptr[v0];
        for (int t = tid; t <= rp; t += kTpThreads) {
            const int tt = t < nv ? t : nv;
            rowrel[t] = (uint32_t)((int64_t)rowptr[v0 + tt] - e0);
        }
        __syncthreads();
        src->rowrel = rowrel;
        src->e0 = e0;
        src->ne = rowrel[rp];
        src->hub_degree = hub_degree;
        src->row0 = (uint32_t)(q * rp);
        src->rp = rp;
        src->has_hubs = pl.sl_nh[gs] != 0;
        return true;
    } else {
        const uint32_t nvs = pl.ch_nvs[c];
        const uint32_t h0 = pl.share_h0[gs], nhs = pl.share_nhs[gs];
        if ((uint32_t)i >= nvs || nhs == 0 || nhs > (uint32_t)share_hubs) return false;
        u64 *hoff = reinterpret_cast<u64 *>(lds);                // nhs + 1  stream offsets of the hubs
        u64 *hrow = hoff + share_hubs + 1;                       // nhs      rowptr of the hub
        const u64 H = pl.ch_H[c];
        const u64 a = H * (u64)i / nvs, b = H * (u64)(i + 1) / nvs;
        const u64 pa = a + (b - a) * (u64)q / (u64)np, pb = a + (b - a) * (u64)(q + 1) / (u64)np;
        const u64 hub0 = pl.ch_hub0[c];
        const u64 *goff = pl.hub_off + hub0 + (u64)c;
        for (uint32_t t = tid; t <= nhs; t += kTpThreads) hoff[t] = goff[h0 + t];
        for (uint32_t t = tid; t < nhs; t += kTpThreads) hrow[t] = (u64)rowptr[pl.hub_row[hub0 + h0 + t]];
        __syncthreads();
        src->hoff = hoff;
        src->hrow = hrow;
        src->a = pa;
        src->len = (uint32_t)(pb - pa);
        src->nhs = nhs;
        return true;
    }
}

// u32 words of LDS the entry source takes (even, so that what follows is 8-byte aligned)
__device__ __host__ inline size_t tp_source_words(bool share, int np, int share_hubs) {
    return share ? 2 * ((size_t)2 * share_hubs + 1) : (((size_t)kSliceRows / np + 2) & ~(size_t)1);
}

// ------------------------------------------------------------------------------------------------
// Re-layout, step 1 (one unit per workgroup, blockIdx.x = (c * per_chunk + i) * np + q, per_chunk
// being nsl for slices and the largest number of shares of a chunk for shares): count the unit's
// entries per column block (added to cnt[c][row][*], which starts at zero), and copy its tuples, grouped by column-block GROUP (2^gb consecutive
// blocks), to the unit's own range of U: first the regular entries of all rows in CSR order (the
// hub rows' entries left out), then, from `hub_base` on, the chunks' hub entry streams.  The range
// starts at ustart[unit]; run g of the unit starts at lo[unit][g] inside it.  The tuples are collected
// in LDS and written as one contiguous piece (a lane-by-lane scatter would cost one L2 request per
// tuple); a unit with more than `cap` tuples writes them one by one instead.
// U tuple: row field << (cb + gb) | block in group << cb | column in block.
// LDS: the entry source's tables, cntf[nblk], cg[ngroups + 1], wtot[kTpThreads / 64], stage[cap]
// ------------------------------------------------------------------------------------------------
template <typename RowT, bool SHARE>
__global__ __launch_bounds__(kTpThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_tp_group(const RowT *__restrict__ rowptr,
                                                         const int32_t *__restrict__ colidx, int64_t n,
                                                         uint32_t hub_degree, SweepPlan pl, TpTables tb,
                                                         int share_hubs, uint32_t cap, int per_chunk,
                                                         uint32_t *__restrict__ U, u64 hub_base) {
    extern __shared__ u64 smem64[];
    const int np = SHARE ? tb.nps : tb.npr;
    uint32_t *cntf = reinterpret_cast<uint32_t *>(smem64) + tp_source_words(SHARE, np, share_hubs);   // nblk
    uint32_t *cg = cntf + tb.nblk;              // ngroups + 1: starts of the groups' runs
    uint32_t *wtot = cg + tb.ngroups + 1;       // kTpThreads / 64: scratch of the prefix sum
    uint32_t *stage = wtot + kTpThreads / 64;   // cap
    const int tid = threadIdx.x;
    const unsigned gs = blockIdx.x / (unsigned)np;
    const int q = (int)(blockIdx.x % (unsigned)np);
    const int64_t c = gs / (unsigned)per_chunk;
    const int i = gs % (unsigned)per_chunk;
    const size_t unit = ((size_t)c * tb.nsl + i) * np + q;
    uint32_t *lo_out = (SHARE ? tb.loh : tb.lo) + unit * (tb.ngroups + 1);
    u64 *ustart_out = (SHARE ? tb.ustart_h : tb.ustart) + unit;
    TpEntrySource src;
    // where the unit's range of U starts: requested now, needed after the counting phase
    const size_t gs_unit = (size_t)c * tb.nsl + i;
    const u64 range0 = SHARE ? pl.ch_hbase[c]
                             : pl.ch_reg0[c] + pl.sl_reg_start[gs_unit] +
                                   pl.sl_part_reg0[gs_unit * kPlanParts + (size_t)q * (kPlanParts / np)];
    for (int j = tid; j < tb.nblk; j += kTpThreads) cntf[j] = 0;    // the source's closing barrier covers this too
    if (!tp_entry_source<RowT, SHARE>(rowptr, colidx, n, hub_degree, pl, tb, c, i, q, np, share_hubs, smem64,
                                      &src)) {
        for (int j = tid; j <= tb.ngroups; j += kTpThreads) lo_out[j] = 0;
        if (tid == 0) *ustart_out = 0;
        return;
    }
    // where the unit's tuples go
    const u64 ustart = SHARE ? hub_base + range0 + src.a : range0;
    if (tid == 0) *ustart_out = ustart;
    // a unit of one round (the usual case) keeps its entries in registers between the two phases
    const uint32_t rounds = tp_rounds<SHARE>(src);
    uint32_t row[kTpBatch], col[kTpBatch];
    bool on[kTpBatch];
    // (col[u] becomes block << kMaxColBits | column in block: the second phase does not work it out again)
    for (uint32_t r = 0; r < rounds; ++r) {
        tp_load_round<SHARE>(src, r, row, col, on);
#pragma unroll
        for (int u = 0; u < kTpBatch; ++u) {
            uint32_t low;
            const uint32_t jb = tp_block_of(col[u], tb, &low);
            col[u] = (jb << kMaxColBits) | low;
            if (on[u]) atomicAdd(&cntf[jb], 1u);
        }
    }
    __syncthreads();
    // counts -> starts (cntf becomes the blocks' cursors: inside a group's run the tuples end up
    // ordered by block, and neighbouring threads seldom meet on a cursor); a thread takes
    // kMaxBlocks / kTpThreads consecutive blocks
    {
        constexpr int kPer = kMaxBlocks / kTpThreads;
        const int lane = lane_id(), wave = tid >> 6;
        uint32_t *row_out = tb.cnt + ((size_t)c * tb.nr + (SHARE ? tb.nsl + i : i)) * tb.nblk;
        uint32_t mine[kPer], sum = 0;
#pragma unroll
        for (int x = 0; x < kPer; ++x) {
            const int j = tid * kPer + x;
            mine[x] = j < tb.nblk ? cntf[j] : 0u;
            if (mine[x]) atomicAdd(&row_out[j], mine[x]);
            sum += mine[x];
        }
        uint32_t inc = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = __shfl_up(inc, off);
            if (lane >= off) inc += o;
        }
        if (lane == 63) wtot[wave] = inc;
        __syncthreads();
        uint32_t run = inc - sum;
        for (int w = 0; w < wave; ++w) run += wtot[w];
        const uint32_t gmask0 = (1u << tb.gb) - 1u;
#pragma unroll
        for (int x = 0; x < kPer; ++x) {
            const int j = tid * kPer + x;
            if (j < tb.nblk) {
                cntf[j] = run;
                if (((uint32_t)j & gmask0) == 0) cg[j >> tb.gb] = run;
            }
            run += mine[x];
        }
        if (tid == kTpThreads - 1) cg[tb.ngroups] = run;
    }
    __syncthreads();
    for (int gq = tid; gq <= tb.ngroups; gq += kTpThreads) lo_out[gq] = cg[gq];
    const uint32_t total = cg[tb.ngroups];
    const bool staged = total <= cap;
    const uint32_t gmask = (1u << tb.gb) - 1u;
    uint32_t *ubase = U + ustart;
    for (uint32_t r = 0; r < rounds; ++r) {
        if (rounds > 1) {
            tp_load_round<SHARE>(src, r, row, col, on);
#pragma unroll
            for (int u = 0; u < kTpBatch; ++u) {
                uint32_t low;
                const uint32_t jb = tp_block_of(col[u], tb, &low);
                col[u] = (jb << kMaxColBits) | low;
            }
        }
        uint32_t w[kTpBatch], tuple[kTpBatch];
#pragma unroll
        for (int u = 0; u < kTpBatch; ++u) {
            const uint32_t jb = col[u] >> kMaxColBits, low = col[u] & ((1u << kMaxColBits) - 1u);
            tuple[u] = (row[u] << (tb.cb + tb.gb)) | ((jb & gmask) << tb.cb) | low;
            w[u] = on[u] ? atomicAdd(&cntf[jb], 1u) : 0u;
        }
#pragma unroll
        for (int u = 0; u < kTpBatch; ++u) {
            if (on[u]) {
                if (staged) stage[w[u]] = tuple[u];
                else ubase[w[u]] = tuple[u];
            }
        }
    }
    if (!staged) return;
    __syncthreads();
    for (uint32_t z = tid; z < total; z += kTpThreads) __builtin_nontemporal_store(stage[z], ubase + z);
}

// ------------------------------------------------------------------------------------------------
// counts -> starts, T side.  One thread per segment (jb, c): exclusive prefix over the chunk's rows of
// the padded counts -> ta[jb][c][0 .. nr]; the segment's length also goes to tstart[jb][c], to be
// scanned by k_tp_scan.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_tp_scan_t(TpTables tb) {
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (int64_t)tb.nch * tb.nblk) return;
    const int c = (int)(id / tb.nblk), jb = (int)(id % tb.nblk);
    const uint32_t *p = tb.cnt + ((size_t)c * tb.nr) * tb.nblk + jb;
    uint32_t *out = tb.ta + ((size_t)jb * tb.nch + c) * (tb.nr + 1);
    uint32_t run = 0;
    for (int r = 0; r < tb.nr; ++r, p += tb.nblk) { out[r] = run; run += (*p + kSubPad - 1u) & ~(kSubPad - 1u); }
    out[tb.nr] = run;
    tb.tstart[(size_t)jb * tb.nch + c] = run;
}

// ------------------------------------------------------------------------------------------------
// counts -> starts, Lx / R side.  One thread per row (c, r): exclusive prefix over the column blocks of
// the padded counts -> dd[jb][c][r]; the row stream's length goes to sstart[c][r], to be scanned.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_tp_scan_d(TpTables tb) {
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (int64_t)tb.nch * tb.nr) return;
    const int c = (int)(id / tb.nr), r = (int)(id % tb.nr);
    const uint32_t *p = tb.cnt + ((size_t)c * tb.nr + r) * tb.nblk;
    uint32_t *out = tb.dd + (size_t)c * tb.nr + r;
    const size_t step = (size_t)tb.nch * tb.nr;
    uint32_t run = 0;
    for (int jb0 = 0; jb0 < tb.nblk; jb0 += 4) {          // four counts per turn: the loads side by side
        uint32_t x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = jb0 + u < tb.nblk ? p[jb0 + u] : 0u;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (jb0 + u < tb.nblk) out[(size_t)(jb0 + u) * step] = run;
            run += (x[u] + kSubPad - 1u) & ~(kSubPad - 1u);
        }
    }
    tb.sstart[(size_t)c * tb.nr + r] = run;
}

// In-place exclusive prefix of a[0..m) by one workgroup, total in a[m]; workgroup b scans array b
// (up to three arrays per launch).
__global__ __launch_bounds__(1024) void k_tp_scan(u64 *__restrict__ a0, int64_t m0, u64 *__restrict__ a1, int64_t m1,
                                                  u64 *__restrict__ a2, int64_t m2) {
    __shared__ u64 part[1024];
    u64 *a = blockIdx.x == 0 ? a0 : (blockIdx.x == 1 ? a1 : a2);
    const int64_t m = blockIdx.x == 0 ? m0 : (blockIdx.x == 1 ? m1 : m2);
    const int tid = threadIdx.x;
    const int64_t per = (m + 1023) / 1024;
    const int64_t lo = tid * per;
    const int64_t hi = lo + per < m ? lo + per : m;
    u64 sum = 0;
    for (int64_t q = lo; q < hi; ++q) sum += a[q];
    part[tid] = sum;
    __syncthreads();
    u64 run = 0;
    for (int s = 0; s < tid; ++s) run += part[s];
    for (int64_t q = lo; q < hi; ++q) { const u64 t = a[q]; a[q] = run; run += t; }
    if (tid == 1023) a[m] = run;      // threads past the end have lo >= m: run = grand total
}

// ------------------------------------------------------------------------------------------------
// Re-layout, step 2: workgroup c * ngroups + g moves the runs of block group g of every unit of
// chunk c (slice parts, then share parts) from U to their sub-segments, `batch` rows (slices, then
// shares) at a time.  In T the sub-segments of consecutive rows are adjacent, so the tuples of a
// batch form one piece per block of the group; the pieces are put together in LDS, pad tuples
// included (row field 2048: the score kernel ignores them; they fill every sub-segment up to a
// multiple of kSubPad), and written out contiguously: the columns (24 bytes per group of eight) to T piece by
// piece, the row fields (16 bits each) to R sub-segment by sub-segment (in R the sub-segments of one
// row for consecutive blocks are adjacent).  A batch that does not fit `cap` slots is halved until it
// does; a row that does not fit is written tuple by tuple.
// LDS: tbase[nbg], sbase[batch], runsrc[batch * npmax] (u64), runlen[batch * npmax + 1],
//      runsl[batch * npmax], joff[nbg + 1], s0[nbg], cur / sub0 / sublen / ddv [batch * nbg], stage[cap]
// ------------------------------------------------------------------------------------------------
constexpr int kPlaceThreads = 512;

// T holds the tuples in groups of eight, 24 bytes each: a 32-bit word with the index of the 32-bit word
// of Lx (eight labels of 4 bits; the pair of words when labels take 8 bits) the group's labels go to,
// then the eight columns, 20 bits each, as one little-endian number of 160 bits.
__device__ __forceinline__ void tp_pack_columns(const uint32_t (&c)[8], uint32_t (&w)[5]) {
    w[0] = c[0] | (c[1] << 20);
    w[1] = (c[1] >> 12) | (c[2] << 8) | (c[3] << 28);
    w[2] = (c[3] >> 4) | (c[4] << 16);
    w[3] = (c[4] >> 16) | (c[5] << 4) | (c[6] << 24);
    w[4] = (c[6] >> 8) | (c[7] << 12);
}
__device__ __forceinline__ void tp_unpack_columns(const uint32_t (&w)[5], uint32_t (&c)[8]) {
    c[0] = w[0] & 0xFFFFFu;
    c[1] = ((w[0] >> 20) | (w[1] << 12)) & 0xFFFFFu;
    c[2] = (w[1] >> 8) & 0xFFFFFu;
    c[3] = ((w[1] >> 28) | (w[2] << 4)) & 0xFFFFFu;
    c[4] = ((w[2] >> 16) | (w[3] << 16)) & 0xFFFFFu;
    c[5] = (w[3] >> 4) & 0xFFFFFu;
    c[6] = ((w[3] >> 24) | (w[4] << 8)) & 0xFFFFFu;
    c[7] = w[4] >> 12;
}

__device__ __host__ inline size_t tp_place_fixed_bytes(int nbg, int batch, int maxruns) {
    return ((size_t)nbg + batch + maxruns) * 8 + ((size_t)2 * maxruns + 1 + 2 * (size_t)nbg + 1 + 4 * (size_t)batch * nbg) * 4;
}

__global__ __launch_bounds__(kPlaceThreads) void k_tp_place(int64_t n, SweepPlan pl, TpTables tb,
                                                            const uint32_t *__restrict__ U,
                                                            uint32_t *__restrict__ T, uint16_t *__restrict__ R,
                                                            int batch, uint32_t cap) {
    extern __shared__ u64 smem64[];
    const int g = (int)(blockIdx.x % (unsigned)tb.ngroups), c = (int)(blockIdx.x / (unsigned)tb.ngroups);
    const int jb0 = g << tb.gb;
    const int nbg = (jb0 + (1 << tb.gb)) <= tb.nblk ? (1 << tb.gb) : tb.nblk - jb0;
    const int npmax = tb.npr > tb.nps ? tb.npr : tb.nps;
    const int maxruns = batch * npmax;
    u64 *tbase = smem64;                                        // nbg        segment (jb, c) in T
    u64 *sbase = tbase + nbg;                                   // batch      row stream (c, r) in R
    u64 *runsrc = sbase + batch;                                // maxruns    first tuple of the run
    uint32_t *runlen = reinterpret_cast<uint32_t *>(runsrc + maxruns);  // maxruns + 1   tuples in the run
    uint32_t *runsl = runlen + maxruns + 1;                     // maxruns    row (in the batch) of the run
    uint32_t *joff = runsl + maxruns;                           // nbg + 1    start of block j's piece in stage
    uint32_t *s0 = joff + nbg + 1;                              // nbg        start of the piece in the segment
    uint32_t *cur = s0 + nbg;                                   // batch * nbg  next free slot of sub-segment (t, j)
    uint32_t *sub0 = cur + batch * nbg;                         // batch * nbg  its first slot (in stage, or in the segment)
    uint32_t *sublen = sub0 + batch * nbg;                      // batch * nbg  its padded length
    uint32_t *ddv = sublen + batch * nbg;                       // batch * nbg  its start in the row stream
    uint32_t *stage = ddv + batch * nbg;                        // cap
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int kNW = kPlaceThreads / 64, kRU = 4, kXU = 3;
    const int64_t chunk_lo = (int64_t)c * tb.chunk;
    const int64_t chunk_hi = (chunk_lo + tb.chunk < n) ? chunk_lo + tb.chunk : n;
    const int nsl_c = (int)((chunk_hi - chunk_lo + kSliceRows - 1) / kSliceRows);
    const int nvs = (int)pl.ch_nvs[c];
    const uint32_t gmask = (1u << tb.gb) - 1u, cmask = (1u << tb.cb) - 1u;
    const uint32_t pad = 2048u << tb.cb;
    for (int j = tid; j < nbg; j += kPlaceThreads) tbase[j] = tb.tstart[(size_t)(jb0 + j) * tb.nch + c];
    // slot w of sub-segment z = (t, j), written on its own (the slow way): its column into the group's
    // 160 bits, which the caller has cleared (the group's first word set), 2 bytes of R
    auto put_entry = [&](uint32_t j, uint32_t z, uint32_t w, uint32_t tuple) {
        const uint32_t row = tuple >> tb.cb;
        const u64 at = sbase[z / (uint32_t)nbg] + ddv[z] + (w - sub0[z]);      // the tuple's slot in R / Lx
        const uint32_t col = tuple & cmask;
        if (col) {
            const u64 slot = tbase[j] + w;
            uint32_t *grp = T + (slot >> 3) * 6ull + 1;
            const uint32_t bit = 20u * ((uint32_t)slot & 7u);
            atomicOr(grp + (bit >> 5), col << (bit & 31u));
            if ((bit & 31u) > 12u) atomicOr(grp + (bit >> 5) + 1, col >> (32u - (bit & 31u)));
        }
        R[at] = (uint16_t)(row >= (uint32_t)kSliceRows ? 1u : row << 5);
    };
    for (int part = 0; part < 2; ++part) {                      // 0: regular slices, 1: hub shares
        const int count = part == 0 ? nsl_c : nvs;
        const int np = part == 0 ? tb.npr : tb.nps;
        const int rfirst = part == 0 ? 0 : tb.nsl;              // the part's first row of the chunk
        const uint32_t *lot = part == 0 ? tb.lo : tb.loh;
        const u64 *ust = part == 0 ? tb.ustart : tb.ustart_h;
        int i0 = 0;
        while (i0 < count) {
            // the largest batch (<= `batch` rows) whose pieces fit the stage; at least one row
            int nb = count - i0 < batch ? count - i0 : batch;
            const int r0 = rfirst + i0;
            uint32_t need;
            for (;;) {
                __syncthreads();                                // previous batch (attempt) done with the LDS tables
                for (int z = tid; z < nb * np; z += kPlaceThreads) {
                    const int t = z / np, q = z % np;
                    const size_t unit = ((size_t)c * tb.nsl + i0 + t) * np + q;
                    const uint32_t a = lot[unit * (tb.ngroups + 1) + g], b = lot[unit * (tb.ngroups + 1) + g + 1];
                    runsrc[z] = ust[unit] + a;                   // (a unit that does not exist has no tuples)
                    runlen[z] = b - a;
                    runsl[z] = (uint32_t)t;
                }
                for (int j = tid; j < nbg; j += kPlaceThreads) {
                    const uint32_t *taj = tb.ta + ((size_t)(jb0 + j) * tb.nch + c) * (tb.nr + 1);
                    const uint32_t a = taj[r0];
                    s0[j] = a;
                    joff[j + 1] = taj[r0 + nb] - a;
                }
                __syncthreads();
                if (nbg <= 64) {                                // lengths of the pieces -> their starts in stage
                    if (tid < 64) {
                        uint32_t inc = tid < nbg ? joff[tid + 1] : 0u;
#pragma unroll
                        for (int off = 1; off < 64; off <<= 1) {
                            const uint32_t o = __shfl_up(inc, off);
                            if (tid >= off) inc += o;
                        }
                        if (tid < nbg) joff[tid + 1] = inc;
                        if (tid == 0) joff[0] = 0;
                    }
                } else if (tid == 0) {
                    uint32_t run = 0;
                    joff[0] = 0;
                    for (int j = 0; j < nbg; ++j) { run += joff[j + 1]; joff[j + 1] = run; }
                }
                __syncthreads();
                need = joff[nbg];
                if (need <= cap || nb == 1) break;
                nb >>= 1;
            }
            const bool staged = need <= cap;
            for (int z = tid; z < nb * nbg; z += kPlaceThreads) {
                const int t = z / nbg, j = z % nbg;
                const uint32_t *taj = tb.ta + ((size_t)(jb0 + j) * tb.nch + c) * (tb.nr + 1);
                const uint32_t a = taj[r0 + t], e = taj[r0 + t + 1];
                // staged: slot in stage; else: slot in the segment
                const uint32_t first = staged ? joff[j] + (a - s0[j]) : a;
                sub0[z] = first;
                cur[z] = first;
                sublen[z] = e - a;
                ddv[z] = tb.dd[((size_t)(jb0 + j) * tb.nch + c) * tb.nr + r0 + t];
            }
            for (int t = tid; t < nb; t += kPlaceThreads) sbase[t] = tb.sstart[(size_t)c * tb.nr + r0 + t];
            if (staged) {
                for (uint32_t z = tid; z < need; z += kPlaceThreads) stage[z] = pad;
            } else {
                // the slow way: every group of the sub-segments gets its first word, its columns start at zero
                __syncthreads();                                // sub0 / sublen / ddv / sbase are complete
                for (int z = 0; z < nb * nbg; ++z) {
                    const int j = z % nbg;
                    const u64 first = (tbase[j] + sub0[z]) >> 3, dest = (sbase[z / nbg] + ddv[z]) >> 3;
                    for (uint32_t q = tid; q < (sublen[z] >> 3); q += kPlaceThreads) {
                        uint32_t *grp = T + (first + q) * 6ull;
                        grp[0] = (uint32_t)(dest + q);
                        grp[1] = 0; grp[2] = 0; grp[3] = 0; grp[4] = 0; grp[5] = 0;
                    }
                }
                __threadfence();
            }
            __syncthreads();
            // a wavefront takes whole runs, kRU at a time, the first kXU * 64 tuples of each loaded side
            // by side before any is placed
            const int nruns = nb * np;
            auto put = [&](uint32_t u, uint32_t sl) {
                const uint32_t j = (u >> tb.cb) & gmask;
                const uint32_t z = sl * (uint32_t)nbg + j;
                const uint32_t w = atomicAdd(&cur[z], 1u);
                const uint32_t tuple = ((u >> (tb.cb + tb.gb)) << tb.cb) | (u & cmask);
                if (staged) stage[w] = tuple;
                else put_entry(j, z, w, tuple);
            };
            for (int z0 = wave; z0 < nruns; z0 += kNW * kRU) {
                uint32_t u[kRU][kXU], len[kRU], sl[kRU];
                const uint32_t *from[kRU];
#pragma unroll
                for (int r = 0; r < kRU; ++r) {
                    const int z = z0 + r * kNW;
                    const int zz = z < nruns ? z : z0;
                    len[r] = z < nruns ? (uint32_t)__builtin_amdgcn_readfirstlane((int)runlen[zz]) : 0u;
                    sl[r] = (uint32_t)__builtin_amdgcn_readfirstlane((int)runsl[zz]);
                    const u64 at = runsrc[zz];
                    from[r] = U + (((u64)(uint32_t)__builtin_amdgcn_readfirstlane((int)(at >> 32)) << 32) |
                                   (u64)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)at));
#pragma unroll
                    for (int x = 0; x < kXU; ++x) {
                        const uint32_t p = (uint32_t)(x * 64 + lane);
                        u[r][x] = p < len[r] ? __builtin_nontemporal_load(from[r] + p) : 0u;
                    }
                }
#pragma unroll
                for (int r = 0; r < kRU; ++r) {
#pragma unroll
                    for (int x = 0; x < kXU; ++x)
                        if ((uint32_t)(x * 64 + lane) < len[r]) put(u[r][x], sl[r]);
                }
#pragma unroll
                for (int r = 0; r < kRU; ++r)
                    for (uint32_t p = (uint32_t)(kXU * 64 + lane); p < len[r]; p += 64)
                        put(__builtin_nontemporal_load(from[r] + p), sl[r]);
            }
            __syncthreads();
            if (staged) {
                // T: a piece per wavefront, a group of eight tuples (24 bytes) per lane; starts and lengths
                // are multiples of 8 tuples
                for (int j = wave; j < nbg; j += kNW) {
                    const uint32_t a = joff[j], len8 = (joff[j + 1] - a) >> 3;
                    uint32_t *outT = T + ((tbase[j] + s0[j]) >> 3) * 6ull;
                    for (uint32_t z = lane; z < len8; z += 64) {
                        // the row of the batch whose sub-segment holds the group, and its slot in R / Lx
                        const uint32_t x = a + 8 * z;
                        int t = 0;
                        while (t + 1 < nb && x >= sub0[(t + 1) * nbg + j]) ++t;
                        const u64 at = sbase[t] + ddv[t * nbg + j] + (x - sub0[t * nbg + j]);
                        uint32_t col[8], w[5];
#pragma unroll
                        for (int q = 0; q < 8; ++q) col[q] = stage[x + q] & cmask;
                        tp_pack_columns(col, w);
                        u32x3a lo3, hi3;
                        lo3.x = (uint32_t)(at >> 3); lo3.y = w[0]; lo3.z = w[1];
                        hi3.x = w[2]; hi3.y = w[3]; hi3.z = w[4];
                        __builtin_nontemporal_store(lo3, reinterpret_cast<u32x3a *>(outT + 6 * z));
                        __builtin_nontemporal_store(hi3, reinterpret_cast<u32x3a *>(outT + 6 * z + 3));
                    }
                }
                // R: a sub-segment per quarter wavefront, four tuples (8 bytes) per lane
                for (int z = wave * 4 + (lane >> 4); z < nb * nbg; z += kNW * 4) {
                    const uint32_t a = sub0[z], len4 = sublen[z] >> 2;
                    uint32_t *outR = reinterpret_cast<uint32_t *>(R + sbase[z / nbg] + ddv[z]);
                    for (uint32_t y = (uint32_t)(lane & 15); y < len4; y += 16) {
                        uint32_t row[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const uint32_t r = stage[a + 4 * y + q] >> tb.cb;
                            row[q] = r >= (uint32_t)kSliceRows ? 1u : r << 5;
                        }
                        u32x2 r2;
                        r2.x = row[0] | (row[1] << 16);
                        r2.y = row[2] | (row[3] << 16);
                        __builtin_nontemporal_store(r2, reinterpret_cast<u32x2 *>(outR + 2 * y));
                    }
                }
            } else {
                for (int z = tid; z < nb * nbg; z += kPlaceThreads) {
                    const uint32_t end = sub0[z] + sublen[z];
                    for (uint32_t w = cur[z]; w < end; ++w) put_entry((uint32_t)(z % nbg), (uint32_t)z, w, pad);
                }
            }
            i0 += nb;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// look-up (phase 1 of the score): the tuples of the column blocks of chunk `c0 + blockIdx.y`,
// restricted to row chunks >= cmin, get their labels.  Workgroup blockIdx.x handles share
// (blockIdx.x % spb) of block (blockIdx.x / spb) of the chunk: an equal part of the block's tuples
// in T, which are one contiguous piece.
//   T  (read)   : per group of eight tuples 24 bytes: the index of the word of Lx their labels go to,
//                 then their columns in the block, 20 bits each
//   Lx (written): the label of every tuple, LB = 4 bits each (8 when k > 16), sub-segments ordered (c', r, jb): a group's
//                 word lies in the stream of its row slice, so the writes of one sub-segment are a
//                 contiguous piece of some 40 bytes; the pieces of the chunk's column blocks are
//                 neighbours and are written by workgroups of one XCD at about the same time, so that
//                 they meet in its L2 (plain stores: the line is kept there until it is complete)
//   R           : the row field of every tuple << 5 (bit 0: padding), 16 bits each, ordered like Lx; written
//                 once by the re-layout
//   FROM_LDS = true : the block's labels are copied to LDS, two per byte (every vertex of the
//                     block is assigned: the chunk has just been relabelled), from Lc, or from Lc4
//                     (the same labels already two per byte) when that is given
//   FROM_LDS = false: labels are read from global memory and may be unassigned; used once, for the
//                     initial labels of a seeded run
//   WRITE_R         : seeded runs only.  Their first pass reads the row fields from a copy Rdyn in
//                     which bit 0 also marks tuples whose neighbour is unassigned: the initial
//                     look-up (FROM_LDS = false) sets it, the first pass's look-ups clear it.
// A thread takes 8 tuples at a time: 24 bytes of T, one 32-bit word of Lx (16 bytes of R / Rdyn).
// ------------------------------------------------------------------------------------------------
constexpr int kLookupUnroll = 2;       // groups of eight per thread in flight

template <bool FROM_LDS, bool WRITE_R, int LB>
__global__ __launch_bounds__(kTpThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_tp_lookup(const uint32_t *__restrict__ T,
                                                          uint32_t *__restrict__ Lx,
                                                          const uint16_t *__restrict__ R,
                                                          uint16_t *__restrict__ Rdyn, TpTables tb,
                                                          const uint8_t *__restrict__ Lc,
                                                          const uint8_t *__restrict__ Lc4, int64_t n, int c0,
                                                          int cmin, int spb) {
    extern __shared__ uint32_t tab[];      // FROM_LDS: 2^cb labels, LB bits each
    const int tid = threadIdx.x;
    const int c = c0 + (int)blockIdx.y;
    const int m = (int)blockIdx.x / spb, s = (int)blockIdx.x % spb;
    const int64_t chunk_lo = (int64_t)c * tb.chunk;
    const int64_t chunk_hi = (chunk_lo + tb.chunk < n) ? chunk_lo + tb.chunk : n;
    const int64_t block_lo = chunk_lo + ((int64_t)m << tb.cb);
    if (block_lo >= chunk_hi || cmin >= tb.nch) return;
    const int jb = c * tb.nbc + m;
    const u64 *ts = tb.tstart + (size_t)jb * tb.nch;       // ts[c'] for c' = 0..nch (ts[nch] = end of block)
    const u64 lo = ts[cmin], hi = ts[tb.nch];
    const u64 groups = (hi - lo) >> 3;                      // (every sub-segment is a multiple of 8 tuples)
    const u64 g0 = groups * (u64)s / (u64)spb, g1 = groups * (u64)(s + 1) / (u64)spb;
    if (g0 >= g1) return;
    const uint32_t ng = (uint32_t)(g1 - g0);
    const uint32_t *src = T + ((lo >> 3) + g0) * 6ull;      // 6 words per group

    constexpr int U = kLookupUnroll;
    u32x3a t[U][2];
    auto load_groups = [&](uint32_t base) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t gi = base + u * kTpThreads;
            t[u][0] = (u32x3a){0u, 0u, 0u};
            t[u][1] = (u32x3a){0u, 0u, 0u};
            if (gi < ng) {
                t[u][0] = __builtin_nontemporal_load(reinterpret_cast<const u32x3a *>(src + 6ull * gi));
                t[u][1] = __builtin_nontemporal_load(reinterpret_cast<const u32x3a *>(src + 6ull * gi + 3));
            }
        }
    };
    // The first tuples are requested while the label table is built -- after the table's own loads,
    // whose data is needed first (a wavefront's loads complete in the order they were issued).
    bool requested = false;
    auto first_groups = [&] {
        if (!requested) load_groups((uint32_t)tid);
        requested = true;
    };
    if (!FROM_LDS) first_groups();

    if (FROM_LDS && LB == 8) {
        // the block's labels as they are, a byte each
        const int64_t bv = (chunk_hi - block_lo) < (1ll << tb.cb) ? (chunk_hi - block_lo) : (1ll << tb.cb);
        const uint8_t *lsrc = Lc + block_lo;
        uint8_t *tb8 = reinterpret_cast<uint8_t *>(tab);
        if ((((uintptr_t)lsrc) & 15u) == 0) {
            // (every workgroup of the block starts its copy at a place of its own: see below)
            const int64_t pieces = bv >> 4;
            const int64_t start = (pieces * (int64_t)s / (int64_t)spb) & ~(int64_t)7;
            for (int64_t i = tid; i < pieces; i += kTpThreads) {
                const int64_t at = i + start < pieces ? i + start : i + start - pieces;
                reinterpret_cast<u32x4 *>(tab)[at] = *reinterpret_cast<const u32x4 *>(lsrc + at * 16);
            }
            for (int64_t o = (pieces << 4) + tid; o < bv; o += kTpThreads) tb8[o] = lsrc[o];
        } else {
            for (int64_t o = tid; o < bv; o += kTpThreads) tb8[o] = lsrc[o];
        }
        first_groups();
        __syncthreads();
    }
    if (FROM_LDS && LB == 4) {
        const int64_t bv = (chunk_hi - block_lo) < (1ll << tb.cb) ? (chunk_hi - block_lo) : (1ll << tb.cb);
        const int words = (int)((bv + 7) >> 3);
        const uint8_t *lsrc = Lc + block_lo;
        const bool aligned = (((uintptr_t)lsrc) & 15u) == 0;
        auto pack4 = [](uint32_t a) {       // four labels, one per byte -> 16 bits
            return (a & 15u) | ((a >> 4) & 0xF0u) | ((a >> 8) & 0xF00u) | ((a >> 12) & 0xF000u);
        };
        const uint8_t *packed = Lc4 ? Lc4 + (block_lo >> 1) : nullptr;
        if (packed && bv == (1ll << tb.cb) && (words % (4 * kTpThreads)) == 0 && (((uintptr_t)packed) & 15u) == 0) {
            // the labels are at hand two per byte (Lc4: kept by the admission once every vertex has a
            // label): a plain copy, 32 labels per load; every workgroup of the block starts at a place
            // of its own (see below)
            const uint32_t pieces = (uint32_t)words / 4u;       // a power of two
            const uint32_t start = (uint32_t)(((u64)pieces * (u64)s) / (u64)spb) & ~7u;
            constexpr int kFill = 4;
            for (uint32_t i0 = 0; i0 < pieces; i0 += kFill * kTpThreads) {
                u32x4 v[kFill];
#pragma unroll
                for (int i = 0; i < kFill; ++i) {
                    const uint32_t at = (i0 + (uint32_t)i * kTpThreads + tid + start) & (pieces - 1u);
                    if (i0 + (uint32_t)i * kTpThreads + tid < pieces) v[i] = reinterpret_cast<const u32x4 *>(packed)[at];
                }
                first_groups();
#pragma unroll
                for (int i = 0; i < kFill; ++i) {
                    const uint32_t at = (i0 + (uint32_t)i * kTpThreads + tid + start) & (pieces - 1u);
                    if (i0 + (uint32_t)i * kTpThreads + tid < pieces) reinterpret_cast<u32x4 *>(tab)[at] = v[i];
                }
            }
        } else if (aligned && bv == (1ll << tb.cb) && (words % (2 * kTpThreads)) == 0) {
            // a whole block at a 16-byte boundary (the usual case): 16 labels per load, all loads of a
            // thread side by side
            // The workgroups of a block all copy the same labels at the same time: each starts at a place
            // of its own and wraps around, so that they do not all queue at the same few L2 channels.
            constexpr int kFill = 8;
            const int per = words / (2 * kTpThreads);          // 16-label pieces per thread
            const uint32_t pieces = (uint32_t)per * kTpThreads;   // a power of two
            const uint32_t start = (uint32_t)(((u64)pieces * (u64)s) / (u64)spb) & ~7u;
            for (int i0 = 0; i0 < per; i0 += kFill) {
                u32x4 v[kFill];
#pragma unroll
                for (int i = 0; i < kFill; ++i)
                    if (i0 + i < per) {
                        const uint32_t at = ((uint32_t)(i0 + i) * kTpThreads + tid + start) & (pieces - 1u);
                        v[i] = *reinterpret_cast<const u32x4 *>(lsrc + (size_t)at * 16);
                    }
                first_groups();
#pragma unroll
                for (int i = 0; i < kFill; ++i)
                    if (i0 + i < per) {
                        const uint32_t at = ((uint32_t)(i0 + i) * kTpThreads + tid + start) & (pieces - 1u);
                        u32x2 o;
                        o.x = pack4(v[i].x) | (pack4(v[i].y) << 16);
                        o.y = pack4(v[i].z) | (pack4(v[i].w) << 16);
                        *reinterpret_cast<u32x2 *>(tab + 2 * (size_t)at) = o;
                    }
            }
        } else {
            for (int w = tid; w < words; w += kTpThreads) {
                uint32_t packed = 0;
                for (int qq = 0; qq < 8; ++qq) {
                    const int64_t o = (int64_t)w * 8 + qq;
                    if (o < bv) packed |= ((uint32_t)lsrc[o] & 15u) << (4 * qq);
                }
                tab[w] = packed;
            }
        }
        first_groups();
        __syncthreads();
    }
    const uint8_t *tbytes = reinterpret_cast<const uint8_t *>(tab);

    for (uint32_t base = tid; base < ng; base += kTpThreads * U) {
        if (base != (uint32_t)tid) load_groups(base);       // (the first turn is on its way)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (base + u * kTpThreads >= ng) continue;
            const uint32_t w5[5] = {t[u][0].y, t[u][0].z, t[u][1].x, t[u][1].y, t[u][1].z};
            uint32_t col[8];
            tp_unpack_columns(w5, col);
            const uint32_t dest = t[u][0].x;
            uint32_t word = 0, word2 = 0, unassigned = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint32_t lab;
                if (FROM_LDS) {
                    lab = LB == 4 ? ((uint32_t)tbytes[col[e] >> 1] >> (4 * (col[e] & 1u))) & 15u : (uint32_t)tbytes[col[e]];
                } else {
                    const int64_t v = block_lo + (int64_t)col[e];
                    const uint32_t l = v < chunk_hi ? (uint32_t)Lc[v] : 0xFFu;
                    if (l == 0xFFu) unassigned |= 1u << e;
                    lab = LB == 4 ? (l & 15u) : (l == 0xFFu ? 0u : l);
                }
                if (LB == 4) word |= lab << (4 * e);
                else if (e < 4) word |= lab << (8 * e);
                else word2 |= lab << (8 * (e - 4));
            }
            if (LB == 4) {
                Lx[dest] = word;
            } else {
                u32x2 o;
                o.x = word; o.y = word2;
                reinterpret_cast<u32x2 *>(Lx)[dest] = o;
            }
            if (WRITE_R) {
                const u64 at = (u64)dest << 3;
                const u32x4 rr = *reinterpret_cast<const u32x4 *>(R + at);
                u32x4 o;
                o.x = rr.x | (unassigned & 1u) | ((unassigned & 2u) << 15);
                o.y = rr.y | ((unassigned >> 2) & 1u) | ((unassigned & 8u) << 13);
                o.z = rr.z | ((unassigned >> 4) & 1u) | ((unassigned & 32u) << 11);
                o.w = rr.w | ((unassigned >> 6) & 1u) | ((unassigned & 128u) << 9);
                *reinterpret_cast<u32x4 *>(Rdyn + at) = o;
            }
        }
    }
}

// The value of lane (l ^ 1) (CTRL = 0xB1: quad_perm [1,0,3,2]) or (l ^ 2) (0x4E: [2,3,0,1]) of the
// lane's quad, by a data-parallel-primitive move instead of a trip through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ uint32_t quad_swap(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

// Counting tuples: row fields from R (16 bits each, bit 0 set: not to be counted), labels from Lx (LB
// = 4 or 8 bits each: 4 while k <= 16).  16 bits of R: row field << 5 | skip (bit 0: padding, or an
// unassigned neighbour).  The row's KP (16 or 32) counters of 16 bits start at byte (row field << 5)
// * KP / 16, to which (label >> 1) << 2 adds the counter pair's; the label's bit 0 picks the half.
template <int LB> struct TpLabels;                      // the labels of a group of eight tuples
template <> struct TpLabels<4> {
    uint32_t w;
    __device__ __forceinline__ uint32_t get(int e) const { return (w >> (4 * e)) & 15u; }
    __device__ __forceinline__ static TpLabels load(const uint32_t *__restrict__ Lx, u64 base, uint32_t g) {
        TpLabels x;
        x.w = __builtin_nontemporal_load(Lx + (base >> 3) + g);
        return x;
    }
    __device__ __forceinline__ static TpLabels none() { TpLabels x; x.w = 0; return x; }
};
template <> struct TpLabels<8> {
    u32x2 w;
    __device__ __forceinline__ uint32_t get(int e) const { return ((e < 4 ? w.x : w.y) >> (8 * (e & 3))) & 255u; }
    __device__ __forceinline__ static TpLabels load(const uint32_t *__restrict__ Lx, u64 base, uint32_t g) {
        TpLabels x;
        x.w = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(Lx + (base >> 2)) + g);
        return x;
    }
    __device__ __forceinline__ static TpLabels none() { TpLabels x; x.w = (u32x2)(0u); return x; }
};

// a group of eight tuples: 16 bytes of R, their labels
// SW (k <= 8, KP = 16): a row's eight counter words would use two to four of their places only, and the
// rows' words eight to thirty-two of the 64 LDS banks; the 8-byte piece of partitions 4p .. 4p+3 of row t
// therefore sits at place p ^ ((t >> 3) & 3) of the row, which spreads them over all banks.
template <bool COUNT16, int KP, int LB, bool SW>
__device__ __forceinline__ void tp_count_eight(const u32x4 rows, const TpLabels<LB> labels, int k, uint32_t *hist) {
    static_assert(!SW || (COUNT16 && KP == 16), "the swizzle is that of the 16-counter rows");
    const uint32_t w[4] = {rows.x, rows.y, rows.z, rows.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t half = (e & 1) ? (w[e >> 1] >> 16) : w[e >> 1];
        const uint32_t lab = labels.get(e);
        const uint32_t r = half & 0xFFE0u;
        const uint32_t one = (~half) & 1u;                // bit 0 clear: the tuple is to be counted
        if (COUNT16) {
            // no branch: what is not to be counted adds zero (to a counter its bits happen to name)
            uint32_t off = (KP == 16 ? r : r << 1) | ((lab & ~1u) << 1);
            if (SW) off ^= (r >> 5) & 0x18u;                  // ((row >> 3) & 3) << 3: the piece's place
            uint32_t *ctr = reinterpret_cast<uint32_t *>(reinterpret_cast<char *>(hist) + off);
            atomicAdd(ctr, one << ((lab & 1u) << 4));
        } else if (one) {
            atomicAdd(&hist[(r >> 5) * (uint32_t)k + lab], 1u);
        }
    }
}

// Groups [g0, g1) of a row stream that starts at slot `base` (a multiple of 8) of R and Lx, counted by
// the whole workgroup, NU groups per thread in flight.
template <bool COUNT16, int KP, int LB, int NU, bool SW = false>
__device__ __forceinline__ void tp_count_stream(const uint16_t *__restrict__ R, const uint32_t *__restrict__ Lx, u64 base,
                                                uint32_t g0, uint32_t g1, int k, uint32_t *hist) {
    const u32x4 *R4 = reinterpret_cast<const u32x4 *>(R + base);
    for (uint32_t g = g0 + threadIdx.x; g < g1; g += kTpThreads * NU) {
        u32x4 rows[NU];
        TpLabels<LB> labs[NU];
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const uint32_t gi = g + u * kTpThreads;
            rows[u] = (u32x4)(1u | (1u << 16));         // nothing to count
            labs[u] = TpLabels<LB>::none();
            if (gi < g1) {
                rows[u] = __builtin_nontemporal_load(R4 + gi);
                labs[u] = TpLabels<LB>::load(Lx, base, gi);
            }
        }
#pragma unroll
        for (int u = 0; u < NU; ++u)
            if (g + u * kTpThreads < g1) tp_count_eight<COUNT16, KP, LB, SW>(rows[u], labs[u], k, hist);
    }
}

// The value of lane (l ^ 4), (l ^ 8): through the LDS crossbar.
__device__ __forceinline__ unsigned long long tp_xor_lane64(unsigned long long v, int mask) {
    return ((unsigned long long)(uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), mask) << 32) |
           (unsigned long long)(uint32_t)__shfl_xor((int)(uint32_t)v, mask);
}

// ------------------------------------------------------------------------------------------------
// score (phase 2): one workgroup per row slice of chunk c.  It counts the slice's row stream: the
// sub-segments of the column blocks in [0, jlim), a prefix of the stream (in the first pass of an
// unseeded run the blocks of chunks >= c hold no label yet and their part of Lx has not been
// written); and, of hub share (slice % nvs), an equal part of that share's stream (same prefix
// rule), so that the hub entries are spread evenly too.  Then it blends E, proposes, and counts the
// movers of its two admission tiles per proposed partition (cnt, the input of the admission;
// k_hub_finalize adds the hubs).
//
// SW: k <= 8 (with KP = 16): the rows' counter pieces are swizzled over the LDS banks (tp_count_eight).
// KP = 16 (k <= 16, 4-bit labels in Lx, 64 KB of counters: two workgroups per CU) or 32 (k <= 32,
// 8-bit labels, 128 KB of counters: one workgroup per CU).  KP / 4 lanes share a vertex in the
// blend: lane q owns partitions 4q .. 4q+3 when k % 4 == 0 (one 8- or 16-byte piece of E's row), else
// q, q + KP/4, q + 2 KP/4, q + 3 KP/4.
// hub_old: see below (may be null).
// coarse (may be null): [tiles / kCoarseTiles][k], the mover counts of kCoarseTiles tiles added up (atomic adds
// into a table that starts at zero), so that the admission need not read every tile's counts.
// LDS: hist[kSliceRows * KP / 2] (16-bit counters, KP per row; a static array when KP = 16),
//      meta[kSliceRows / 2] (per row: old label, hub flag << 8), hhist[share_hubs * k], room[k], tcnt[2 * k]
// ------------------------------------------------------------------------------------------------
constexpr int kCoarseTiles = 32;         // tiles per row of the coarse mover counts (a slice's two tiles share one)

template <typename ET, int KP, bool SW = false>
__global__ __launch_bounds__(kTpThreads) __attribute__((amdgpu_waves_per_eu(KP == 16 ? 8 : 4, KP == 16 ? 8 : 4))) void k_tp_score(
    const uint16_t *__restrict__ R, const uint32_t *__restrict__ Lx, TpTables tb, SweepPlan pl,
    const uint8_t *__restrict__ Lc, const long long *__restrict__ S, ET *__restrict__ E,
    uint32_t *__restrict__ Hhub, uint8_t *__restrict__ prop, uint32_t *__restrict__ cnt,
    long long *__restrict__ room_out, int c, int64_t chunk_lo, int64_t chunk_hi, int k, int jlim,
    int share_hubs, uint32_t nvs, int pass, long long P, int store_e, uint8_t *__restrict__ hub_old,
    uint32_t *__restrict__ coarse) {
    extern __shared__ uint32_t smem[];
    constexpr int LB = KP == 16 ? 4 : 8;
    constexpr int LPV = KP / 4;                                 // lanes per vertex in the blend
    constexpr int hist_words = kSliceRows * KP / 2;
    constexpr int BU = kSliceRows * LPV / kTpThreads;           // (vertex, lane of the vertex) pairs per thread
    constexpr int IDB = KP == 16 ? 4 : 5;                       // bits of a partition id in the arg-max key
    static_assert(kSliceRows == 2 * kAdmitTile, "a slice is two admission tiles");
    // KP = 16: the counters are a static array: its address is a compile-time constant, which spares an
    // add per counted entry
    __shared__ uint32_t hist_static[KP == 16 ? hist_words : 1];
    uint32_t *hist = KP == 16 ? hist_static : smem;
    uint32_t *dyn = KP == 16 ? smem : smem + hist_words;
    uint16_t *meta = reinterpret_cast<uint16_t *>(dyn);                 // kSliceRows
    uint32_t *hhist = dyn + kSliceRows / 2;                             // share_hubs * k, 32-bit
    uint32_t *room = hhist + share_hubs * k;    // k
    uint32_t *tcnt = room + k;                  // 2 * k
    const int tid = threadIdx.x;
    // Workgroups are dispatched round-robin over the 8 XCDs, each with its own L2: give XCD x a
    // contiguous range of slices, so that neighbouring slices, whose streams and rows of E are
    // neighbours in memory, meet in one L2.
    const unsigned xcd = blockIdx.x & 7u, turn = blockIdx.x >> 3;
    const unsigned slice = xcd * (gridDim.x >> 3) + (xcd < (gridDim.x & 7u) ? xcd : (gridDim.x & 7u)) + turn;
    const int64_t v0 = chunk_lo + (int64_t)slice * kSliceRows;
    const int64_t left = chunk_hi - v0;
    const int nv = left < kSliceRows ? (int)left : kSliceRows;
    const bool vec = (k & 3) == 0;

    // the hub share this workgroup helps with (nvs: the chunk's number of shares, known to the host, so
    // that everything this workgroup has to fetch before it can start is requested at once)
    const uint32_t share = nvs ? slice % nvs : 0u;
    const int cls = nvs ? (int)(slice / nvs) : 0;
    const int ncls = nvs ? (int)((gridDim.x - share + nvs - 1) / nvs) : 1;   // workgroups that took this share
    // what to count: a prefix of the slice's stream, and this workgroup's part of the share's (all
    // addresses follow from the arguments: the loads are independent of each other)
    const size_t gs = (size_t)c * tb.nsl + slice;
    const u64 *ss = tb.sstart + (size_t)c * tb.nr;
    const size_t ddrow = ((size_t)(jlim < tb.nblk ? jlim : 0) * tb.nch + c) * tb.nr;     // dd[jlim][c][*]
    const bool whole = jlim >= tb.nblk;
    const uint32_t hr = (uint32_t)tb.nsl + share;
    const u64 sbeg = ss[slice], send = ss[slice + 1];
    const u64 hbeg = nvs ? ss[hr] : 0ull, hend = nvs ? ss[hr + 1] : 0ull;
    const uint32_t sdd = (!whole && jlim > 0) ? tb.dd[ddrow + slice] : 0u;
    const uint32_t hdd = (!whole && jlim > 0 && nvs) ? tb.dd[ddrow + hr] : 0u;
    const bool any_hub = nvs != 0 && pl.share_nhs[(size_t)c * tb.nsl + share] != 0;
    const uint32_t share_h0 = pl.share_h0[(size_t)c * tb.nsl + share];
    const uint32_t snh = pl.sl_nh[gs];
    const u64 slice_hub0 = pl.ch_hub0[c] + pl.sl_hub_start[gs];
    const uint32_t slen = whole ? (uint32_t)(send - sbeg) : sdd;
    uint32_t hg0 = 0, hg1 = 0;
    if (any_hub) {
        const u64 groups = (whole ? (uint32_t)(hend - hbeg) : hdd) >> 3;
        hg0 = (uint32_t)(groups * (u64)cls / (u64)ncls);
        hg1 = (uint32_t)(groups * (u64)(cls + 1) / (u64)ncls);
    }

    {
        u32x4 *z = reinterpret_cast<u32x4 *>(hist);
        for (int q = tid; q < hist_words / 4; q += kTpThreads) z[q] = (u32x4)(0u);
        for (int q = tid; q < share_hubs * k; q += kTpThreads) hhist[q] = 0;
        for (int j = tid; j < k; j += kTpThreads) {
            const long long rj = P - S[j];
            room[j] = (uint32_t)rj;
            if (slice == 0) room_out[j] = rj;           // the sizes' snapshot the admission works against
        }
        for (int j = tid; j < 2 * k; j += kTpThreads) tcnt[j] = 0;
        for (int t = tid; t < nv; t += kTpThreads) meta[t] = (uint16_t)Lc[v0 + t];
    }
    __syncthreads();
    // the slice's hubs, from the chunk's list (read by the blend, after the next barrier)
    // (hub_old, when given: the hubs' labels, by their place in the chunk's list, for the admission kernel that
    // also works the hubs out: it then need not look them up through the list)
    for (uint32_t i = tid; i < snh; i += kTpThreads) {
        const int64_t at = (int64_t)pl.hub_row[slice_hub0 + i] - v0;
        if (hub_old) hub_old[pl.sl_hub_start[gs] + i] = (uint8_t)meta[at];
        meta[at] |= (uint16_t)0x100u;
    }

    tp_count_stream<true, KP, LB, 3, SW>(R, Lx, sbeg, 0u, slen >> 3, k, hist);
    if (any_hub) tp_count_stream<false, KP, LB, 2>(R, Lx, hbeg, hg0, hg1, k, hhist);
    __syncthreads();

    // partial counts of the share's hubs -> the chunk's hub table
    if (any_hub) {
        for (int q = tid; q < share_hubs * k; q += kTpThreads) {
            const uint32_t x = hhist[q];
            if (x) atomicAdd(&Hhub[(size_t)share_h0 * k + q], x);
        }
    }

    const int sh = pass > 0 ? pass - 1 : 0;
    const int q = tid & (LPV - 1);                              // this thread's lane of its vertices
    // k a multiple of 4 with 16-bit estimates (and sizes below 2^27 - IDB): a thread's four partitions
    // are one 8-byte piece of E and one of the counters; two packed adds blend them (no carry between
    // the halves: an estimate stays below 2^16), and the arg-max by (E desc, room desc, id asc) is the
    // maximum of one 64-bit key per partition, E << 40 | room << IDB | KP - 1 - id, 0 if the partition
    // is full (or does not exist: the lanes past k of a vertex hold no partition).
    if (sizeof(ET) == 2 && vec && P < (1ll << (31 - IDB))) {
        const bool mine = 4 * q < k;
        u32x2 e[BU];
#pragma unroll
        for (int u = 0; u < BU; ++u) {
            const int g = tid + u * kTpThreads;
            e[u] = (u32x2)(0u);
            if (pass > 0 && mine && g < nv * LPV)
                e[u] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x2 *>(E + (size_t)(v0 + g / LPV) * (size_t)k + 4 * q));
        }
        uint32_t lo_base[4];
#pragma unroll
        for (int z = 0; z < 4; ++z) lo_base[z] = mine ? (room[4 * q + z] << IDB) | (uint32_t)(KP - 1 - (4 * q + z)) : 0u;
#pragma unroll
        for (int u = 0; u < BU; ++u) {
            const int g = tid + u * kTpThreads;
            if (g >= nv * LPV) continue;
            const int t = g / LPV;
            const uint32_t mt = meta[t];
            if (mt & 0x100u) continue;                              // hubs are k_hub_finalize's
            const uint32_t old = mt & 0xFFu;
            const uint32_t oldz = old - 4u * (uint32_t)q;           // < 4: the old label is one of this thread's
            const uint2 hw = *reinterpret_cast<const uint2 *>(hist + t * (KP / 2) + 2 * (SW ? (q ^ ((t >> 3) & 3)) : q));
            u32x2 o;
            o.x = e[u].x + (hw.x << sh);
            o.y = e[u].y + (hw.y << sh);
            if (store_e && mine)
                __builtin_nontemporal_store(o, reinterpret_cast<u32x2 *>(E + (size_t)(v0 + t) * (size_t)k + 4 * q));
            unsigned long long best = 0;
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const uint32_t ez = z == 0 ? (o.x & 0xFFFFu) : z == 1 ? (o.x >> 16) : z == 2 ? (o.y & 0xFFFFu) : (o.y >> 16);
                const uint32_t lo = lo_base[z] + (oldz == (uint32_t)z ? (1u << IDB) : 0u);    // room + 1 without the vertex itself
                const unsigned long long key = lo >= (1u << IDB) ? (((unsigned long long)(ez << 8) << 32) | lo) : 0ull;
                best = key > best ? key : best;
            }
#pragma unroll
            for (int step = 0; step < 2; ++step) {
                const unsigned long long other =
                    step == 0 ? (((unsigned long long)quad_swap<0xB1>((uint32_t)(best >> 32)) << 32) | quad_swap<0xB1>((uint32_t)best))
                              : (((unsigned long long)quad_swap<0x4E>((uint32_t)(best >> 32)) << 32) | quad_swap<0x4E>((uint32_t)best));
                best = other > best ? other : best;
            }
            if (LPV > 4) {
                const unsigned long long other = tp_xor_lane64(best, 4);
                best = other > best ? other : best;
            }
            if (q == 0) {
                uint32_t bj = (uint32_t)(KP - 1) - ((uint32_t)best & (uint32_t)(KP - 1));
                if (pass == 0 && old != 0xFFu) bj = old;        // seeded vertex keeps its label
                prop[v0 + t - chunk_lo] = (uint8_t)bj;
                if (bj != old) atomicAdd(&tcnt[(t >> 10) * k + (int)bj], 1u);
            }
        }
        __syncthreads();
        const int64_t tile0 = (v0 - chunk_lo) / kAdmitTile;
        const int ntl = nv > kAdmitTile ? 2 : 1;
        for (int j = tid; j < ntl * k; j += kTpThreads) cnt[(size_t)tile0 * k + j] = tcnt[j];
        if (coarse)
            for (int j = tid; j < k; j += kTpThreads) {
                const uint32_t x = tcnt[j] + (ntl > 1 ? tcnt[k + j] : 0u);
                if (x) atomicAdd(&coarse[(size_t)(tile0 / kCoarseTiles) * k + j], x);
            }
        return;
    }

    // any k, 16- or 32-bit estimates: partition j = 4q + z (k % 4 == 0) or q + LPV z of lane q, a (vertex,
    // lane) pair at a time; arg-max by (E desc, room desc, id asc)
#pragma unroll 2
    for (int u = 0; u < BU; ++u) {
        const int g = tid + u * kTpThreads;
        if (g >= nv * LPV) continue;                            // (whole vertices: the lanes of a vertex agree)
        const int t = g / LPV;
        const uint32_t mt = meta[t];
        if (mt & 0x100u) continue;                              // hubs are k_hub_finalize's
        const uint32_t old = mt & 0xFFu;
        const int64_t v = v0 + t;
        ET *Erow = E + (size_t)v * (size_t)k;
        uint32_t ev[4] = {0u, 0u, 0u, 0u};
        if (pass > 0) {
            if (vec) {
                if (4 * q < k) {
                    if (sizeof(ET) == 4) {
                        const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Erow + 4 * q));
                        ev[0] = x.x; ev[1] = x.y; ev[2] = x.z; ev[3] = x.w;
                    } else {
                        const u32x2 x = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(Erow + 4 * q));
                        ev[0] = x.x & 0xFFFFu; ev[1] = x.x >> 16; ev[2] = x.y & 0xFFFFu; ev[3] = x.y >> 16;
                    }
                }
            } else {
#pragma unroll
                for (int z = 0; z < 4; ++z)
                    if (q + LPV * z < k) ev[z] = (uint32_t)Erow[q + LPV * z];
            }
        }
        unsigned long long bestkey = 0;
        int bestj = 0x7fffffff;
#pragma unroll
        for (int z = 0; z < 4; ++z) {
            const int j = vec ? 4 * q + z : q + LPV * z;
            if (j < k) {
                const uint32_t jj = SW ? ((uint32_t)j ^ ((((uint32_t)t >> 3) & 3u) << 2)) : (uint32_t)j;   // (the piece's place)
                const uint32_t cidx = (uint32_t)t * (uint32_t)KP + jj;
                const uint32_t h = (hist[cidx >> 1] >> (16 * (cidx & 1u))) & 0xFFFFu;
                ev[z] += h << sh;
                const uint32_t rm = room[j] + ((uint32_t)j == old ? 1u : 0u);
                const unsigned long long key = rm ? (((unsigned long long)ev[z] << 32) | rm) : 0ull;
                if (key > bestkey) { bestkey = key; bestj = j; }
            }
        }
        if (store_e) {
            if (vec) {
                if (4 * q < k) {
                    if (sizeof(ET) == 4) {
                        u32x4 o;
                        o.x = ev[0]; o.y = ev[1]; o.z = ev[2]; o.w = ev[3];
                        __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(Erow + 4 * q));
                    } else {
                        u32x2 o;
                        o.x = ev[0] | (ev[1] << 16);
                        o.y = ev[2] | (ev[3] << 16);
                        __builtin_nontemporal_store(o, reinterpret_cast<u32x2 *>(Erow + 4 * q));
                    }
                }
            } else {
#pragma unroll
                for (int z = 0; z < 4; ++z)
                    if (q + LPV * z < k) Erow[q + LPV * z] = (ET)ev[z];
            }
        }
        {   // lanes q ^ 1, then q ^ 2, by quad permutes; q ^ 4 through the crossbar
            unsigned long long okey = ((unsigned long long)quad_swap<0xB1>((uint32_t)(bestkey >> 32)) << 32) |
                                      quad_swap<0xB1>((uint32_t)bestkey);
            int oj = (int)quad_swap<0xB1>((uint32_t)bestj);
            if (okey > bestkey || (okey == bestkey && oj < bestj)) { bestkey = okey; bestj = oj; }
            okey = ((unsigned long long)quad_swap<0x4E>((uint32_t)(bestkey >> 32)) << 32) |
                   quad_swap<0x4E>((uint32_t)bestkey);
            oj = (int)quad_swap<0x4E>((uint32_t)bestj);
            if (okey > bestkey || (okey == bestkey && oj < bestj)) { bestkey = okey; bestj = oj; }
            if (LPV > 4) {
                okey = tp_xor_lane64(bestkey, 4);
                oj = __shfl_xor(bestj, 4);
                if (okey > bestkey || (okey == bestkey && oj < bestj)) { bestkey = okey; bestj = oj; }
            }
        }
        if (q == 0) {
            uint32_t best = (uint32_t)bestj;
            if (pass == 0 && old != 0xFFu) best = old;      // seeded vertex keeps its label
            prop[v - chunk_lo] = (uint8_t)best;
            if (best != old) atomicAdd(&tcnt[(t >> 10) * k + (int)best], 1u);
        }
    }
    __syncthreads();
    {
        const int64_t tile0 = (v0 - chunk_lo) / kAdmitTile;
        const int ntl = nv > kAdmitTile ? 2 : 1;
        for (int j = tid; j < ntl * k; j += kTpThreads) cnt[(size_t)tile0 * k + j] = tcnt[j];
        if (coarse)
            for (int j = tid; j < k; j += kTpThreads) {
                const uint32_t x = tcnt[j] + (ntl > 1 ? tcnt[k + j] : 0u);
                if (x) atomicAdd(&coarse[(size_t)(tile0 / kCoarseTiles) * k + j], x);
            }
    }
}

// ------------------------------------------------------------------------------------------------
// hubs of the chunk: counts from the hub table (complete once k_tp_score has finished), blend,
// propose, add the movers to their tiles' counts; the table row is cleared for the next chunk.
// KP lanes per hub, lane j takes partition j (k <= KP).
// Estimates of the hubs: row v of E (n rows) when E is given, else row (ch_hub0[c] + i) of Ehub, the
// table of the hubs alone.
// The last workgroup: tot[t] = an upper bound of the chunk's movers to partition t, for k_apply_small.
// ------------------------------------------------------------------------------------------------
template <int KP>
__global__ __launch_bounds__(256) void k_hub_finalize(SweepPlan pl, const uint8_t *__restrict__ Lc,
                                                      const long long *__restrict__ room,
                                                      uint32_t *__restrict__ E, uint32_t *__restrict__ Ehub,
                                                      uint32_t *__restrict__ Hhub,
                                                      uint8_t *__restrict__ prop, uint32_t *__restrict__ cnt,
                                                      int c, int64_t chunk_lo, int k, int pass, int store_e,
                                                      int ntiles, uint32_t *__restrict__ tot) {
    const uint32_t nh = pl.ch_nh[c];
    if (blockIdx.x == gridDim.x - 1) {
        // the tiles' counts as far as they are complete, plus one for every hub
        __shared__ uint32_t part[256];
        constexpr int SEGS = 256 / KP;                           // threads per column
        const int col = threadIdx.x & (KP - 1), seg = threadIdx.x / KP;
        uint32_t sum = 0;
        if (col < k) {
            for (int r0 = seg; r0 < ntiles; r0 += SEGS * 16) {   // 16 loads side by side
                uint32_t x[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int r = r0 + SEGS * u;
                    x[u] = r < ntiles ? cnt[(size_t)r * k + col] : 0u;
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) sum += x[u];
            }
        }
        part[threadIdx.x] = sum;
        __syncthreads();
        if (threadIdx.x < KP && threadIdx.x < (unsigned)k) {
            uint32_t total = nh;
            for (int q = 0; q < SEGS; ++q) total += part[q * KP + threadIdx.x];
            tot[threadIdx.x] = total;
        }
        return;
    }
    constexpr int kPerBlock = 256 / KP;
    const uint32_t i = blockIdx.x * (uint32_t)kPerBlock + (threadIdx.x / KP);
    const int j = threadIdx.x & (KP - 1);
    const bool on = i < nh;
    const int sh = pass > 0 ? pass - 1 : 0;
    unsigned long long key = 0;
    int bj = 0x7fffffff;
    int64_t v = 0;
    uint32_t old = 0xFFu;
    if (on) {
        const u64 hub = pl.ch_hub0[c] + i;
        v = pl.hub_row[hub];
        old = (uint32_t)Lc[v];
        if (j < k) {
            uint32_t *hp = Hhub + (size_t)i * k + j;
            const uint32_t h = *hp;
            *hp = 0;
            uint32_t *ep = E ? E + (size_t)v * (size_t)k + j : Ehub + (size_t)hub * (size_t)k + j;
            const uint32_t e = (pass > 0 ? *ep : 0u) + (h << sh);
            if (store_e) *ep = e;
            const uint32_t rm = (uint32_t)room[j] + ((uint32_t)j == old ? 1u : 0u);
            key = rm ? (((unsigned long long)e << 32) | rm) : 0ull;
            bj = j;
        }
    }
#pragma unroll
    for (int off = 1; off <= KP / 2; off <<= 1) {      // every lane of the wavefront takes part
        const unsigned long long okey = __shfl_xor(key, off);
        const int oj = __shfl_xor(bj, off);
        if (okey > key || (okey == key && oj < bj)) { key = okey; bj = oj; }
    }
    if (on && j == 0) {
        uint32_t best = (uint32_t)bj;
        if (pass == 0 && old != 0xFFu) best = old;
        prop[v - chunk_lo] = (uint8_t)best;
        if (best != old) atomicAdd(&cnt[(size_t)((v - chunk_lo) / kAdmitTile) * k + best], 1u);   // after k_tp_score's store
    }
}

// ------------------------------------------------------------------------------------------------
// Admission of a chunk with the hubs' part folded in, for chunks of few hubs and few tiles: what
// k_hub_finalize and k_apply_small do in two launches.  Every workgroup works the chunk's hubs out for
// itself (blend, proposal: nh * KP lanes of work), so nothing has to pass between workgroups:
//   - the hubs' labels come from hub_old (k_tp_score leaves them there, by place in the chunk's list);
//   - the hubs' counts are read from Hnow and left alone (the host alternates between two tables
//     from chunk to chunk; workgroup 0 clears the rows the chunk before used in the other one);
//   - their estimates are read from Eold and written to Enew (two tables of the hubs' rows, alternating
//     from pass to pass) by the one workgroup whose tiles hold the hub;
//   - a hub's proposal reaches the thread of its vertex through LDS (`over`); its move counts for the
//     tiles' mover counts exactly as the atomic add of k_hub_finalize did;
//   - every workgroup adds up all tiles' counts itself: the chunk's movers per partition (exact, where
//     k_apply_small gets an upper bound) and those of the tiles before its own -- from the coarse table
//     k_tp_score leaves (Cnow; two tables take turns from chunk to chunk, workgroup 0 clears the other one,
//     Cclear) and the rows of the tiles of its own coarse group.
// cnt[tile][t]: movers to t among the tile's regular rows (from k_tp_score).
// ------------------------------------------------------------------------------------------------
constexpr int kAdmitHubsMax = 512;        // hubs of a chunk
constexpr int kAdmitTilesMax = 1024;      // tiles of a chunk

template <int KP>
__global__ __launch_bounds__(kAdmitTile) void k_admit_hubs(
    uint8_t *__restrict__ Lc, const uint8_t *__restrict__ prop, int64_t chunk_lo, int64_t chunk_hi, int k,
    const uint32_t *__restrict__ cnt, int ntiles, const long long *__restrict__ room,
    unsigned long long *__restrict__ S, uint32_t *__restrict__ ocnt, int pass, uint8_t *__restrict__ Lc4,
    const int32_t *__restrict__ hub_row, const uint8_t *__restrict__ hub_old, uint32_t nh,
    const uint32_t *__restrict__ Hnow,
    uint32_t *__restrict__ Hclear, uint32_t nclear, const uint32_t *__restrict__ Eold,
    uint32_t *__restrict__ Enew, int store_e, const uint32_t *__restrict__ Cnow, uint32_t *__restrict__ Cclear) {
    static_assert(KP == 16 || KP == 32, "partitions per workgroup table");
    constexpr int nwaves = kAdmitTile / 64;
    constexpr int TPW = kSmallApplyTiles;
    constexpr int SEGS = kAdmitTile / KP;           // threads per column of cnt
    constexpr int HPR = kAdmitTile / KP;            // hubs per round of the workgroup
    constexpr int HB = 4;                           // rounds whose loads are issued side by side
    __shared__ uint32_t tbl[KP];                    // movers in the tiles before the workgroup's
    __shared__ uint32_t totl[KP];                   // movers in the whole chunk
    __shared__ uint32_t ownh[TPW][KP];              // hubs among the movers of the workgroup's tiles
    __shared__ uint32_t wcnt[TPW][nwaves][KP];      // movers per tile and wave, then their exclusive prefix
    __shared__ int32_t dS[KP];
    __shared__ long long s_room[KP];
    __shared__ uint32_t s_unassigned[TPW];
    __shared__ __align__(16) uint8_t over[TPW * kAdmitTile];   // a hub's proposal, for the thread of its vertex (0xFF: none)
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
    // all tiles' counts, column `col` by SEGS threads
    const int col = tid & (KP - 1), seg = tid / KP;
    uint32_t all = 0, before = 0;
    if (col < k && Cnow) {
        // the coarse rows (kCoarseTiles tiles each) for the whole chunk and the groups before the workgroup's,
        // the tiles' own rows only inside its group: (tiles / 32 + 32) * k counts instead of tiles * k
        const int g0 = tile0 / kCoarseTiles, ng = (ntiles + kCoarseTiles - 1) / kCoarseTiles;
        for (int r0 = seg; r0 < ng + kCoarseTiles; r0 += SEGS) {
            uint32_t x = 0;
            if (r0 < ng) {
                x = Cnow[(size_t)r0 * k + col];
                all += x;
                if (r0 < g0) before += x;
            } else {
                const int r = g0 * kCoarseTiles + (r0 - ng);
                if (r < tile0 && r < ntiles) before += cnt[(size_t)r * k + col];
            }
        }
    } else if (col < k) {
        for (int r0 = seg; r0 < ntiles; r0 += SEGS * 16) {      // (16 loads side by side: one turn when KP = 16)
            uint32_t x[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int r = r0 + SEGS * u;
                x[u] = r < ntiles ? cnt[(size_t)r * k + col] : 0u;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                all += x[u];
                if (r0 + SEGS * u < tile0) before += x[u];
            }
        }
    }
    uint32_t own[TPW];
#pragma unroll
    for (int h = 0; h < TPW; ++h)
        own[h] = (tid < k && tile0 + h < ntiles) ? cnt[(size_t)(tile0 + h) * k + tid] : 0u;
    long long rm0 = 0;
    if (tid < k) rm0 = room[tid];
    // the hubs this thread takes part in, HB rounds at a time: KP lanes per hub, lane j takes partition j;
    // the first rounds' loads are on their way with everything above
    const int j = col;
    int64_t hv[HB];
    uint32_t hold[HB], hh[HB], he[HB];
    auto load_hubs = [&](uint32_t i0) {
#pragma unroll
        for (int u = 0; u < HB; ++u) {
            const uint32_t i = i0 + (uint32_t)u * HPR;
            hv[u] = i < nh ? (int64_t)hub_row[i] : chunk_lo;
            hold[u] = i < nh ? (uint32_t)hub_old[i] : 0xFFu;     // (left by k_tp_score: no trip through the list)
            hh[u] = (i < nh && j < k) ? Hnow[(size_t)i * k + j] : 0u;
            he[u] = (i < nh && j < k && pass > 0) ? Eold[(size_t)i * k + j] : 0u;
        }
    };
    load_hubs((uint32_t)seg);
    if (tid < KP) {
        tbl[tid] = 0; totl[tid] = 0; dS[tid] = 0; s_room[tid] = rm0;
#pragma unroll
        for (int h = 0; h < TPW; ++h) ownh[h][tid] = 0;
    }
    if (tid < TPW) s_unassigned[tid] = 0;
    reinterpret_cast<uint32_t *>(over)[tid] = 0xFFFFFFFFu;
    if (blockIdx.x == 0) {
        for (uint32_t q = tid; q < nclear * (uint32_t)k; q += kAdmitTile) Hclear[q] = 0;
        if (Cclear)
            for (int q = tid; q < (kAdmitTilesMax / kCoarseTiles) * k; q += kAdmitTile) Cclear[q] = 0;
    }
    __syncthreads();
    if (all) atomicAdd(&totl[col], all);
    if (before) atomicAdd(&tbl[col], before);
    // the chunk's hubs
    {
        const int sh = pass > 0 ? pass - 1 : 0;
        for (uint32_t i0 = (uint32_t)seg; i0 < nh; i0 += HPR * HB) {
            if (i0 != (uint32_t)seg) load_hubs(i0);
#pragma unroll
            for (int u = 0; u < HB; ++u) {
                const uint32_t i = i0 + (uint32_t)u * HPR;
                const bool on = i < nh;                      // (uniform over the KP lanes of a hub)
                unsigned long long key = 0;
                int bj = 0x7fffffff;
                const uint32_t e = he[u] + (hh[u] << sh);
                if (on && j < k) {
                    const uint32_t rm = (uint32_t)s_room[j] + ((uint32_t)j == hold[u] ? 1u : 0u);
                    key = rm ? (((unsigned long long)e << 32) | rm) : 0ull;
                    bj = j;
                }
#pragma unroll
                for (int off = 1; off <= KP / 2; off <<= 1) {      // the KP lanes of a hub are on or off together
                    const unsigned long long okey = __shfl_xor(key, off);
                    const int oj = __shfl_xor(bj, off);
                    if (okey > key || (okey == key && oj < bj)) { key = okey; bj = oj; }
                }
                if (!on) continue;
                const int tile = (int)((hv[u] - chunk_lo) / kAdmitTile);
                const bool mine = tile >= tile0 && tile < tile0 + TPW;
                if (mine && store_e && j < k) Enew[(size_t)i * k + j] = e;
                if (j == 0) {
                    uint32_t best = (uint32_t)bj;
                    if (pass == 0 && hold[u] != 0xFFu) best = hold[u];      // a seeded vertex keeps its label
                    if (best != hold[u]) {
                        atomicAdd(&totl[best], 1u);
                        if (tile < tile0) atomicAdd(&tbl[best], 1u);
                        else if (mine) atomicAdd(&ownh[tile - tile0][best], 1u);
                    }
                    if (mine) over[(tile - tile0) * kAdmitTile + (int)((hv[u] - chunk_lo) % kAdmitTile)] = (uint8_t)best;
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < TPW; ++h) {
        const uint32_t o = over[h * kAdmitTile + tid];
        if (o != 0xFFu) t[h] = o;
        own[h] += tid < KP ? ownh[h][tid] : 0u;
    }
    // bit t: partition t has room for some of its movers only (every wavefront works it out for itself)
    uint32_t ranked;
    {
        const long long rl = lane < k ? s_room[lane] : 0;
        const bool some = lane < k && rl > 0 && (long long)totl[lane] > rl;
        ranked = (uint32_t)__ballot(some);
    }
    bool mover[TPW];
    uint32_t wrank[TPW];
#pragma unroll
    for (int h = 0; h < TPW; ++h) { mover[h] = inside[h] && t[h] != old[h]; wrank[h] = 0; }
    if (ranked) {
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
            for (int h = 0; h < TPW; ++h) ownh[h][tid] = own[h];    // (regular rows and hubs together now)
        __syncthreads();
        wave_counts_to_prefix<KP, TPW>(wcnt, ownh);
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
    if (pass == 0 && tid < TPW && tile0 + tid < ntiles) ocnt[tile0 + tid] = s_unassigned[tid];
}

// ------------------------------------------------------------------------------------------------
// 16-bit estimates of the regular rows -> the caller's 32-bit array (hub rows are already there)
// ------------------------------------------------------------------------------------------------
template <typename RowT>
__global__ __launch_bounds__(256) void k_expand_estimates(const RowT *__restrict__ rowptr, int64_t n, int k,
                                                          uint32_t hub_degree, const uint16_t *__restrict__ E16,
                                                          uint32_t *__restrict__ out) {
    const int64_t total = n * (int64_t)k;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const int64_t v = idx / k;
        if ((u64)(rowptr[v + 1] - rowptr[v]) < hub_degree) out[idx] = E16[idx];
    }
}

}  // namespace grem
